"""Pins for the oracle's modified rejection step and its host loops.

Section 3 states the property everything here rests on: speculative sampling recovers the target
distribution, so its output has the same law as autoregressive sampling from the target.  The
tests pin the implemented procedure to that law (exact enumeration, chi-square on a tiny
vocabulary), to closed forms, to brute force, and to the greedy special case where the two loops
must agree token for token.
"""
from fractions import Fraction

import numpy as np
import pytest
import scipy.stats

import oracle
import seeded_inputs as si


def _rand_dist(rng, V, zeros=0):
    x = rng.gamma(0.7, size=V)
    if zeros:
        x[rng.choice(V, zeros, replace=False)] = 0.0
    return (x / x.sum()).astype(np.float32)


# ---------------------------------------------------------------- the law itself (no code under test)

def test_accept_plus_residual_law_is_the_target_exactly():
    """P(out = v) = min(p_v, q_v) + (1 - sum_x min(p_x, q_x)) * max(0, p_v - q_v) / sum_x max(0, p_x - q_x)
    equals p_v: checked in exact rational arithmetic, so the rule the oracle implements is the right one."""
    rng = np.random.default_rng(0)
    for _ in range(50):
        V = int(rng.integers(2, 9))
        p = [Fraction(int(a), 1) for a in rng.integers(0, 20, V)]
        q = [Fraction(int(a), 1) for a in rng.integers(1, 20, V)]
        if sum(p) == 0:
            p[0] = Fraction(1)
        p = [a / sum(p) for a in p]
        q = [a / sum(q) for a in q]
        res = [max(Fraction(0), a - b) for a, b in zip(p, q)]
        rej = 1 - sum(min(a, b) for a, b in zip(p, q))
        for v in range(V):
            out = q[v] * min(Fraction(1), p[v] / q[v]) + (rej * res[v] / sum(res) if sum(res) else 0)
            assert out == p[v]


# ---------------------------------------------------------------- Bernoulli realisation

def test_accept_rule_edges_and_rate():
    assert oracle.accept(0.999, 0.3, 0.3)              # p >= q always accepts
    assert oracle.accept(0.999, 0.5, 0.0)              # q = 0 accepts
    assert oracle.accept(0.0, 0.0, 0.0)
    assert not oracle.accept(0.0, 0.0, 0.5)            # p = 0 < q never accepts (0 < 0 is false)
    assert oracle.accept(0.0, 1e-30, 0.5)              # u = 0 accepts whenever p > 0
    assert oracle.accept(0.25, 0.26, 1.0) and not oracle.accept(0.25, 0.25, 1.0)  # strict u*q < p
    # acceptance frequency over the whole 2^-12 grid of uniforms equals ceil(p/q * 4096)/4096
    p, q = np.float32(0.3), np.float32(0.7)
    n = sum(oracle.accept(m / 4096.0, p, q) for m in range(4096))
    assert abs(n / 4096.0 - float(p) / float(q)) <= 1.0 / 4096


# ---------------------------------------------------------------- integer inverse CDF vs brute force

def test_sample_matches_exact_rational_inverse_cdf():
    """On a tiny vocabulary every uniform near a bin edge is checked against exact arithmetic:
    weights w_v = floor(p_v 2^32), the token is the first v whose inclusive prefix exceeds
    floor(m S / 2^24)."""
    rng = np.random.default_rng(1)
    for trial in range(20):
        V = int(rng.integers(2, 17))
        p = _rand_dist(rng, V, zeros=int(rng.integers(0, V // 2 + 1)) if V > 2 else 0)
        w = [int(Fraction(float(x)) * 2 ** 32) for x in p]          # exact floor
        S = sum(w)
        pref = np.cumsum(w)
        edges = [Fraction(int(c), S) for c in pref[:-1]]
        ms = {0, 2 ** 24 - 1}
        for e in edges:                                             # uniforms straddling each edge
            m0 = int(e * 2 ** 24)
            ms.update(m for m in (m0 - 1, m0, m0 + 1) if 0 <= m < 2 ** 24)
        ms.update(int(m) for m in rng.integers(0, 2 ** 24, 50))
        for m in ms:
            T = (m * S) >> 24
            expect = next(v for v in range(V) if pref[v] > T)
            assert oracle.sample(p, m / 2.0 ** 24) == expect
            assert p[expect] > 0                                    # never a zero-probability token


def test_residual_sampling_matches_exact_rational_inverse_cdf():
    rng = np.random.default_rng(2)
    for trial in range(20):
        V = int(rng.integers(2, 17))
        p, q = _rand_dist(rng, V), _rand_dist(rng, V)
        r = np.maximum(np.float32(0), p - q)                        # one fp32 subtract per entry
        w = [int(Fraction(float(x)) * 2 ** 32) for x in r]
        S, pref = sum(w), np.cumsum(w)
        for m in [0, 2 ** 24 - 1] + [int(x) for x in rng.integers(0, 2 ** 24, 200)]:
            T = (m * S) >> 24
            expect = next(v for v in range(V) if pref[v] > T)
            got = oracle.sample_residual(p, q, m / 2.0 ** 24)
            assert got == expect and p[got] > q[got]


def test_degenerate_residual_falls_back_to_target_then_argmax():
    p = np.float32([0.25, 0.5, 0.25])
    assert oracle.sample_residual(p, p, 0.6) == oracle.sample(p, 0.6) == 1     # residual all zero
    tiny = np.float32([1e-12, 3e-12, 2e-12])                                   # every weight quantises to 0
    assert oracle.sample(tiny, 0.9) == 1 and oracle.sample_residual(tiny, tiny, 0.1) == 1


# ---------------------------------------------------------------- batch step: special cases

def test_speculative_accept_special_cases():
    rng = np.random.default_rng(3)
    B, K, V = 6, 4, 11
    p = np.stack([[_rand_dist(rng, V) for _ in range(K + 1)] for _ in range(B)])
    u = si.uniforms(3, "u", (B, K + 1)).numpy()
    draft = rng.integers(0, V, (B, K)).astype(np.int32)
    # q = p: everything accepted, bonus token ~ p_{K+1} with the last uniform
    na, nx = oracle.speculative_accept(p, p[:, :K].copy(), draft, u)
    assert np.all(na == K)
    assert all(nx[b] == oracle.sample(p[b, K], u[b, K]) for b in range(B))
    # disjoint supports: q lives where p is zero -> a = 0 and next ~ p_1 (residual = p_1)
    q = np.zeros((B, K, V), np.float32)
    pd = p.copy()
    pd[:, :, :3] = 0
    pd /= pd.sum(-1, keepdims=True)
    q[:, :, :3] = np.float32(1.0 / 3)
    d0 = rng.integers(0, 3, (B, K)).astype(np.int32)
    na, nx = oracle.speculative_accept(pd, q, d0, u)
    assert np.all(na == 0)
    for b in range(B):
        assert nx[b] == oracle.sample_residual(pd[b, 0], q[b, 0], u[b, K]) and nx[b] >= 3
    # K = 0: a plain sample from p
    na, nx = oracle.speculative_accept(p[:, :1], np.zeros((B, 0, V), np.float32),
                                       np.zeros((B, 0), np.int32), u[:, :1])
    assert np.all(na == 0) and all(nx[b] == oracle.sample(p[b, 0], u[b, 0]) for b in range(B))
    # first rejection stops the scan: later uniforms/tokens do not matter
    q2 = np.stack([[_rand_dist(rng, V) for _ in range(K)] for _ in range(B)])
    na1, nx1 = oracle.speculative_accept(p, q2, draft, u)
    for b in range(B):
        a = na1[b]
        if a < K:
            draft2, u2 = draft.copy(), u.copy()
            draft2[b, a + 1:] = (draft2[b, a + 1:] + 1) % V
            u2[b, a + 1:K] = 0.0
            na2, nx2 = oracle.speculative_accept(p, q2, draft2, u2)
            assert na2[b] == a and nx2[b] == nx1[b]
    with pytest.raises(ValueError):
        oracle.speculative_accept(p, q2, np.full((B, K), V, np.int32), u)


def test_one_hot_distributions_reduce_to_the_greedy_rule():
    rng = np.random.default_rng(4)
    B, K, V = 8, 5, 13
    logits = rng.normal(size=(B, K + 1, V)).astype(np.float32)
    logits[0, 2, 4] = logits[0, 2].max() + 1
    logits[0, 2, 9] = logits[0, 2, 4]                       # a tie: lowest index wins
    tgt = logits.argmax(-1)
    draft = tgt[:, :K].astype(np.int32).copy()
    for b in range(B):                                      # plant the first mismatch at position b % (K+1)
        if b % (K + 1) < K:
            draft[b, b % (K + 1)] = (draft[b, b % (K + 1)] + 1) % V
    na, nx = oracle.greedy_accept(logits, draft)
    assert list(na) == [b % (K + 1) for b in range(B)]
    assert all(nx[b] == tgt[b, na[b]] for b in range(B))
    assert oracle.argmax(logits[0, 2]) == 4
    # the same answer from the probabilistic rule fed one-hot p and q
    p = np.eye(V, dtype=np.float32)[tgt]
    q = np.eye(V, dtype=np.float32)[draft]
    u = si.uniforms(4, "u", (B, K + 1)).numpy()
    na2, nx2 = oracle.speculative_accept(p, q, draft, u)
    assert np.array_equal(na, na2) and np.array_equal(nx, nx2)


# ---------------------------------------------------------------- chi-square on a tiny vocabulary

def test_single_step_output_distribution_is_the_target():
    """Brute force: draw d ~ q, run the implemented accept / residual-resample step a million
    times with seeded uniforms; the histogram of the emitted token follows p and the acceptance
    frequency is 1 - ||p - q||_1 / 2."""
    rng = np.random.default_rng(5)
    V, N = 8, 1_000_000
    p, q = _rand_dist(rng, V), _rand_dist(rng, V, zeros=1)
    ud = si.uniforms(5, "ud", (N,)).numpy()
    # draft tokens through the oracle's own sampler (its law is pinned above by exact arithmetic)
    cdf_edges = np.cumsum([int(Fraction(float(x)) * 2 ** 32) for x in q])
    thr = (np.round(ud * 2 ** 24).astype(np.uint64) * np.uint64(cdf_edges[-1])) >> np.uint64(24)
    d = np.searchsorted(cdf_edges, thr, side="right").astype(np.int32)
    assert all(d[i] == oracle.sample(q, ud[i]) for i in range(0, N, N // 200))
    pp = np.broadcast_to(np.stack([p, p])[None], (N, 2, V)).copy()
    qq = np.broadcast_to(q[None, None], (N, 1, V)).copy()
    u = si.uniforms(5, "u", (N, 2)).numpy()
    na, nx = oracle.speculative_accept(pp, qq, d[:, None], u)
    out = np.where(na == 1, d, nx)
    hist = np.bincount(out, minlength=V)
    pd = p.astype(np.float64) / p.astype(np.float64).sum()
    chi = scipy.stats.chisquare(hist, pd * N)
    assert chi.pvalue > 1e-4, (hist, pd * N)
    rate = 1.0 - 0.5 * np.abs(p.astype(np.float64) - q.astype(np.float64)).sum()
    assert abs(na.mean() - rate) < 4 * np.sqrt(rate * (1 - rate) / N)
    # sanity of the test itself: against a wrong law (q) the same histogram is rejected
    assert scipy.stats.chisquare(hist, q.astype(np.float64) / q.sum() * N + 1e-9).pvalue < 1e-12


def test_chain_of_three_recovers_the_target_joint():
    """K = 3 with context-dependent (first-order Markov) toy models: the joint law of the first two
    emitted tokens equals the target's p(t1 | x0) p(t2 | t1)."""
    rng = np.random.default_rng(6)
    V, K, N = 4, 3, 400_000
    P = np.stack([_rand_dist(rng, V) for _ in range(V)])      # target p(. | prev)
    Q = np.stack([_rand_dist(rng, V) for _ in range(V)])      # draft q(. | prev)
    Qcdf = np.cumsum(Q.astype(np.float64), axis=1)

    def step(prev, tag):
        ud = si.uniforms(6, "ud" + tag, (N, K)).numpy()
        u = si.uniforms(6, "u" + tag, (N, K + 1)).numpy()
        d = np.zeros((N, K), np.int32)
        ctx = prev.copy()
        for i in range(K):                                    # d_i ~ q(. | previous token)
            d[:, i] = np.minimum((ud[:, i, None] * Qcdf[ctx, -1:] >= Qcdf[ctx]).sum(1), V - 1)
            ctx = d[:, i]
        rows = np.concatenate([prev[:, None], d], axis=1)     # contexts of the K+1 target rows
        na, nx = oracle.speculative_accept(P[rows], Q[rows[:, :K]], d, u)
        return d, na, nx

    x0 = np.zeros(N, np.int32)
    d, na, nx = step(x0, "a")
    t1 = np.where(na >= 1, d[:, 0], nx)
    t2 = np.where(na >= 2, d[:, 1], nx)                       # valid where na >= 1
    need = na == 0                                            # only one token emitted: run another step
    d2, na2, nx2 = step(t1, "b")
    t2 = np.where(need, np.where(na2 >= 1, d2[:, 0], nx2), t2)
    hist = np.bincount(t1 * V + t2, minlength=V * V).astype(np.float64)
    Pd = P.astype(np.float64) / P.astype(np.float64).sum(1, keepdims=True)
    joint = (Pd[0][:, None] * Pd).reshape(-1)
    assert scipy.stats.chisquare(hist, joint * N).pvalue > 1e-4


# ---------------------------------------------------------------- the loops: greedy equivalence

@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("K", [1, 2, 4, 8])
def test_greedy_speculative_equals_greedy_autoregressive(seed, K):
    """With argmax selection the speculative loop (two caches, truncation, the two-token draft
    catch-up after a fully accepted step) must emit exactly the autoregressive tokens."""
    tw = si.decoder_weights(si.TINY_TARGET, seed)
    dw = si.decoder_weights(si.TINY_DRAFT, seed + 100)
    if seed == 2:   # a draft that agrees with the target often: the target's own first layer
        dshape, dw = si.early_exit_draft(si.TINY_TARGET, tw, 1)
    else:
        dshape = si.TINY_DRAFT
    target, draft = oracle.Model(si.TINY_TARGET, tw), oracle.Model(dshape, dw)
    prompt = si.token_ids(seed, "prompt", (32,), 1024).numpy()
    n_new = 64 if (seed == 0 and K == 4) else 24
    ar = oracle.autoregressive_generate(target, prompt, n_new, 0.0)
    sp, stats = oracle.speculative_generate(target, draft, prompt, n_new, K, 0.0)
    assert sp == ar
    assert len(stats["accepted"]) == stats["steps"] and all(0 <= a <= K for a in stats["accepted"])


def test_full_acceptance_exercises_the_two_token_catch_up():
    """Draft == target: every draft token is accepted (a = K each step), so every step after the
    first goes through the two-token draft call; the output still equals autoregressive greedy."""
    tw = si.decoder_weights(si.TINY_TARGET, 7)
    target = oracle.Model(si.TINY_TARGET, tw)
    prompt = si.token_ids(7, "prompt", (8,), 1024).numpy()
    ar = oracle.autoregressive_generate(target, prompt, 20, 0.0)
    sp, stats = oracle.speculative_generate(target, target, prompt, 20, 3, 0.0)
    assert sp == ar and all(a == 3 for a in stats["accepted"])


def test_sampled_speculative_with_identical_models_equals_sampling_from_the_target():
    """Draft == target at temperature 1: p = q, so every token is accepted and the emitted stream
    is d_1..d_K (drawn from q = p with the draft uniforms) then the bonus drawn with the accept
    uniform - i.e. autoregressive sampling from the target with that interleaved uniform stream."""
    tw = si.decoder_weights(si.TINY_TARGET, 8)
    target = oracle.Model(si.TINY_TARGET, tw)
    prompt = si.token_ids(8, "prompt", (8,), 1024).numpy()
    K, n_new = 3, 16
    steps = n_new // (K + 1)
    ud = si.uniforms(8, "ud", (steps, K)).numpy()
    ua = si.uniforms(8, "ua", (steps, K + 1)).numpy()
    sp, stats = oracle.speculative_generate(target, target, prompt, n_new, K, 1.0, ud, ua)
    assert all(a == K for a in stats["accepted"])
    u_ar = np.concatenate([np.concatenate([ud[s], ua[s, K:]]) for s in range(steps)])
    assert sp == oracle.autoregressive_generate(target, prompt, n_new, 1.0, u_ar)


@pytest.mark.parametrize("K,temperature", [(1, 0.0), (4, 0.0), (3, 1.0), (8, 1.0)])
def test_shared_cache_for_an_early_exit_draft_changes_nothing(K, temperature):
    """Section 4.4 asks whether two separate caches are needed.  For a draft made of the target's first
    layers they are not: the draft can work in the leading layers of the target's cache (its rows are
    rewritten by the verify call).  The keys and values it would have kept in a cache of its own are
    the same numbers, so the token stream and the accept counts are identical to the two-cache loop -
    and the greedy stream still equals autoregressive greedy decoding."""
    tw = si.decoder_weights(si.TINY_TARGET, 11)
    dshape, dw = si.early_exit_draft(si.TINY_TARGET, tw, 1)
    target, draft = oracle.Model(si.TINY_TARGET, tw), oracle.Model(dshape, dw)
    prompt = si.token_ids(11, "prompt", (20,), 1024).numpy()
    n_new = 30
    ud = si.uniforms(11, "ud", (n_new, K)).numpy()
    ua = si.uniforms(11, "ua", (n_new, K + 1)).numpy()
    two, st2 = oracle.speculative_generate(target, draft, prompt, n_new, K, temperature, ud, ua)
    one, st1 = oracle.speculative_generate(target, draft, prompt, n_new, K, temperature, ud, ua, shared_kv=True)
    assert one == two and st1["accepted"] == st2["accepted"]
    if temperature == 0.0:
        assert one == oracle.autoregressive_generate(target, prompt, n_new, 0.0)


def test_shared_cache_with_the_target_as_its_own_draft_accepts_everything():
    """Draft == target on one cache: every step accepts all K tokens, and no two-token catch-up exists."""
    tw = si.decoder_weights(si.TINY_TARGET, 12)
    target = oracle.Model(si.TINY_TARGET, tw)
    prompt = si.token_ids(12, "prompt", (8,), 1024).numpy()
    sp, stats = oracle.speculative_generate(target, target, prompt, 20, 3, 0.0, shared_kv=True)
    assert sp == oracle.autoregressive_generate(target, prompt, 20, 0.0) and all(a == 3 for a in stats["accepted"])
