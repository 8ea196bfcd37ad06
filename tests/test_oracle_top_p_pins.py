"""Pins of the oracle's top-p filter (Section 3 names sampling from the top-p set as a token selection
rule; the arithmetic is this build's reading: integer weights, ties by index, fp32 renormalisation).
Brute force over all subsets on tiny rows, hand-made cases with exact arithmetic, the defining properties
on random rows, and the distribution the rejection step emits when both models are filtered."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import scipy.stats

import oracle
import seeded_inputs as si


def _w(p):
    return [min(int(Fraction(float(x)) * 2 ** 32), 2 ** 32 - 1) if x > 0 else 0 for x in p]


def _target(w, top_p):
    P24 = min(max(int(round(float(np.float32(top_p)) * 2 ** 24)), 1), 2 ** 24)
    return max(1, -(-(P24 * sum(w)) // 2 ** 24))


def test_hand_made_rows():
    p = np.array([0.5, 0.25, 0.125, 0.125], dtype=np.float32)            # exact binary fractions
    assert np.array_equal(oracle.top_p_filter(p, 0.5), np.array([1, 0, 0, 0], dtype=np.float32))
    assert np.array_equal(oracle.top_p_filter(p, 0.75), np.array([2 / 3, 1 / 3, 0, 0], dtype=np.float32))
    # 0.8 needs a third token: the tie between tokens 2 and 3 goes to the lower index
    np.testing.assert_array_equal(oracle.top_p_filter(p, 0.8), (p / np.float32(0.875)) * np.array([1, 1, 1, 0], dtype=np.float32))
    # just above what two tokens hold -> three; exactly what two hold -> two
    assert np.count_nonzero(oracle.top_p_filter(p, 0.75 + 2 ** -20)) == 3
    # the order of the row does not matter, only weights and indices
    perm = np.array([0.125, 0.5, 0.125, 0.25], dtype=np.float32)
    assert np.array_equal(oracle.top_p_filter(perm, 0.8) > 0, np.array([True, True, False, True]))
    # top_p = 1 (and above) is the identity; a tiny top_p keeps the argmax only (lowest index on ties)
    assert np.array_equal(oracle.top_p_filter(p, 1.0), p)
    assert np.array_equal(oracle.top_p_filter(np.array([0.25, 0.25, 0.25, 0.25], dtype=np.float32), 1e-9), np.array([1, 0, 0, 0], dtype=np.float32))
    # rows are independent
    both = oracle.top_p_filter(np.stack([p, perm]), 0.8)
    assert np.array_equal(both[0], oracle.top_p_filter(p, 0.8)) and np.array_equal(both[1], oracle.top_p_filter(perm, 0.8))


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_smallest_heaviest_set_on_tiny_rows(seed):
    """V = 7: among all subsets whose integer weight reaches the target, the kept set is one of minimum
    size, and among those of maximum weight; with ties broken towards low indices it is unique."""
    rng = np.random.default_rng(seed)
    V = 7
    p = rng.random(V).astype(np.float32)
    if seed % 2:
        p[rng.integers(0, V, 3)] = p[0]            # ties
    p = (p / p.sum()).astype(np.float32)
    w = _w(p)
    for top_p in (0.1, 0.35, 0.5, 0.77, 0.9, 0.999):
        T = _target(w, top_p)
        best = None
        for k in range(1, V + 1):
            cands = [c for c in itertools.combinations(range(V), k) if sum(w[i] for i in c) >= T]
            if cands:
                top = max(sum(w[i] for i in c) for c in cands)
                best = min(c for c in cands if sum(w[i] for i in c) == top)   # lexicographically lowest indices
                break
        got = oracle.top_p_filter(p, top_p)
        assert tuple(np.nonzero(got)[0]) == best
        Z = np.float32(float(np.float32(sum(w[i] for i in best))) * 2.0 ** -32)
        np.testing.assert_array_equal(got[list(best)], (p[list(best)] / Z).astype(np.float32))


def test_defining_properties_on_random_rows():
    rows = oracle.softmax(si.normal(9, "tp", (12, 1000), 2.0).numpy(), 1.0)
    for top_p in (0.2, 0.5, 0.9, 0.99):
        f = oracle.top_p_filter(rows, top_p)
        for r in range(rows.shape[0]):
            keep = f[r] > 0
            mass = rows[r][keep].astype(np.float64).sum()
            assert mass >= top_p * rows[r].astype(np.float64).sum() - 1e-6            # enough mass
            assert rows[r][keep].min() >= rows[r][~keep].max()                          # the most probable ones
            assert mass - rows[r][keep].min() < top_p * rows[r].astype(np.float64).sum() + 1e-6   # none to spare
            np.testing.assert_allclose(f[r].astype(np.float64).sum(), 1.0, rtol=1e-5)   # renormalised
            np.testing.assert_allclose(f[r][keep], rows[r][keep] / mass, rtol=1e-5)     # proportions kept
        # a larger top_p keeps a superset
        assert np.all((oracle.top_p_filter(rows, 0.5) > 0) <= (f > 0)) or top_p < 0.5


def test_filtered_speculative_step_emits_the_filtered_target():
    """Both rows filtered with the same top_p, then the rejection step: the emitted token follows the
    filtered target row (chi-square, 400 000 trials) and never leaves its nucleus."""
    rng = np.random.default_rng(3)
    V, N, top_p = 10, 400_000, 0.7
    p = rng.random(V).astype(np.float32); p = (p / p.sum()).astype(np.float32)
    q = rng.random(V).astype(np.float32); q = (q / q.sum()).astype(np.float32)
    pf, qf = oracle.top_p_filter(p, top_p), oracle.top_p_filter(q, top_p)
    assert 1 < np.count_nonzero(pf) < V and 1 < np.count_nonzero(qf) < V
    ud = si.uniforms(3, "ud", (N,)).numpy()
    edges = np.cumsum(_w(qf))
    thr = (np.round(ud * 2 ** 24).astype(np.uint64) * np.uint64(edges[-1])) >> np.uint64(24)
    d = np.searchsorted(edges, thr, side="right").astype(np.int32)
    assert all(d[i] == oracle.sample(qf, ud[i]) for i in range(0, N, N // 100))
    pp = np.broadcast_to(np.stack([pf, pf])[None], (N, 2, V)).copy()
    qq = np.broadcast_to(qf[None, None], (N, 1, V)).copy()
    na, nx = oracle.speculative_accept(pp, qq, d[:, None], si.uniforms(3, "u", (N, 2)).numpy())
    out = np.where(na == 1, d, nx)
    hist = np.bincount(out, minlength=V)
    assert np.all(hist[pf == 0] == 0)
    keep = pf > 0
    pd = pf[keep].astype(np.float64) / pf.astype(np.float64).sum()
    assert scipy.stats.chisquare(hist[keep], pd * N).pvalue > 1e-4
    # the unfiltered target is rejected as the law of the same histogram
    pu = p.astype(np.float64)
    assert scipy.stats.chisquare(hist, pu / pu.sum() * N).pvalue < 1e-12


def test_loops_with_top_p():
    """Identical models: everything is accepted and the stream is autoregressive top-p sampling with the
    interleaved uniforms; top_p = 1 is the unfiltered loop; every emitted token lies in the nucleus of
    the target's row at its position."""
    tw = si.decoder_weights(si.TINY_TARGET, 8)
    target = oracle.Model(si.TINY_TARGET, tw)
    draft = oracle.Model(si.TINY_DRAFT, si.decoder_weights(si.TINY_DRAFT, 108))
    prompt = si.token_ids(8, "prompt", (8,), 1024).numpy()
    K, n_new, top_p = 3, 16, 0.6
    steps = n_new // (K + 1)
    ud, ua = si.uniforms(8, "ud", (n_new, K)).numpy(), si.uniforms(8, "ua", (n_new, K + 1)).numpy()
    sp, stats = oracle.speculative_generate(target, target, prompt, n_new, K, 1.0, ud, ua, top_p=top_p)
    assert all(a == K for a in stats["accepted"])
    u_ar = np.concatenate([np.concatenate([ud[s], ua[s, K:]]) for s in range(steps)])
    assert sp == oracle.autoregressive_generate(target, prompt, n_new, 1.0, u_ar, top_p=top_p)
    assert sp != oracle.autoregressive_generate(target, prompt, n_new, 1.0, u_ar)          # the filter is not ignored
    a, _ = oracle.speculative_generate(target, draft, prompt, n_new, K, 1.0, ud, ua, top_p=1.0)
    b, _ = oracle.speculative_generate(target, draft, prompt, n_new, K, 1.0, ud, ua)
    assert a == b
    toks, st = oracle.speculative_generate(target, draft, prompt, n_new, K, 1.0, ud, ua, top_p=top_p)
    x = list(prompt)
    for t in toks:
        row = oracle.softmax(target.forward(target.new_kv(64), x)[-1], 1.0)
        assert oracle.top_p_filter(row, top_p)[t] > 0
        x.append(t)
