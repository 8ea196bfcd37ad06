"""Pins of the oracle's top-k filter (Section 3 lists top-k with top-p among the usual token selection rules;
the arithmetic is this build's reading: integer weights, ties by index, fp32 renormalisation, top-k before
top-p).  Hand-made rows with exact arithmetic, brute force over all subsets on tiny rows, a re-derivation in
exact integer arithmetic on random rows with ties, the defining properties, and the distribution the
rejection step emits when both models are filtered."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import scipy.stats

import oracle
import seeded_inputs as si


def _w(p):
    return [min(int(Fraction(float(x)) * 2 ** 32), 2 ** 32 - 1) if x > 0 else 0 for x in p]


def test_hand_made_rows():
    p = np.array([0.125, 0.5, 0.125, 0.25], dtype=np.float32)            # exact binary fractions
    assert np.array_equal(oracle.top_k_filter(p, 1), np.array([0, 1, 0, 0], dtype=np.float32))
    assert np.array_equal(oracle.top_k_filter(p, 2), np.array([0, 2 / 3, 0, 1 / 3], dtype=np.float32))
    # the third token is one of two equal ones: the lower index wins
    np.testing.assert_array_equal(oracle.top_k_filter(p, 3), (p / np.float32(0.875)) * np.array([1, 1, 0, 1], dtype=np.float32))
    # k = V and beyond, and k < 1: the row comes back unchanged (not even renormalised)
    half = (p * np.float32(0.5)).astype(np.float32)
    for k in (4, 5, 1000, 0, -3):
        assert np.array_equal(oracle.top_k_filter(half, k), half)
    # all equal: the k lowest indices, 1/k each
    flat = np.full(8, 0.125, dtype=np.float32)
    assert np.array_equal(oracle.top_k_filter(flat, 4), np.array([0.25] * 4 + [0] * 4, dtype=np.float32))
    # a row without any weight is returned as it is
    tiny = np.full(4, 1e-12, dtype=np.float32)
    assert np.array_equal(oracle.top_k_filter(tiny, 2), tiny)
    # rows are independent
    both = oracle.top_k_filter(np.stack([p, flat[:4]]), 2)
    assert np.array_equal(both[0], oracle.top_k_filter(p, 2)) and np.array_equal(both[1], oracle.top_k_filter(flat[:4], 2))
    # both rules: top-k first, top-p on its output ([2/3, 1/3] at 0.6 keeps the first only)
    assert np.array_equal(oracle.select(p, top_k=2, top_p=0.6), np.array([0, 1, 0, 0], dtype=np.float32))
    assert np.array_equal(oracle.select(p, top_k=2, top_p=1.0), oracle.top_k_filter(p, 2))
    assert np.array_equal(oracle.select(p, top_k=0, top_p=0.8), oracle.top_p_filter(p, 0.8))


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_heaviest_subset_of_size_k_on_tiny_rows(seed):
    """V = 7: among all subsets of k tokens the kept set has the largest integer weight, and among those of the
    largest weight it is the first in index order; the values are the fp32 quotients by the kept weight."""
    rng = np.random.default_rng(seed)
    V = 7
    p = rng.random(V).astype(np.float32)
    if seed % 2:
        p[rng.integers(0, V, 3)] = p[0]            # ties
    p = (p / p.sum()).astype(np.float32)
    w = _w(p)
    for k in range(1, V):
        best = max(itertools.combinations(range(V), k), key=lambda c: (sum(w[i] for i in c), [-i for i in c]))
        got = oracle.top_k_filter(p, k)
        assert sorted(np.flatnonzero(got).tolist()) == sorted(best), (seed, k)
        Z = np.float32(np.float32(sum(w[i] for i in best)) * np.float32(2.0 ** -32))
        want = np.zeros(V, dtype=np.float32)
        want[list(best)] = p[list(best)] / Z
        assert np.array_equal(got, want), (seed, k)


@pytest.mark.parametrize("V,k", [(50, 1), (50, 7), (1000, 40), (1000, 999), (4097, 50)])
def test_against_exact_integer_rederivation_with_ties(V, k):
    rows = si.accept_workload(77, 3, 1, V)[0][:, 0].numpy()
    rows = oracle.softmax(rows, 0.8)
    rows[1, ::3] = rows[1, 0]            # many equal weights straddling the cut
    rows[2, V // 2:] = 0.0               # fewer tokens with weight than k may ask for
    for r in range(rows.shape[0]):
        p = rows[r]
        w = _w(p)
        order = sorted(range(V), key=lambda v: (-w[v], v))[:k]
        S = sum(w[v] for v in order)
        got = oracle.top_k_filter(p, k)
        Z = np.float32(np.float32(S) * np.float32(2.0 ** -32))
        want = np.zeros(V, dtype=np.float32)
        want[order] = p[order] / Z
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (V, k, r)


def test_properties_on_random_rows():
    rows = oracle.softmax(si.accept_workload(5, 6, 1, 2000)[0][:, 0].numpy(), 1.0)
    prev = None
    for k in (1, 5, 50, 500, 1999):
        f = oracle.top_k_filter(rows, k)
        for r in range(rows.shape[0]):
            keep = f[r] > 0
            assert keep.sum() == k
            assert rows[r][keep].min() >= rows[r][~keep].max()                 # nothing dropped outweighs anything kept
            assert abs(f[r].astype(np.float64).sum() - 1.0) < 1e-5               # renormalised
            ratio = f[r][keep].astype(np.float64) / rows[r][keep].astype(np.float64)
            assert ratio.max() / ratio.min() < 1 + 1e-6                         # one common factor
        if prev is not None:
            assert np.all((prev > 0) <= (f > 0))                                # a larger k keeps a superset
        prev = f


def test_filtered_speculative_step_emits_the_filtered_target():
    """Both rows filtered with the same top_k, then the rejection step: the emitted token follows the filtered
    target row (chi-square, 400 000 trials) and never leaves its k tokens."""
    rng = np.random.default_rng(4)
    V, N, k = 10, 400_000, 4
    p = rng.random(V).astype(np.float32); p = (p / p.sum()).astype(np.float32)
    q = rng.random(V).astype(np.float32); q = (q / q.sum()).astype(np.float32)
    pf, qf = oracle.top_k_filter(p, k), oracle.top_k_filter(q, k)
    assert np.count_nonzero(pf) == k and np.count_nonzero(qf) == k and np.any((pf > 0) != (qf > 0))
    ud = si.uniforms(4, "ud", (N,)).numpy()
    edges = np.cumsum(_w(qf))
    thr = (np.round(ud * 2 ** 24).astype(np.uint64) * np.uint64(edges[-1])) >> np.uint64(24)
    d = np.searchsorted(edges, thr, side="right").astype(np.int32)
    assert all(d[i] == oracle.sample(qf, ud[i]) for i in range(0, N, N // 100))
    pp = np.broadcast_to(np.stack([pf, pf])[None], (N, 2, V)).copy()
    qq = np.broadcast_to(qf[None, None], (N, 1, V)).copy()
    na, nx = oracle.speculative_accept(pp, qq, d[:, None], si.uniforms(4, "u", (N, 2)).numpy())
    out = np.where(na == 1, d, nx)
    hist = np.bincount(out, minlength=V)
    assert np.all(hist[pf == 0] == 0)
    keep = pf > 0
    pd = pf[keep].astype(np.float64) / pf.astype(np.float64).sum()
    assert scipy.stats.chisquare(hist[keep], pd * N).pvalue > 1e-4
    pu = p.astype(np.float64)
    assert scipy.stats.chisquare(hist, pu / pu.sum() * N).pvalue < 1e-12      # the unfiltered target is rejected


def test_loops_with_top_k():
    """Identical models: everything is accepted and the stream is autoregressive top-k sampling with the
    interleaved uniforms; top_k = 1 is greedy decoding whatever the uniforms are."""
    tw = si.decoder_weights(si.TINY_TARGET, 8)
    target = oracle.Model(si.TINY_TARGET, tw)
    draft = oracle.Model(si.TINY_DRAFT, si.decoder_weights(si.TINY_DRAFT, 108))
    prompt = si.token_ids(8, "prompt", (8,), 1024).numpy()
    K, n_new, k = 3, 16, 5
    steps = n_new // (K + 1)
    ud, ua = si.uniforms(8, "ud", (n_new, K)).numpy(), si.uniforms(8, "ua", (n_new, K + 1)).numpy()
    sp, stats = oracle.speculative_generate(target, target, prompt, n_new, K, 1.0, ud, ua, top_k=k)
    assert all(a == K for a in stats["accepted"])
    u_ar = np.concatenate([np.concatenate([ud[s], ua[s, K:]]) for s in range(steps)])
    assert sp == oracle.autoregressive_generate(target, prompt, n_new, 1.0, u_ar, top_k=k)
    assert sp != oracle.autoregressive_generate(target, prompt, n_new, 1.0, u_ar)          # the filter is not ignored
    greedy = oracle.autoregressive_generate(target, prompt, n_new, 0.0)
    assert oracle.autoregressive_generate(target, prompt, n_new, 1.0, u_ar, top_k=1) == greedy
    one, _ = oracle.speculative_generate(target, draft, prompt, n_new, K, 1.0, ud, ua, top_k=1)
    assert one == greedy                                                                   # a real draft changes nothing
