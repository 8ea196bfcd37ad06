"""Pins of the oracle's int4 path (groups of 128 entries along K share one scale; the coarser reading of the
"quantized model" of Sections 2 and 3).  Matrices on an int4 grid with power-of-two group scales are recovered
exactly and make the int4 linear layer and the int4 model equal the plain ones bit for bit; error bound, packing,
ties and the group-major scale layout are checked directly."""
import numpy as np
import pytest
import torch

import oracle
import seeded_inputs as si

G = oracle.W4_GROUP


def _grid(rng, N, K, shift=0):
    """q in [-7, 7] with a +-7 in every group of every row; scale[j][n] = 2**-(5 + (n + 2j + shift) % 4)."""
    q = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    for j in range(K // G):
        q[np.arange(N), j * G + rng.integers(0, G, size=N)] = np.where(rng.random(N) < 0.5, 7, -7)
    e = 5 + (np.arange(N)[None, :] + 2 * np.arange(K // G)[:, None] + shift) % 4
    s = (2.0 ** -e).astype(np.float32)                                  # [K/G, N]
    W = (q.astype(np.float32).reshape(N, K // G, G) * s.T[:, :, None]).reshape(N, K).astype(np.float32)
    return q, s, W


def _unpack(p):
    lo = (p & 0xf).astype(np.int8)
    hi = (p >> 4).astype(np.int8)
    out = np.empty((p.shape[0], p.shape[1] * 2), dtype=np.int8)
    out[:, 0::2] = np.where(lo >= 8, lo - 16, lo)
    out[:, 1::2] = np.where(hi >= 8, hi - 16, hi)
    return out


def test_quantiser_recovers_grid_matrices_and_packs_low_nibble_first():
    rng = np.random.default_rng(0)
    q, s, W = _grid(rng, 19, 3 * G)
    gq, gs = oracle.quantize_rows_int4(W)
    assert gq.shape == (19, 3 * G // 2) and gs.shape == (3, 19)
    assert np.array_equal(_unpack(gq), q) and np.array_equal(gs, s)
    Wb = torch.from_numpy(W).to(torch.bfloat16)
    assert torch.equal(Wb.float(), torch.from_numpy(W))
    gq, gs = oracle.quantize_rows_int4(Wb, is_bf16=True)
    assert np.array_equal(_unpack(gq), q) and np.array_equal(gs, s)
    # packing by hand: entries (1, -2) of one byte -> low nibble 1, high nibble 0xE
    row = np.zeros((1, G), dtype=np.float32)
    row[0, :4] = [1, -2, 7, -7]
    p, sc = oracle.quantize_rows_int4(row)
    assert sc[0, 0] == 1.0 and p[0, 0] == 0xE1 and p[0, 1] == 0x97 and not p[0, 2:].any()


def test_quantiser_error_bound_ties_and_zero_groups():
    W = si.normal(4, "w4", (33, 4 * G), 0.02).numpy()
    W[3, G:2 * G] = 0.0
    p, s = oracle.quantize_rows_int4(W)
    q = _unpack(p).astype(np.float64)
    assert s[1, 3] == 1.0 and not q[3, G:2 * G].any()
    srow = np.repeat(s.T.astype(np.float64), G, axis=1)                  # [N, K]
    assert np.all(np.abs(W - q * srow) <= 0.5 * srow * (1 + 1e-6))
    amax = np.abs(W.reshape(33, 4, G)).max(axis=2)
    live = amax > 0
    np.testing.assert_allclose(s.T[live], amax[live] / 7.0, rtol=2e-7)
    assert np.abs(q).max() == 7
    # ties to even, scale 2**-2 (group maximum 7/4)
    row = np.zeros((1, G), dtype=np.float32)
    row[0, :8] = np.array([7, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 6.5], dtype=np.float32) / 4
    p, sc = oracle.quantize_rows_int4(row)
    assert sc[0, 0] == 0.25 and _unpack(p)[0, :8].tolist() == [7, 0, 2, 2, 0, -2, -2, 6]


def test_int4_linear_equals_plain_linear_on_grid_weights_and_numpy_elsewhere():
    rng = np.random.default_rng(1)
    q, s, W = _grid(rng, 40, 2 * G)
    p, _ = oracle.quantize_rows_int4(W)
    x = si.normal(1, "x4", (2 * G,), 1.0).numpy()
    # power-of-two scales: sum_j s_j sum_k q x and sum_k (s q) x are the same fp64 number
    assert np.array_equal(oracle.linear_w4(p, s, x), oracle.linear(W, x))
    s2 = (np.abs(si.normal(2, "s4", (2, 40), 0.01).numpy()) + 1e-3).astype(np.float32)
    want = np.einsum("ngk,gn,gk->n", q.astype(np.float64).reshape(40, 2, G), s2.astype(np.float64), x.astype(np.float64).reshape(2, G))
    np.testing.assert_allclose(oracle.linear_w4(p, s2, x), want, rtol=1e-6, atol=1e-9)
    # the scale layout is group-major: its transpose-in-memory or a swap of the two groups must show
    assert not np.allclose(oracle.linear_w4(p, s2[::-1].copy(), x), want, rtol=1e-3)
    assert not np.allclose(oracle.linear_w4(p, np.ascontiguousarray(s2.T).reshape(2, 40), x), want, rtol=1e-3)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_int4_model_equals_plain_model_when_quantisation_loses_nothing(dtype):
    shape = si.DecoderShape(2, 128, 2, 64, 384, 512, dtype=dtype)
    w = si.decoder_weights(shape, 13)
    rng = np.random.default_rng(13)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    for l, lw in enumerate(w["layers"]):
        for i, n in enumerate(("wq", "wk", "wv", "wo", "wg", "wu", "wd")):
            lw[n] = torch.from_numpy(_grid(rng, *lw[n].shape, shift=i + l)[2]).to(dt)
    w["lm_head"] = torch.from_numpy(_grid(rng, *w["lm_head"].shape, shift=5)[2]).to(dt)
    plain, quant = oracle.Model(shape, w), oracle.Model(shape, w, int4_weights=True)
    toks = si.token_ids(13, "t", (9,), shape.vocab).numpy()
    kp, kq = plain.new_kv(16), quant.new_kv(16)
    assert np.array_equal(plain.forward(kp, toks[:6]), quant.forward(kq, toks[:6]))
    assert np.array_equal(plain.forward(kp, toks[6:]), quant.forward(kq, toks[6:]))


def test_int4_model_differs_from_the_int8_and_the_plain_model_on_ordinary_weights():
    shape = si.DecoderShape(2, 256, 4, 64, 640, 1024, dtype="f32")
    w = si.decoder_weights(shape, 0)
    toks = si.token_ids(0, "t4", (5,), shape.vocab).numpy()
    outs = [oracle.Model(shape, w, **kw) for kw in ({}, {"int8_weights": True}, {"int4_weights": True})]
    a, b, c = [m.forward(m.new_kv(8), toks) for m in outs]
    d8, d4 = np.abs(a - b).max(), np.abs(a - c).max()
    assert 0 < d8 < d4 < 0.5 * np.abs(a).max()
