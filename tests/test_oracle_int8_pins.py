"""Pins of the oracle's weight-only int8 path (the reading of the paper's "quantized model", Sections 2
and 3: int8 weights with one scale per output row, activations untouched).  The quantiser is pinned by
matrices that lie exactly on an int8 grid, by its error bound and by hand-made ties; the int8 linear layer
and the int8 model are pinned to the plain ones (themselves pinned against library routines and a library
Llama) through weights for which quantisation loses nothing."""
import numpy as np
import pytest
import torch

import oracle
import seeded_inputs as si


def _grid_matrix(rng, N, K, exps):
    """Rows s_n * integers in [-127, 127] with s_n = 2**-exps[n] and at least one +-127 per row."""
    q = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    q[np.arange(N), rng.integers(0, K, size=N)] = np.where(rng.random(N) < 0.5, 127, -127)
    s = (2.0 ** -np.asarray(exps, dtype=np.float64)).astype(np.float32)
    return q, s, (q.astype(np.float32) * s[:, None]).astype(np.float32)


def test_quantiser_recovers_a_matrix_that_lies_on_the_grid():
    rng = np.random.default_rng(0)
    q, s, W = _grid_matrix(rng, 37, 96, 5 + np.arange(37) % 4)
    gq, gs = oracle.quantize_rows_int8(W)
    assert np.array_equal(gq, q) and np.array_equal(gs, s)
    # the same through bf16 storage (integers up to 127 times a power of two are exact in bf16)
    Wb = torch.from_numpy(W).to(torch.bfloat16)
    assert torch.equal(Wb.float(), torch.from_numpy(W))
    gq, gs = oracle.quantize_rows_int8(Wb, is_bf16=True)
    assert np.array_equal(gq, q) and np.array_equal(gs, s)


def test_quantiser_error_bound_extremes_and_zero_rows():
    W = si.normal(3, "w8", (64, 200), 0.02).numpy()
    W[5] = 0.0
    q, s = oracle.quantize_rows_int8(W)
    assert q.dtype == np.int8 and s.dtype == np.float32
    assert np.all(q[5] == 0) and s[5] == 1.0
    live = np.arange(64) != 5
    amax = np.abs(W).max(axis=1)
    np.testing.assert_allclose(s[live], amax[live] / 127.0, rtol=2e-7)
    # the largest element of a row maps to +-127, nothing leaves [-127, 127]
    arg = np.abs(W).argmax(axis=1)
    assert np.all(np.abs(q[np.arange(64), arg][live]) == 127) and np.abs(q.astype(np.int32)).max() == 127
    # nearest grid point: |w - q s| <= s/2 (plus the rounding of the fp32 division)
    err = np.abs(W.astype(np.float64) - q.astype(np.float64) * s[:, None].astype(np.float64))
    assert np.all(err <= 0.5 * s[:, None].astype(np.float64) * (1 + 1e-6))
    # signs are kept and the map is monotone along a row
    assert np.all(np.sign(q[live]) * np.sign(W[live]) >= 0)
    order = np.argsort(W[7])
    assert np.all(np.diff(q[7][order].astype(np.int32)) >= 0)


def test_quantiser_rounds_ties_to_even():
    # scale 2**-4 (the row maximum is 127/16); halves of the grid step are exact in fp32
    row = np.array([127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, 126.5, -126.5], dtype=np.float32) / 16.0
    q, s = oracle.quantize_rows_int8(row[None, :])
    assert s[0] == np.float32(1 / 16)
    assert q[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 4, 126, -126]


def test_int8_linear_equals_plain_linear_on_grid_weights_and_library_matmul_elsewhere():
    rng = np.random.default_rng(1)
    q, s, W = _grid_matrix(rng, 48, 160, 3 + np.arange(48) % 5)
    x = si.normal(1, "x8", (160,), 1.0).numpy()
    # scales are powers of two: s * sum(q x) and sum((s q) x) are the same fp64 number
    assert np.array_equal(oracle.linear_w8(q, s, x), oracle.linear(W, x))
    # arbitrary scales: against numpy in fp64
    s2 = np.abs(si.normal(2, "s8", (48,), 0.01).numpy()) + 1e-3
    want = (s2.astype(np.float64)[:, None] * q.astype(np.float64)) @ x.astype(np.float64)
    np.testing.assert_allclose(oracle.linear_w8(q, s2, x), want, rtol=1e-6, atol=1e-9)
    # a transposed or shifted scale vector must show: the rows have different scales
    assert not np.allclose(oracle.linear_w8(q, np.roll(s2, 1), x), want, rtol=1e-3)


def _grid_model_weights(shape, seed):
    """decoder_weights whose seven matrices per layer and LM head lie on int8 grids with row-dependent
    power-of-two scales (a different exponent pattern per matrix, so a swapped scale vector shows)."""
    w = si.decoder_weights(shape, seed)
    rng = np.random.default_rng(seed)
    dt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32

    def grid(t, shift):
        N, K = t.shape
        _, _, W = _grid_matrix(rng, N, K, 9 + (np.arange(N) + shift) % 3)
        return torch.from_numpy(W).to(dt)

    for l, lw in enumerate(w["layers"]):
        for i, n in enumerate(("wq", "wk", "wv", "wo", "wg", "wu", "wd")):
            lw[n] = grid(lw[n], i + l)
    w["lm_head"] = grid(w["lm_head"], 5)
    return w


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_int8_model_equals_plain_model_when_quantisation_loses_nothing(dtype):
    shape = si.DecoderShape(2, 128, 2, 64, 352, 512, dtype=dtype)
    w = _grid_model_weights(shape, 11)
    plain, quant = oracle.Model(shape, w), oracle.Model(shape, w, int8_weights=True)
    toks = si.token_ids(11, "t", (9,), shape.vocab).numpy()
    kp, kq = plain.new_kv(16), quant.new_kv(16)
    a = plain.forward(kp, toks[:6])
    b = quant.forward(kq, toks[:6])
    assert np.array_equal(a, b)
    assert np.array_equal(plain.forward(kp, toks[6:]), quant.forward(kq, toks[6:]))   # rows against the cache


def test_int8_model_is_close_to_but_not_equal_to_the_unquantised_model():
    """On ordinary weights quantisation changes the logits a little (so the int8 flag is not ignored) and
    the result is exactly what dequantised weights would give in the plain model when the scales are kept
    out of the rounding: checked through the int8 linear layer on one matrix."""
    shape = si.TINY_TARGET
    w = si.decoder_weights(shape, 0)
    plain, quant = oracle.Model(shape, w), oracle.Model(shape, w, int8_weights=True)
    toks = si.token_ids(0, "t8", (5,), shape.vocab).numpy()
    a, b = plain.forward(plain.new_kv(8), toks), quant.forward(quant.new_kv(8), toks)
    d = np.abs(a - b).max()
    assert 0 < d < 0.05 * np.abs(a).max()
