"""Weight-only int8 matrices on the GPU path (the quantised model Sections 2 and 3 assume; reading: one fp32
scale per output row, activations and cache untouched): the library's quantiser against the oracle's bit for
bit, the forward pass of an int8 model against the oracle's int8 model (logits max-abs 2e-2, the bf16
tolerance: activations and cache are bf16), the speculative loop on int8 models, refused configurations."""
import numpy as np
import pytest
import torch

import oracle
import paper_2311_04951_amd as sv
import seeded_inputs as si
from paper_2311_04951_amd import generate as gen
from gpu_util import dev, maxabs, weights_to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,N,K", [("f32", 37, 200), ("bf16", 64, 4096), ("bf16", 5, 11008), ("f32", 300, 16), ("bf16", 3, 1)])
def test_quantiser_equals_oracle_bit_for_bit(dtype, N, K):
    W = si.normal(21, f"wq8_{N}_{K}", (N, K), 0.02, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)
    if N > 2:
        W[1] = 0.0                       # a zero row: scale 1, all zeros
        W[2, K // 2] = 3.0               # one large element: everything else in the row rounds to few levels
    oq, osc = oracle.quantize_rows_int8(W, is_bf16=dtype == "bf16")
    gq, gsc = sv.ss_quantize_rows_int8(W.to(dev()))
    assert np.array_equal(gq.cpu().numpy(), oq)
    assert np.array_equal(gsc.cpu().numpy().view(np.uint32), osc.view(np.uint32))


def _int8_pair(shape, seed, max_pos=256):
    w = si.decoder_weights(shape, seed)
    om = oracle.Model(shape, w, int8_weights=True)
    gm = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=max_pos, int8_weights=True)
    return om, gm, w


@pytest.mark.parametrize("shape", [si.DecoderShape(2, 256, 4, 64, 688, 1000, dtype="bf16"),     # K = 688: a ragged last 128-entry step
                                   si.DecoderShape(1, 128, 4, 32, 336, 515, dtype="bf16")])     # vocabulary not a multiple of 16
def test_int8_model_forward_matches_int8_oracle(shape):
    om, gm, _ = _int8_pair(shape, 31)
    toks = si.token_ids(31, "t", (30,), shape.vocab).numpy().astype(np.int32)
    okv, gkv = om.new_kv(64), sv.KVCache(gm, 1, 64)
    worst = 0.0
    for lo, hi in [(0, 16), (16, 21), (21, 22), (22, 30)]:       # prefill chunk, a 5-row verify call, one row, 8 rows
        ref = om.forward(okv, toks[lo:hi])
        got = sv.ss_verify_forward(gm, gkv, torch.tensor(toks[None, lo:hi], device=dev()), hi - lo)
        worst = max(worst, maxabs(got[0], ref))
    assert worst < 2e-2
    assert sv.ss_device_status(gm) == 0
    # the quantised model is not the plain one: the flag is not ignored
    pm = sv.Model(shape, weights_to_device(si.decoder_weights(shape, 31)), max_rows=16, max_pos=256)
    pkv = sv.KVCache(pm, 1, 64)
    plain = sv.ss_verify_forward(pm, pkv, torch.tensor(toks[None, :16], device=dev()), 16)
    gkv2 = sv.KVCache(gm, 1, 64)
    quant = sv.ss_verify_forward(gm, gkv2, torch.tensor(toks[None, :16], device=dev()), 16)
    assert maxabs(plain, quant.cpu().numpy()) > 1e-4


def test_int8_7b_layer_and_head_match_oracle():
    """A 7B-shaped model of one layer with int8 matrices: 5 query rows against 1024 cached positions through
    embedding, layer, final norm and the int8 LM head (32000 x 4096) - logits against the oracle."""
    shape = si.LAYER_7B
    w = si.decoder_weights(shape, 0)
    om = oracle.Model(shape, w, int8_weights=True)
    gm = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=2048, int8_weights=True)
    L, M = 1024, 5
    ctx = si.kv_context(shape, 0, "ctx", L)
    gkv = sv.KVCache(gm, 1, L + 64)
    sv.ss_kv_cache_append(gkv, 0, 0, 0, ctx[0][0].to(dev()), ctx[0][1].to(dev()))
    sv.ss_kv_cache_set_len(gkv, [L])
    okv = om.new_kv(L + 64)
    okv.append_raw(ctx)
    toks = si.token_ids(0, "t7b8", (M,), shape.vocab).numpy().astype(np.int32)
    got = sv.ss_verify_forward(gm, gkv, torch.tensor(toks[None], device=dev()), M)[0].cpu().numpy()
    ref = om.forward(okv, toks)
    assert maxabs(got, ref) < 2e-2
    assert maxabs(got, ref) < 2e-3
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [L + M]


def test_greedy_speculative_equals_greedy_autoregressive_with_int8_models():
    shape = si.DecoderShape(3, 256, 4, 64, 688, 1000, dtype="bf16")
    w = si.decoder_weights(shape, 41)
    dshape, dw = si.early_exit_draft(shape, w, 1)
    gt = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=256, int8_weights=True)
    gd = sv.Model(dshape, weights_to_device(dw), max_rows=16, max_pos=256, int8_weights=True)
    prompt = si.token_ids(41, "prompt", (20,), shape.vocab).numpy().tolist()
    ar = gen.autoregressive_generate(gt, prompt, 40, 0.0)
    sp, stats = gen.speculative_generate(gt, gd, prompt, 40, 4, 0.0)
    assert sp == ar and all(0 <= a <= 4 for a in stats["accepted"])
    # sampled: the one-call step and the call-by-call step give the same stream on the same uniforms
    ud, ua = si.uniforms(41, "ud", (40, 4)).numpy(), si.uniforms(41, "ua", (40, 5)).numpy()
    s1, st1 = gen.speculative_generate(gt, gd, prompt, 40, 4, 1.0, ud, ua)
    s2, st2 = gen.speculative_generate(gt, gd, prompt, 40, 4, 1.0, ud, ua, observer=lambda s: None)
    assert s1 == s2 and st1["accepted"] == st2["accepted"]


@pytest.mark.parametrize("B,M,vocab", [(3, 8, 1000), (3, 16, 1000), (8, 9, 1000),      # 24, 48 and 72 rows per call: 2, 3 and 5 row tiles
                                       (3, 8, 20000), (3, 16, 20000), (8, 9, 20000)])  # an LM head of 1250 tiles: 8-wave workgroups
def test_int8_model_in_launches_of_more_than_16_rows(B, M, vocab):
    """Batched calls of an int8 model go through the wide GEMMs (LDS-shared activation slabs, split-K): whole
    forward with ragged contexts, every sequence against the oracle's int8 model run on that sequence alone.
    d_ff = 688 gives the down projection a ragged last K slab."""
    shape = si.DecoderShape(2, 256, 4, 64, 688, vocab, dtype="bf16")
    w = si.decoder_weights(shape, 51)
    om = oracle.Model(shape, w, int8_weights=True)
    gm = sv.Model(shape, weights_to_device(w), max_rows=B * M, max_pos=256, int8_weights=True)
    lens = [37, 1, 150, 64, 9, 200, 77, 128][:B]
    gkv = sv.KVCache(gm, B, 256)
    toks = si.token_ids(51, f"t{B}x{M}", (B, M), shape.vocab).numpy().astype(np.int32)
    refs = []
    for b in range(B):
        ctx = si.kv_context(shape, 51, f"ctx{b}", lens[b])
        okv = om.new_kv(256)
        okv.append_raw(ctx)
        for l in range(shape.n_layers):
            sv.ss_kv_cache_append(gkv, l, b, 0, ctx[l][0].to(dev()), ctx[l][1].to(dev()))
        refs.append(om.forward(okv, toks[b]))
    sv.ss_kv_cache_set_len(gkv, lens)
    got = sv.ss_verify_forward(gm, gkv, torch.from_numpy(toks).to(dev()), M).cpu().numpy()
    for b in range(B):
        assert maxabs(got[b], refs[b]) < 2e-2, b
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [l + M for l in lens]
    assert sv.ss_device_status(gm) == 0


def test_int8_configurations_that_are_refused():
    shape = si.DecoderShape(1, 128, 4, 32, 336, 512, dtype="bf16")
    w = weights_to_device(si.decoder_weights(shape, 5))
    f32 = si.DecoderShape(1, 128, 4, 32, 336, 512, dtype="f32")
    with pytest.raises(sv.SpecVerifyError):
        sv.Model(f32, weights_to_device(si.decoder_weights(f32, 5)), max_rows=16, max_pos=64, int8_weights=True)
    odd = si.DecoderShape(1, 128, 4, 32, 344, 512, dtype="bf16")                   # d_ff = 344: not a multiple of 16
    with pytest.raises(sv.SpecVerifyError):
        sv.Model(odd, weights_to_device(si.decoder_weights(odd, 5)), max_rows=16, max_pos=64, int8_weights=True)
    gm = sv.Model(shape, w, max_rows=16, max_pos=64, int8_weights=True)
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_model_set_persistent(gm, True)                                       # the persistent kernel does not take int8 matrices
