"""Weight-only int4 matrices with group scales on the GPU path (groups of 128 entries along K; the coarser of
the two readings of the quantised model Sections 2 and 3 assume): the library's quantiser against the oracle's
bit for bit (packed bytes and scales), the forward pass of an int4 model against the oracle's int4 model
(logits max-abs 2e-2: activations and cache are bf16), the loop, refused configurations."""
import numpy as np
import pytest
import torch

import oracle
import paper_2311_04951_amd as sv
import seeded_inputs as si
from paper_2311_04951_amd import generate as gen
from gpu_util import dev, maxabs, weights_to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,N,K", [("f32", 37, 256), ("bf16", 64, 4096), ("bf16", 5, 11008), ("f32", 300, 128)])
def test_quantiser_equals_oracle_bit_for_bit(dtype, N, K):
    W = si.normal(22, f"wq4_{N}_{K}", (N, K), 0.02, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)
    W[1, :128] = 0.0                      # a zero group: scale 1, zero nibbles
    W[2, K // 2] = 3.0                    # one large element: the rest of its group rounds to zero
    oq, osc = oracle.quantize_rows_int4(W, is_bf16=dtype == "bf16")
    gq, gsc = sv.ss_quantize_rows_int4(W.to(dev()))
    assert np.array_equal(gq.cpu().numpy(), oq)
    assert np.array_equal(gsc.cpu().numpy().view(np.uint32), osc.view(np.uint32))
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_quantize_rows_int4(W[:, :100].contiguous().to(dev()))


@pytest.mark.parametrize("shape", [si.DecoderShape(2, 256, 4, 64, 640, 1000, dtype="bf16"),
                                   si.DecoderShape(1, 128, 4, 32, 384, 515, dtype="bf16")])      # vocabulary not a multiple of 16
def test_int4_model_forward_matches_int4_oracle(shape):
    w = si.decoder_weights(shape, 32)
    om = oracle.Model(shape, w, int4_weights=True)
    gm = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=256, int4_weights=True)
    toks = si.token_ids(32, "t", (30,), shape.vocab).numpy().astype(np.int32)
    okv, gkv = om.new_kv(64), sv.KVCache(gm, 1, 64)
    worst = 0.0
    for lo, hi in [(0, 16), (16, 21), (21, 22), (22, 30)]:
        ref = om.forward(okv, toks[lo:hi])
        got = sv.ss_verify_forward(gm, gkv, torch.tensor(toks[None, lo:hi], device=dev()), hi - lo)
        worst = max(worst, maxabs(got[0], ref))
    assert worst < 2e-2
    assert sv.ss_device_status(gm) == 0
    # not the int8 model: the flag selects the path
    g8 = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=256, int8_weights=True)
    a = sv.ss_verify_forward(gm, sv.KVCache(gm, 1, 64), torch.tensor(toks[None, :16], device=dev()), 16)
    b = sv.ss_verify_forward(g8, sv.KVCache(g8, 1, 64), torch.tensor(toks[None, :16], device=dev()), 16)
    assert maxabs(a, b.cpu().numpy()) > 1e-4


def test_int4_7b_layer_and_head_match_oracle():
    shape = si.LAYER_7B
    w = si.decoder_weights(shape, 0)
    om = oracle.Model(shape, w, int4_weights=True)
    gm = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=2048, int4_weights=True)
    L, M = 1024, 5
    ctx = si.kv_context(shape, 0, "ctx", L)
    gkv = sv.KVCache(gm, 1, L + 64)
    sv.ss_kv_cache_append(gkv, 0, 0, 0, ctx[0][0].to(dev()), ctx[0][1].to(dev()))
    sv.ss_kv_cache_set_len(gkv, [L])
    okv = om.new_kv(L + 64)
    okv.append_raw(ctx)
    toks = si.token_ids(0, "t7b4", (M,), shape.vocab).numpy().astype(np.int32)
    got = sv.ss_verify_forward(gm, gkv, torch.tensor(toks[None], device=dev()), M)[0].cpu().numpy()
    ref = om.forward(okv, toks)
    assert maxabs(got, ref) < 2e-2
    assert maxabs(got, ref) < 2e-3


def test_loops_with_int4_models():
    shape = si.DecoderShape(3, 256, 4, 64, 640, 1000, dtype="bf16")
    w = si.decoder_weights(shape, 42)
    dshape, dw = si.early_exit_draft(shape, w, 1)
    gt = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=256, int4_weights=True)
    gd = sv.Model(dshape, weights_to_device(dw), max_rows=16, max_pos=256, int4_weights=True)
    prompt = si.token_ids(42, "prompt", (20,), shape.vocab).numpy().tolist()
    ar = gen.autoregressive_generate(gt, prompt, 40, 0.0)
    sp, stats = gen.speculative_generate(gt, gd, prompt, 40, 4, 0.0)
    assert sp == ar
    ud, ua = si.uniforms(42, "ud", (40, 4)).numpy(), si.uniforms(42, "ua", (40, 5)).numpy()
    s1, st1 = gen.speculative_generate(gt, gd, prompt, 40, 4, 1.0, ud, ua)
    s2, st2 = gen.speculative_generate(gt, gd, prompt, 40, 4, 1.0, ud, ua, observer=lambda s: None)
    assert s1 == s2 and st1["accepted"] == st2["accepted"]


@pytest.mark.parametrize("B,M", [(3, 8), (8, 9)])      # 24 and 72 rows per call: 2 and 5 row tiles
def test_int4_model_in_launches_of_more_than_16_rows(B, M):
    """Batched calls of an int4 model (one workgroup per column tile and row tile): whole forward with ragged
    contexts, every sequence against the oracle's int4 model run on that sequence alone."""
    shape = si.DecoderShape(2, 256, 4, 64, 768, 1000, dtype="bf16")
    w = si.decoder_weights(shape, 52)
    om = oracle.Model(shape, w, int4_weights=True)
    gm = sv.Model(shape, weights_to_device(w), max_rows=B * M, max_pos=256, int4_weights=True)
    lens = [37, 1, 150, 64, 9, 200, 77, 128][:B]
    gkv = sv.KVCache(gm, B, 256)
    toks = si.token_ids(52, f"t{B}x{M}", (B, M), shape.vocab).numpy().astype(np.int32)
    refs = []
    for b in range(B):
        ctx = si.kv_context(shape, 52, f"ctx{b}", lens[b])
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


def test_int4_configurations_that_are_refused():
    shape = si.DecoderShape(1, 128, 4, 32, 384, 512, dtype="bf16")
    w = weights_to_device(si.decoder_weights(shape, 5))
    odd = si.DecoderShape(1, 128, 4, 32, 336, 512, dtype="bf16")                   # d_ff = 336: not a multiple of 128
    with pytest.raises(sv.SpecVerifyError):
        sv.Model(odd, weights_to_device(si.decoder_weights(odd, 5)), max_rows=16, max_pos=64, int4_weights=True)
    gm = sv.Model(shape, w, max_rows=16, max_pos=64, int4_weights=True)
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_model_set_persistent(gm, True)
