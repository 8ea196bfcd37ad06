"""GPU parity of the verify pass (decoder forward against the KV cache) with the CPU oracle.

Tolerance on logits / hidden rows: max-abs 1e-4 with fp32 storage, 2e-2 with bf16 storage
(the contract of this repository's target; the fp32 figure is ~100x the fp32 accumulation noise of
these shapes, the bf16 figure covers a flipped bf16 rounding of a cache entry)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2311_04951_amd as sv
import seeded_inputs as si
from gpu_util import PATHS, dev, maxabs, model_pair, set_path, tol, weights_to_device

pytestmark = pytest.mark.gpu


def _gpu_forward_chunks(gm, gkv, toks, chunks):
    outs, i = [], 0
    for c in chunks:
        t = torch.tensor(toks[i:i + c][None].astype(np.int32), device=dev())
        outs.append(sv.ss_verify_forward(gm, gkv, t, c)[0].cpu().numpy())
        i += c
    return np.concatenate(outs)


@pytest.mark.parametrize("shape", [si.TINY_TARGET, si.TINY_DRAFT,
                                   si.DecoderShape(2, 64, 2, 32, 96, 50, rope_base=500.0, rms_eps=1e-6, dtype="f32"),
                                   si.DecoderShape(2, 256, 2, 128, 344, 300, dtype="f32")])
@pytest.mark.parametrize("persistent", PATHS)
def test_fp32_verify_logits_match_oracle(shape, persistent):
    om, gm, _ = model_pair(shape, seed=3, persistent=persistent)
    toks = si.token_ids(3, "toks", (70,), shape.vocab).numpy()
    chunks = [16, 16, 1, 5, 5, 2, 9, 16]            # prefill chunks, single rows, K+1-row verify passes
    gkv = sv.KVCache(gm, 1, 100)
    got = _gpu_forward_chunks(gm, gkv, toks, chunks)
    ref = om.forward(om.new_kv(100), toks)
    assert maxabs(got, ref) < tol(shape)
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [70]
    assert sv.ss_device_status(gm) == 0


@pytest.mark.parametrize("shape", [si.DecoderShape(2, 128, 2, 64, 344, 512, dtype="bf16"),
                                   si.DecoderShape(2, 128, 2, 64, 4608, 512, dtype="bf16"),   # down projection: K spans two LDS slabs
                                   si.DecoderShape(1, 512, 4, 128, 1376, 1000, dtype="bf16"),
                                   si.DecoderShape(3, 256, 8, 32, 688, 333, dtype="bf16")])
@pytest.mark.parametrize("persistent", PATHS)
def test_bf16_verify_logits_match_oracle(shape, persistent):
    om, gm, _ = model_pair(shape, seed=4, persistent=persistent)
    toks = si.token_ids(4, "toks", (150,), shape.vocab).numpy()
    chunks = [16] * 8 + [5, 1, 9, 7]                # crosses the 64- and 128-position cache blocks
    gkv = sv.KVCache(gm, 1, 160)
    got = _gpu_forward_chunks(gm, gkv, toks, chunks)
    ref = om.forward(om.new_kv(160), toks)
    assert maxabs(got, ref) < tol(shape)
    # the bf16 path keeps fp32 activations (hi + lo split), so it is in fact far inside the bar
    assert maxabs(got, ref) < 2e-3


@pytest.mark.parametrize("kind,shape", [
    ("f32", si.DecoderShape(2, 256, 4, 64, 344, 333, dtype="f32")),      # K = 344: the last 128-byte step ends inside
    ("bf16", si.DecoderShape(2, 256, 4, 64, 688, 333, dtype="bf16")),    # K = 688 likewise; 333 columns: a ragged last tile
    ("int8", si.DecoderShape(2, 256, 4, 64, 688, 333, dtype="bf16")),    # K = 688: a ragged last 128-entry step
    ("int4", si.DecoderShape(2, 256, 4, 64, 640, 333, dtype="bf16"))])   # K = 640: a last step of one scale group
def test_every_row_count_of_the_kernels_for_at_most_16_rows_matches_oracle(kind, shape):
    """Calls of 1, 2, ... 16 rows one after the other on the per-phase path (both sizes of the kernels' LDS staging,
    every number of load-to-LDS instructions per step), all logits against one oracle pass over the same tokens."""
    w = si.decoder_weights(shape, 17)
    kw = {"int8": {"int8_weights": True}, "int4": {"int4_weights": True}}.get(kind, {})
    om = oracle.Model(shape, w, **kw)
    gm = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=256, **kw)
    set_path(gm, False)
    chunks = list(range(1, 17))
    toks = si.token_ids(17, "toks", (sum(chunks),), shape.vocab).numpy()
    gkv = sv.KVCache(gm, 1, 160)
    got = _gpu_forward_chunks(gm, gkv, toks, chunks)
    ref = om.forward(om.new_kv(160), toks)
    assert maxabs(got, ref) < (tol(shape) if kind in ("f32", "bf16") else 2e-2)
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [sum(chunks)]
    assert sv.ss_device_status(gm) == 0


@pytest.mark.parametrize("persistent", PATHS)
def test_rollback_then_reverify_matches_oracle(persistent):
    """Rejected rows are dropped by a length write and overwritten by the next pass (Section 4.4)."""
    shape = si.TINY_TARGET
    om, gm, _ = model_pair(shape, seed=5, persistent=persistent)
    toks = si.token_ids(5, "toks", (40,), shape.vocab).numpy()
    gkv = sv.KVCache(gm, 1, 64)
    _gpu_forward_chunks(gm, gkv, toks[:20], [16, 4])
    junk = torch.tensor([[7, 8, 9, 10, 11]], dtype=torch.int32, device=dev())
    sv.ss_verify_forward(gm, gkv, junk, 5)
    na = torch.tensor([1], dtype=torch.int32, device=dev())          # keep x_n and one draft token
    sv.ss_kv_cache_rollback(gkv, na, 5, n_accepted_host=[1])
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [22]
    sv.ss_kv_cache_set_len(gkv, [20])                                # and drop those two as well
    got = _gpu_forward_chunks(gm, gkv, toks[20:], [5, 15])
    okv = om.new_kv(64)
    om.forward(okv, toks[:20], want_logits=False)
    ref = om.forward(okv, toks[20:])
    assert maxabs(got, ref) < tol(shape)


@pytest.mark.parametrize("B,M,persistent", [(3, 9, False), (3, 5, True), (3, 5, False), (5, 9, False), (8, 9, False),
                                            (3, 3, True), (1, 9, True), (4, 4, True), (3, 3, "grid8"), (1, 9, "grid8"), (4, 4, "grid8")])   # 9 and 16 rows: the persistent kernel's largest calls (bf16 / fp32)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_batched_ragged_lengths_match_per_sequence_oracle(dtype, B, M, persistent):
    """Several sequences with different context lengths verified in one call (up to 72 rows: every
    row-tile variant of the GEMMs); each must equal the oracle run on that sequence alone.  Contexts
    are built with the raw append."""
    shape = si.DecoderShape(2, 128, 2, 64, 344, 512, dtype=dtype)
    w = si.decoder_weights(shape, seed=6)
    om = oracle.Model(shape, w)
    gm = sv.Model(shape, weights_to_device(w), max_rows=80, max_pos=512)
    set_path(gm, persistent)
    lens = [70, 3, 129, 40, 1, 100, 64, 17][:B]
    gkv = sv.KVCache(gm, B, 200)
    toks = si.token_ids(6, "toks", (B, M), shape.vocab)
    refs = []
    for b in range(B):
        ctx = si.kv_context(shape, 6, f"ctx{b}", lens[b])
        for l, (k, v) in enumerate(ctx):
            sv.ss_kv_cache_append(gkv, l, b, 0, k.to(dev()), v.to(dev()))
        okv = om.new_kv(200)
        okv.append_raw(ctx)
        refs.append(om.forward(okv, toks[b].numpy()))
    sv.ss_kv_cache_set_len(gkv, lens)
    got = sv.ss_verify_forward(gm, gkv, toks.to(dev()), M).cpu().numpy()
    for b in range(B):
        assert maxabs(got[b], refs[b]) < tol(shape), b
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [l + M for l in lens]
    # ragged roll-back: different accept counts per sequence
    acc = [min(a, M - 1) for a in [0, M - 1, 3, M - 1, 0, 1, 2, 4][:B]]
    na = torch.tensor(acc, dtype=torch.int32, device=dev())
    sv.ss_kv_cache_rollback(gkv, na, M)
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [l + a + 1 for l, a in zip(lens, acc)]


@pytest.mark.parametrize("persistent", PATHS)
def test_single_7b_layer_verify_matches_oracle(persistent):
    """One 7B-shaped bf16 layer, 5 query rows against 1024 cached positions (the microbench shape):
    hidden rows out of the layer vs the oracle, max-abs 2e-2."""
    shape = si.LAYER_7B
    lw = si.layer_weights(shape, seed=0, layer=0)
    w = {"embed": None, "gf": None, "lm_head": None, "layers": [lw]}
    om = oracle.Model(shape, w)
    gm = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=2048)
    set_path(gm, persistent)
    L, M = 1024, 5
    ctx = si.kv_context(shape, 0, "ctx", L)
    gkv = sv.KVCache(gm, 1, L + 64)
    sv.ss_kv_cache_append(gkv, 0, 0, 0, ctx[0][0].to(dev()), ctx[0][1].to(dev()))
    sv.ss_kv_cache_set_len(gkv, [L])
    okv = om.new_kv(L + 64)
    okv.append_raw(ctx)
    h = si.normal(0, "h", (M, shape.d_model), 1.0)
    got = sv.ss_decoder_layers_forward(gm, gkv, h.to(dev()).clone(), 1, M).cpu().numpy()
    ref = om.layers_forward(okv, h.numpy())
    assert maxabs(got, ref) < 2e-2
    assert maxabs(got, ref) < 1e-3


@pytest.mark.parametrize("dtype,M,ctx", [("bf16", 5, 40), ("bf16", 9, 40), ("f32", 16, 40), ("bf16", 5, 456)])   # 456: split-KV attention with its merge
def test_persistent_kernel_is_deterministic_and_independent_of_its_synchronisation(dtype, M, ctx):
    """The same call three ways: barriers at every phase boundary, self-validating activations, and the
    latter once more.  The arithmetic does not depend on how the phases are ordered in time, so the
    logits agree bit for bit (a stale or half-written activation would show up here)."""
    shape = si.DecoderShape(3, 256, 4, 64, 688, 1000, dtype=dtype)
    w = weights_to_device(si.decoder_weights(shape, seed=12))
    toks = si.token_ids(12, "toks", (ctx + M,), shape.vocab).numpy().astype(np.int32)
    outs = []
    for data_sync in (False, True, True):
        gm = sv.Model(shape, w, max_rows=16, max_pos=512)
        sv.ss_model_set_persistent(gm, True)
        sv.ss_model_set_persistent_options(gm, 8, data_sync)
        gkv = sv.KVCache(gm, 1, 512)
        _gpu_forward_chunks(gm, gkv, toks[:ctx], [16] * (ctx // 16) + [ctx % 16] * (ctx % 16 > 0))
        outs.append(sv.ss_verify_forward(gm, gkv, torch.tensor(toks[None, ctx:], device=dev()), M).clone())
        assert sv.ss_device_status(gm) == 0
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[1], outs[2])


def test_7b_width_data_synchronisation_equals_barriers_over_many_launches():
    """Three 7B-shaped layers + LM head on the default grid (one workgroup per compute unit, where the
    self-validating protocol is what runs): 200 launches with the row count changing from call to call
    (1, 5, 9, 2, ... rows: the buffers keep rows of earlier, larger calls), context growing and rolled
    back.  Every launch must give the logits of the barrier-only mode bit for bit."""
    shape, packed, io = si.packed_7b(5, 3, dev())
    ms = []
    for data_sync in (False, True):
        gm = sv.Model(shape, io, max_rows=16, max_pos=1024, packed_layers=packed)
        sv.ss_model_set_persistent_options(gm, 0, data_sync)
        ms.append((gm, sv.KVCache(gm, 1, 1024)))
    toks = si.token_ids(5, "many", (200, 9), shape.vocab).to(dev()).int()
    rows = [1, 5, 9, 2, 9, 1, 4, 8, 3, 5]
    for it in range(200):
        M = rows[it % len(rows)]
        t = toks[it:it + 1, :M].contiguous()
        a = sv.ss_verify_forward(ms[0][0], ms[0][1], t, M)
        b = sv.ss_verify_forward(ms[1][0], ms[1][1], t, M)
        assert torch.equal(a, b), it
        if it % 7 == 6:   # reject most of the rows of this call, as the rejection step would
            for gm, kv in ms:
                sv.ss_kv_cache_rollback(kv, torch.zeros(1, dtype=torch.int32, device=dev()), M, n_accepted_host=[0])
        if it % 50 == 49:  # and start over on a short context now and then
            for gm, kv in ms:
                sv.ss_kv_cache_set_len(kv, [33])
    assert sv.ss_device_status(ms[0][0]) == 0 and sv.ss_device_status(ms[1][0]) == 0
    assert sv.ss_kv_cache_get_len(ms[0][1]).tolist() == sv.ss_kv_cache_get_len(ms[1][1]).tolist()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("quant", [None, "int8", "int4"])
def test_batched_7b_layer_72_rows_matches_per_sequence_oracle(quant):
    """The batched workload's launch shapes at full width: one 7B-shaped bf16 layer, 8 sequences with
    ragged contexts, K = 8 -> 72 rows in one call (wide GEMMs with split-K, split-KV attention), with bf16
    matrices and with the int8 and int4 matrices the library quantises from them (the wide kernel's two
    quantised modes at K = 4096 and 11008).  Each sequence's hidden rows against the oracle's model of the
    same kind run on that sequence alone (reduced depth and context: the full 32-layer, 4096-position pass
    is out of the oracle's reach)."""
    shape = si.LAYER_7B
    lw = si.layer_weights(shape, seed=0, layer=0)
    w = {"embed": None, "gf": None, "lm_head": None, "layers": [lw]}
    qkw = {} if quant is None else {f"{quant}_weights": True}
    om = oracle.Model(shape, w, **qkw)
    B, M = 8, 9
    lens = [300, 17, 129, 64, 1, 255, 190, 77]
    gm = sv.Model(shape, weights_to_device(w), max_rows=B * M, max_pos=512, **qkw)
    gkv = sv.KVCache(gm, B, 384)
    h = si.normal(9, "h72", (B, M, shape.d_model), 1.0)
    refs = []
    for b in range(B):
        ctx = si.kv_context(shape, 9, f"ctx72_{b}", lens[b])
        sv.ss_kv_cache_append(gkv, 0, b, 0, ctx[0][0].to(dev()), ctx[0][1].to(dev()))
        okv = om.new_kv(384)
        okv.append_raw(ctx)
        refs.append(om.layers_forward(okv, h[b].numpy()))
    sv.ss_kv_cache_set_len(gkv, lens)
    got = sv.ss_decoder_layers_forward(gm, gkv, h.reshape(B * M, -1).to(dev()).clone(), B, M).cpu().numpy().reshape(B, M, -1)
    for b in range(B):
        assert maxabs(got[b], refs[b]) < 2e-2, b
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [l + M for l in lens]


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("B", [8, 2])
def test_batched_long_context_layer_at_its_real_shape_matches_per_sequence_oracle(B):
    """The batched long-context workload at its real shape, reduced in depth only (the oracle cannot run 32 layers
    of it): one 7B-shaped bf16 layer, 8 sequences whose caches hold 4096 - jitter(0..63) positions (Section 2: the
    cache of a long context is a large object), K = 8 -> 72 rows in one call against a cache of 4608 positions per
    sequence: block indices far past the first cache blocks, the transposed value blocks of a long sequence,
    one workgroup per (sequence, head) walking the whole context, split-K wide GEMMs.  With 2 sequences (18 rows:
    two row tiles) the same contexts go through 8-way split-KV attention with a partly empty tail split and the
    merge launch.  Every sequence's hidden rows against the oracle run on that sequence alone; then a ragged
    roll-back (Section 4.4: sequences accept different numbers of tokens) and a second pass over the shortened
    caches, checked the same way."""
    shape = si.LAYER_7B
    lw = si.layer_weights(shape, seed=0, layer=0)
    w = {"embed": None, "gf": None, "lm_head": None, "layers": [lw]}
    om = oracle.Model(shape, w)
    M, S = 9, 4608
    lens = [4096 - j for j in [0, 63, 1, 37, 50, 12, 31, 64 - 41]][:B]
    assert len(set(lens)) == B and min(lens) > 4096 - 64
    gm = sv.Model(shape, weights_to_device(w), max_rows=B * M, max_pos=S)
    gkv = sv.KVCache(gm, B, S)
    h = si.normal(21, "h72", (2, B, M, shape.d_model), 1.0)
    okvs = []
    for b in range(B):
        ctx = si.kv_context(shape, 21, f"ctx4096_{b}", lens[b])
        sv.ss_kv_cache_append(gkv, 0, b, 0, ctx[0][0].to(dev()), ctx[0][1].to(dev()))
        okv = om.new_kv(S)
        okv.append_raw(ctx)
        okvs.append(okv)
        del ctx
    sv.ss_kv_cache_set_len(gkv, lens)
    got = sv.ss_decoder_layers_forward(gm, gkv, h[0].reshape(B * M, -1).to(dev()).clone(), B, M).cpu().numpy().reshape(B, M, -1)
    worst = 0.0
    for b in range(B):
        err = maxabs(got[b], om.layers_forward(okvs[b], h[0, b].numpy()))
        worst = max(worst, err)
        assert err < 2e-2, (b, err)
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [l + M for l in lens]
    # ragged roll-back, then the next pass
    acc = [0, 8, 3, 8, 1, 5, 2, 7][:B]
    sv.ss_kv_cache_rollback(gkv, torch.tensor(acc, dtype=torch.int32, device=dev()), M, n_accepted_host=acc)
    lens2 = [l + a + 1 for l, a in zip(lens, acc)]
    assert sv.ss_kv_cache_get_len(gkv).tolist() == lens2
    got = sv.ss_decoder_layers_forward(gm, gkv, h[1].reshape(B * M, -1).to(dev()).clone(), B, M).cpu().numpy().reshape(B, M, -1)
    for b in range(B):
        okvs[b].set_len(lens2[b])
        err = maxabs(got[b], om.layers_forward(okvs[b], h[1, b].numpy()))
        worst = max(worst, err)
        assert err < 2e-2, (b, err)
    assert worst < 2e-3          # the bf16 path keeps fp32 activations: far inside the bar
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [l + M for l in lens2]
    assert sv.ss_device_status(gm) == 0


@pytest.mark.timeout(1200)
def test_persistent_kernel_at_7b_width_for_every_row_count_and_a_long_context_matches_oracle():
    """The persistent kernel on its default grid (one workgroup per compute unit, self-validating activations)
    at 7B width, three layers + LM head, against the ORACLE (not against its own barrier mode): 1 row (the
    autoregressive baseline and every draft step, Section 3 Eq. 1), 3 rows (K = 2), 5 and 9 rows (K = 4, 8), each
    against 140 cached positions (one attention unit per head) and against about 4000 (eight KV splits merged
    inside the kernel)."""
    shape, packed, io = si.packed_7b(5, 3, dev())
    gm = sv.Model(shape, io, max_rows=16, max_pos=4096, packed_layers=packed)
    sv.ss_model_set_persistent(gm, True)
    om = oracle.Model(shape, {"embed": io["embed"].cpu(), "gf": io["gf"].cpu(), "lm_head": io["lm_head"].cpu(),
                              "layers": si.unpack_layers(shape, packed)})
    Lbig = 4003
    ctx = si.kv_context(shape, 22, "ctx_long", Lbig)
    gkv = sv.KVCache(gm, 1, 4096)
    dctx = [(k.to(dev()), v.to(dev())) for k, v in ctx]
    worst = 0.0
    for L, M in [(Lbig, 9), (Lbig, 1), (3990, 5), (140, 1), (140, 3), (140, 9), (385, 5)]:   # 385: the shortest context that is split
        for l, (k, v) in enumerate(dctx):                     # the previous case overwrote rows of the context
            sv.ss_kv_cache_append(gkv, l, 0, 0, k[:L].contiguous(), v[:L].contiguous())
        sv.ss_kv_cache_set_len(gkv, [L])
        okv = om.new_kv(L + 16)
        okv.append_raw([(k[:L], v[:L]) for k, v in ctx])
        toks = si.token_ids(22, f"rows{L}_{M}", (M,), shape.vocab).numpy().astype(np.int32)
        got = sv.ss_verify_forward(gm, gkv, torch.tensor(toks[None], device=dev()), M)[0].cpu().numpy()
        ref = om.forward(okv, toks)
        err = maxabs(got, ref)
        print(f"context {L}, {M} rows: max |logits - oracle| = {err:.2e}", flush=True)
        worst = max(worst, err)
        assert err < 2e-2, (L, M, err)
        assert sv.ss_kv_cache_get_len(gkv).tolist() == [L + M]
    assert worst < 2e-3
    assert sv.ss_device_status(gm) == 0


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("quant", [None, "persistent", "int8", "int4"])
def test_full_7b_verify_pass_matches_oracle(quant):
    """The benchmark workload at its full size and in the launch configurations bench.py times (32
    7B-shaped bf16 layers + LM head, 5 query rows, 128 cached positions; the default forward path with one
    launch per phase, and the persistent kernel): every logit of the verify pass against the oracle, max-abs
    2e-2; the greedy token of a row must agree wherever the oracle's top-2 margin exceeds twice that
    tolerance.  Also with the matrices quantised to int8 and to int4 (the bench's int8_weights /
    int4_weights legs), against the oracle's model quantised the same way."""
    qkw = {} if quant in (None, "persistent") else {f"{quant}_weights": True}
    shape, packed, io = si.packed_7b(0, si.FULL_7B.n_layers, dev())
    gm = sv.Model(shape, io, max_rows=16, max_pos=512, packed_layers=packed, **qkw)
    if quant == "persistent":
        sv.ss_model_set_persistent(gm, True)
    om = oracle.Model(shape, {"embed": io["embed"].cpu(), "gf": io["gf"].cpu(), "lm_head": io["lm_head"].cpu(),
                              "layers": si.unpack_layers(shape, packed)}, **qkw)
    L, M = 128, 5
    ctx = si.kv_context(shape, 3, "ctx7b", L)
    gkv = sv.KVCache(gm, 1, L + 64)
    for l, (k, v) in enumerate(ctx):
        sv.ss_kv_cache_append(gkv, l, 0, 0, k.to(dev()), v.to(dev()))
    sv.ss_kv_cache_set_len(gkv, [L])
    okv = om.new_kv(L + 64)
    okv.append_raw(ctx)
    toks = si.token_ids(3, "verify7b", (M,), shape.vocab).numpy().astype(np.int32)
    got = sv.ss_verify_forward(gm, gkv, torch.tensor(toks[None], device=dev()), M)[0].cpu().numpy()
    ref = om.forward(okv, toks)
    assert got.shape == ref.shape == (M, shape.vocab)
    assert maxabs(got, ref) < 2e-2
    top2 = np.sort(ref, axis=1)[:, -2:]
    clear = (top2[:, 1] - top2[:, 0]) > 4e-2
    assert (got.argmax(1)[clear] == ref.argmax(1)[clear]).all()
    assert sv.ss_kv_cache_get_len(gkv).tolist() == [L + M]


def test_capacity_and_shape_errors_come_from_the_host():
    shape = si.TINY_DRAFT
    _, gm, _ = model_pair(shape, seed=7, max_rows=8)
    gkv = sv.KVCache(gm, 1, 10)
    t = torch.zeros((1, 8), dtype=torch.int32, device=dev())
    sv.ss_verify_forward(gm, gkv, t, 8, logits=False)
    with pytest.raises(sv.SpecVerifyError) as e:
        sv.ss_verify_forward(gm, gkv, t, 8, logits=False)           # 8 + 8 > 10
    assert e.value.code == sv.SS_ECAPACITY
    with pytest.raises(sv.SpecVerifyError) as e:
        sv.ss_verify_forward(gm, sv.KVCache(gm, 2, 10), torch.zeros((2, 8), dtype=torch.int32, device=dev()), 8)
    assert e.value.code == sv.SS_EINVAL                              # 16 rows > max_rows 8
    bad = torch.full((1, 1), shape.vocab + 5, dtype=torch.int32, device=dev())
    sv.ss_verify_forward(gm, gkv, bad, 1, logits=False)
    assert sv.ss_device_status(gm) == 1 and sv.ss_device_status(gm) == 0   # clamped, flagged, cleared


def test_read_stream_probe_reports_a_plausible_rate():
    """The probe reads a 1 GiB buffer (never written: the contents are checked afterwards) at a rate between
    a tenth of and the whole nominal HBM peak; bad arguments are refused on the host."""
    buf = torch.full((1 << 28,), 3.0, dtype=torch.float32, device=dev())
    rate = sv.ss_probe_read_bandwidth(buf, iters=5)
    assert 800.0 < rate < 8000.0
    assert float(buf[::4097].min()) == 3.0 and float(buf[-1]) == 3.0
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_probe_read_bandwidth(buf[:1024])
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_probe_read_bandwidth(buf, iters=0)


@pytest.mark.parametrize("persistent", [False, True])
@pytest.mark.parametrize("d,H,F", [(5120, 40, 13824), (3072, 24, 8192)])
def test_single_layer_of_13b_and_3b_width_matches_oracle(d, H, F, persistent):
    """One bf16 layer at the widths of a 13B-shaped target and a 3B-shaped draft (the size ratio of the
    paper's Section 6 experiment), K = 5 (6 query rows) against 200 cached positions: weight rows of 10 KB
    and 27 KB (at d_model 5120 the persistent kernel takes its 12 KB slabs: one and three slab trips; at 3072
    its 8 KB slabs), 20 and 12 output rows per workgroup."""
    shape = si.DecoderShape(1, d, H, 128, F, 32000, dtype="bf16")
    lw = si.layer_weights(shape, seed=3, layer=0)
    w = {"embed": None, "gf": None, "lm_head": None, "layers": [lw]}
    om = oracle.Model(shape, w)
    gm = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=512)
    set_path(gm, persistent)
    L, M = 200, 6
    ctx = si.kv_context(shape, 3, "ctx", L)
    gkv = sv.KVCache(gm, 1, L + 64)
    sv.ss_kv_cache_append(gkv, 0, 0, 0, ctx[0][0].to(dev()), ctx[0][1].to(dev()))
    sv.ss_kv_cache_set_len(gkv, [L])
    okv = om.new_kv(L + 64)
    okv.append_raw(ctx)
    h = si.normal(3, "h", (M, shape.d_model), 1.0)
    got = sv.ss_decoder_layers_forward(gm, gkv, h.to(dev()).clone(), 1, M).cpu().numpy()
    ref = om.layers_forward(okv, h.numpy())
    assert maxabs(got, ref) < 2e-2
    assert maxabs(got, ref) < 2e-3
    assert sv.ss_device_status(gm) == 0


@pytest.mark.parametrize("M", [1, 3, 6, 7, 9])
def test_persistent_kernel_at_13b_width_with_either_slab_size_matches_oracle(M):
    """Two bf16 layers at d_model 5120 on the persistent kernel: up to 6 rows fit its 12 KB activation slabs (a
    weight row of 10 KB in one slab), 7 and 9 rows fall back to 8 KB slabs (two slab groups per tile, reloaded for
    every tile of a workgroup's share); both against the oracle, twice in a row on the same model."""
    shape = si.DecoderShape(2, 5120, 40, 128, 13824, 32000, dtype="bf16")
    w = {"embed": None, "gf": None, "lm_head": None, "layers": [si.layer_weights(shape, seed=4, layer=l) for l in range(2)]}
    om = oracle.Model(shape, w)
    gm = sv.Model(shape, weights_to_device(w), max_rows=16, max_pos=512)
    set_path(gm, True)
    L = 150
    ctx = si.kv_context(shape, 4, "ctx", L)
    gkv = sv.KVCache(gm, 1, L + 64)
    for l in range(2):
        sv.ss_kv_cache_append(gkv, l, 0, 0, ctx[l][0].to(dev()), ctx[l][1].to(dev()))
    okv = om.new_kv(L + 64)
    okv.append_raw(ctx)
    h = si.normal(4, f"h{M}", (M, shape.d_model), 1.0)
    ref = om.layers_forward(okv, h.numpy())
    for _ in range(2):
        sv.ss_kv_cache_set_len(gkv, [L])
        got = sv.ss_decoder_layers_forward(gm, gkv, h.to(dev()).clone(), 1, M).cpu().numpy()
        assert maxabs(got, ref) < 2e-2, M               # the stated bf16 bar; hidden rows reach |h| of about 10 after two layers
        assert maxabs(got, ref) < 1e-3 * float(np.abs(ref).max()), M
    assert sv.ss_device_status(gm) == 0


@pytest.mark.parametrize("path", [True, "grid8"])
def test_a_wait_that_gives_up_is_reported_and_the_model_recovers(path):
    """Every wait of the persistent kernel is bounded.  With the bound set to a single poll the kernel gives
    up at its first unsatisfied wait (and still ends normally); the status word says so, the synchronisation
    state is reset, and the same model then reproduces its earlier result bit for bit."""
    shape = si.DecoderShape(3, 256, 4, 64, 688, 1000, dtype="bf16")
    gm = sv.Model(shape, weights_to_device(si.decoder_weights(shape, seed=12)), max_rows=16, max_pos=256)
    set_path(gm, path)
    toks = si.token_ids(12, "toks", (25,), shape.vocab).numpy().astype(np.int32)
    kv = sv.KVCache(gm, 1, 128)
    _gpu_forward_chunks(gm, kv, toks[:20], [16, 4])
    rows = torch.tensor(toks[None, 20:], device=dev())
    ref = sv.ss_verify_forward(gm, kv, rows, 5).clone()
    assert sv.ss_device_status(gm) == 0
    sv.ss_model_set_wait_limit(gm, 1)
    sv.ss_kv_cache_set_len(kv, [20])
    sv.ss_verify_forward(gm, kv, rows, 5)             # enqueues; the kernel leaves early
    assert sv.ss_device_status(gm) & 2                # ... and says so; the call's results are not used
    sv.ss_model_set_wait_limit(gm, 1 << 20)
    sv.ss_kv_cache_set_len(kv, [20])
    again = sv.ss_verify_forward(gm, kv, rows, 5)
    assert sv.ss_device_status(gm) == 0
    assert torch.equal(again, ref)
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_model_set_wait_limit(gm, 0)
