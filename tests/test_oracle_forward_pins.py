"""Pins for the oracle's decoder forward: library routines, closed forms and invariants.

The paper prints no numbers for this path, so absolute logits are pinned against an independent
library implementation of the same architecture (the Llama decoder of HF transformers, evaluated
in fp64 on the CPU) and against what KV caching must preserve (Sections 2 and 4.2: caching changes
no result).
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

import oracle
import seeded_inputs as si


# ---------------------------------------------------------------- small pieces

def test_bf16_rounding_matches_library_and_ties_to_even():
    x = si.normal(1, "bf", (4096,), 3.0)
    ours = np.array([oracle.lib().orc_f32_to_bf16(float(v)) for v in x.numpy()], dtype=np.uint16)
    ref = x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    # exact ties: 1 + 2^-8 is halfway between bf16(1.0) and the next value -> even mantissa (1.0)
    assert oracle.lib().orc_f32_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    # 1 + 3*2^-8 is halfway between 0x3F81 and 0x3F82 -> even (0x3F82)
    assert oracle.lib().orc_f32_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    assert oracle.lib().orc_bf16_to_f32(0x3FC0) == 1.5


def test_rmsnorm_closed_form_and_library():
    # hand value: x = (3, 4), eps = 0 -> rms = sqrt(12.5)
    out = oracle.rmsnorm([3.0, 4.0], [1.0, 2.0], eps=0.0)
    r = math.sqrt(12.5)
    assert np.allclose(out, [3 / r, 8 / r], rtol=1e-7)
    x = si.normal(2, "x", (512,), 1.7).numpy()
    g = si.normal(2, "g", (512,), 0.02, mean=1.0).numpy()
    ref = torch.nn.functional.rms_norm(torch.tensor(x, dtype=torch.float64), (512,),
                                       torch.tensor(g, dtype=torch.float64), eps=1e-5).numpy()
    assert np.max(np.abs(oracle.rmsnorm(x, g, 1e-5) - ref)) < 1e-6
    # invariants: unit gains -> unit RMS; scale invariance (eps negligible)
    y = oracle.rmsnorm(x, np.ones(512, np.float32), 1e-12)
    assert abs(np.sqrt(np.mean(y.astype(np.float64) ** 2)) - 1.0) < 1e-6
    assert np.allclose(oracle.rmsnorm(8 * x, g, 1e-12), oracle.rmsnorm(x, g, 1e-12), rtol=1e-6)


def test_linear_against_library_matmul_both_storage_types():
    W = si.normal(3, "W", (37, 96), 0.5)
    x = si.normal(3, "x", (96,), 1.0).numpy()
    ref = W.double().numpy() @ x.astype(np.float64)
    assert np.max(np.abs(oracle.linear(W, x) - ref)) < 1e-5
    Wb = W.to(torch.bfloat16)
    refb = Wb.double().numpy() @ x.astype(np.float64)
    assert np.max(np.abs(oracle.linear(Wb, x, is_bf16=True) - refb)) < 1e-5
    # not transposed: a one-hot input picks a column of W
    e = np.zeros(96, np.float32)
    e[5] = 1.0
    assert np.array_equal(oracle.linear(W, e), W[:, 5].numpy())


def test_softmax_against_library_and_invariants():
    l = si.normal(4, "l", (3, 1000), 2.0).numpy()
    for T in (1.0, 0.8, 2.5):
        ref = scipy.special.softmax(l.astype(np.float64) / T, axis=-1)
        out = oracle.softmax(l, T)
        assert np.max(np.abs(out - ref)) < 1e-7
        assert np.allclose(out.astype(np.float64).sum(-1), 1.0, atol=1e-5)
    # shift invariance, and a closed form: two equal logits -> 1/2 each
    assert np.allclose(oracle.softmax(l[0] + 7.0), oracle.softmax(l[0]), rtol=1e-5, atol=1e-9)
    assert np.array_equal(oracle.softmax([5.0, 5.0]), np.float32([0.5, 0.5]))
    assert np.allclose(oracle.softmax([0.0, math.log(3.0)]), [0.25, 0.75], rtol=1e-6)


def test_rope_closed_forms_and_relative_position_property():
    hd = 64
    v = si.normal(5, "v", (hd,), 1.0).numpy()
    assert np.array_equal(oracle.rope(v, 0), v)                       # position 0 is the identity
    e0 = np.zeros(hd, np.float32)
    e0[0] = 1.0                                                       # pair j=0 turns by pos radians
    r = oracle.rope(e0, 3)
    assert abs(r[0] - math.cos(3.0)) < 1e-7 and abs(r[hd // 2] - math.sin(3.0)) < 1e-7
    assert np.count_nonzero(r) == 2
    ej = np.zeros(hd, np.float32)
    ej[hd // 2 + 16] = 1.0                                            # pair j=16: angle pos*base^(-32/64)
    r = oracle.rope(ej, 50, base=10000.0)
    ang = 50 * 10000.0 ** (-0.5)
    assert abs(r[16] + math.sin(ang)) < 1e-7 and abs(r[hd // 2 + 16] - math.cos(ang)) < 1e-7
    assert abs(np.linalg.norm(oracle.rope(v, 4097).astype(np.float64)) - np.linalg.norm(v.astype(np.float64))) < 1e-5
    # q_m . k_n depends on m - n only
    k = si.normal(5, "k", (hd,), 1.0).numpy()
    d1 = float(oracle.rope(v, 9).astype(np.float64) @ oracle.rope(k, 4).astype(np.float64))
    d2 = float(oracle.rope(v, 1005).astype(np.float64) @ oracle.rope(k, 1000).astype(np.float64))
    assert abs(d1 - d2) < 1e-4


# ---------------------------------------------------------------- whole decoder vs a library Llama

def _hf_llama(shape, w, attn="eager"):
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(hidden_size=shape.d_model, intermediate_size=shape.d_ff,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
                      num_key_value_heads=shape.n_heads, head_dim=shape.head_dim, vocab_size=shape.vocab,
                      rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_base, tie_word_embeddings=False,
                      attention_bias=False, mlp_bias=False, max_position_embeddings=4096,
                      attn_implementation=attn)
    m = LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "model.norm.weight": w["gf"], "lm_head.weight": w["lm_head"]}
    for l, lw in enumerate(w["layers"]):
        p = f"model.layers.{l}."
        sd.update({p + "self_attn.q_proj.weight": lw["wq"], p + "self_attn.k_proj.weight": lw["wk"],
                   p + "self_attn.v_proj.weight": lw["wv"], p + "self_attn.o_proj.weight": lw["wo"],
                   p + "mlp.gate_proj.weight": lw["wg"], p + "mlp.up_proj.weight": lw["wu"],
                   p + "mlp.down_proj.weight": lw["wd"], p + "input_layernorm.weight": lw["g1"],
                   p + "post_attention_layernorm.weight": lw["g2"]})
    missing, unexpected = m.load_state_dict({k: v.double() for k, v in sd.items()}, strict=False)
    assert not [k for k in missing if "rotary" not in k] and not unexpected
    return m


@pytest.mark.parametrize("shape", [si.TINY_TARGET, si.TINY_DRAFT,
                                   si.DecoderShape(2, 64, 2, 32, 96, 50, rope_base=500.0, rms_eps=1e-6, dtype="f32")])
def test_forward_matches_library_llama_fp64(shape):
    w = si.decoder_weights(shape, seed=11)
    toks = si.token_ids(11, "toks", (40,), shape.vocab).numpy()
    with torch.no_grad():
        ref = _hf_llama(shape, w)(torch.tensor(toks[None].astype(np.int64))).logits[0].numpy()
    m = oracle.Model(shape, w)
    # prefill 33 rows, then a 5-row verify pass, then two single rows: all against the cache
    kv = m.new_kv(64)
    got = np.concatenate([m.forward(kv, toks[:33]), m.forward(kv, toks[33:38]),
                          m.forward(kv, toks[38:39]), m.forward(kv, toks[39:40])])
    assert len(kv) == 40
    assert np.max(np.abs(got - ref)) < 2e-6


def test_bf16_storage_rounds_only_weights_and_cache():
    """bf16 storage rounds (to nearest even) the weights and the cache entries, nothing else.  Reference: the
    library Llama in fp64 over the same bf16 weights, with an attention function that rounds the keys (after the
    rotary embedding) and the values to bf16, as a cache in that storage type holds them, before they are used.
    A further rounding anywhere in the oracle (of the queries, of the hidden rows, of an attention output)
    would show as an error of 1e-3, two orders above the bound."""
    from transformers import AttentionInterface
    from transformers.masking_utils import AttentionMaskInterface, eager_mask
    from transformers.models.llama.modeling_llama import eager_attention_forward

    def attention_over_bf16_cache(module, query, key, value, attention_mask, **kw):
        rnd = lambda t: t.float().to(torch.bfloat16).double()   # one rounding to fp32, then the storage rounding
        return eager_attention_forward(module, query, rnd(key), rnd(value), attention_mask, **kw)

    AttentionInterface.register("eager_bf16_cache", attention_over_bf16_cache)
    AttentionMaskInterface.register("eager_bf16_cache", eager_mask)     # the same additive causal mask as "eager"
    shape = si.DecoderShape(2, 128, 2, 64, 344, 512, dtype="bf16")
    w = si.decoder_weights(shape, seed=12)
    toks = si.token_ids(12, "toks", (24,), shape.vocab).numpy()
    m = oracle.Model(shape, w)
    got = np.concatenate([m.forward(kv := m.new_kv(32), toks[:19]), m.forward(kv, toks[19:])])   # prefill + a 5-row verify pass
    ids = torch.tensor(toks[None].astype(np.int64))
    with torch.no_grad():
        ref = _hf_llama(shape, w, attn="eager_bf16_cache")(ids).logits[0].numpy()
        unrounded = _hf_llama(shape, w)(ids).logits[0].numpy()
    assert np.max(np.abs(got - ref)) < 1e-6     # measured 1.1e-7
    # and the cache rounding is really there: against a cache that keeps fp64 keys and values the gap is far larger
    assert 1e-4 < np.max(np.abs(got - unrounded)) < 5e-3


# ---------------------------------------------------------------- what KV caching must preserve

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_cached_equals_recompute_and_rows_are_independent(dtype):
    shape = si.DecoderShape(2, 128, 2, 64, 344, 300, dtype=dtype)
    w = si.decoder_weights(shape, seed=13)
    toks = si.token_ids(13, "toks", (21,), shape.vocab).numpy()
    m = oracle.Model(shape, w)
    full = m.forward(m.new_kv(32), toks)                 # recompute everything in one call
    kv = m.new_kv(32)
    chunks = [m.forward(kv, toks[:7]), m.forward(kv, toks[7:12])]   # prefill, then a 5-row verify pass
    chunks += [m.forward(kv, toks[i:i + 1]) for i in range(12, 21)]  # then one row at a time
    assert np.array_equal(np.concatenate(chunks), full)             # identical bits


def test_truncation_then_reappend_overwrites_stale_rows():
    shape = si.DecoderShape(1, 128, 2, 64, 344, 300, dtype="f32")
    w = si.decoder_weights(shape, seed=14)
    toks = si.token_ids(14, "toks", (12,), shape.vocab).numpy()
    m = oracle.Model(shape, w)
    kv = m.new_kv(32)
    m.forward(kv, toks[:6])
    m.forward(kv, [1, 2, 3, 4, 5])          # speculated rows that get rejected
    kv.set_len(6)
    got = m.forward(kv, toks[6:])
    ref = m.forward(m.new_kv(32), toks)[6:]
    assert np.array_equal(got, ref)
    with pytest.raises(ValueError):
        kv.set_len(len(kv) + 1)             # truncation only


def test_raw_append_equals_forward_written_cache():
    """A cache filled through the raw append with the rows a forward would have written gives the
    same logits (pins the raw-append layout and the 'keys are stored rotated' convention)."""
    shape = si.DecoderShape(1, 128, 2, 64, 344, 300, dtype="f32")
    w = si.decoder_weights(shape, seed=15)
    m = oracle.Model(shape, w)
    toks = si.token_ids(15, "toks", (9,), shape.vocab).numpy()
    lw = w["layers"][0]
    E = w["embed"].double().numpy()
    rows_k, rows_v = [], []
    for pos in range(6):
        a = oracle.rmsnorm(E[toks[pos]].astype(np.float32), lw["g1"].numpy(), shape.rms_eps)
        k = oracle.linear(lw["wk"], a).reshape(2, 64)
        rows_k.append(np.concatenate([oracle.rope(k[h], pos) for h in range(2)]))
        rows_v.append(oracle.linear(lw["wv"], a))
    kv = m.new_kv(16)
    kv.append_raw([(np.stack(rows_k), np.stack(rows_v))])
    assert len(kv) == 6
    got = m.forward(kv, toks[6:])
    ref = m.forward(m.new_kv(16), toks)[6:]
    assert np.array_equal(got, ref)
