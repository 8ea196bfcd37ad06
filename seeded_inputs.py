"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests / bench.

This module only draws random numbers and shapes them: it holds none of the method's
arithmetic (no softmax, no sampling, no attention).  Everything is a pure function of
(seed, name, shape), produced with torch's Philox/MT generators, so the oracle and the HIP
library always receive the same bits.  Tensors are generated on the CPU unless a device is
given; a tensor generated on a GPU is handed to the oracle by copying it back (same bits).

Workload recipes (value distributions follow the synthetic configurations this repository is
measured on; "N(0, s)" always means standard deviation s):
  * decoder weights: every matrix N(0, 0.02); RMSNorm gains 1 + N(0, 0.02)
  * token ids: uniform on [0, vocab)
  * uniforms: multiples of 2^-24 in [0, 1)
  * standalone accept workload: draft logits N(0, 2), target logits = draft + N(0, 0.5),
    bonus row N(0, 2)
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, asdict

import torch


@dataclass(frozen=True)
class DecoderShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    dtype: str = "bf16"  # storage type of weights and KV cache: "bf16" or "f32"

    def as_dict(self):
        return asdict(self)


# The shapes the tests and the bench use.
TINY_TARGET = DecoderShape(2, 256, 4, 64, 688, 1024, dtype="f32")
TINY_DRAFT = DecoderShape(1, 128, 2, 64, 344, 1024, dtype="f32")
LAYER_7B = DecoderShape(1, 4096, 32, 128, 11008, 32000, dtype="bf16")
FULL_7B = DecoderShape(32, 4096, 32, 128, 11008, 32000, dtype="bf16")


def _seed_for(seed: int, name: str) -> int:
    h = hashlib.sha256(f"{seed}:{name}".encode()).digest()
    return int.from_bytes(h[:7], "little")


def _gen(seed: int, name: str, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(_seed_for(seed, name))
    return g


def normal(seed: int, name: str, shape, std: float, mean: float = 0.0, device="cpu",
           dtype=torch.float32) -> torch.Tensor:
    """mean + std * N(0,1) drawn in fp32, then rounded (nearest-even) to `dtype`."""
    x = torch.randn(shape, generator=_gen(seed, name, device), device=device, dtype=torch.float32)
    x.mul_(std)
    if mean != 0.0:
        x.add_(mean)
    return x.to(dtype)


def token_ids(seed: int, name: str, shape, vocab: int, device="cpu") -> torch.Tensor:
    return torch.randint(0, vocab, shape, generator=_gen(seed, name, device), device=device,
                         dtype=torch.int32)


def uniforms(seed: int, name: str, shape, device="cpu") -> torch.Tensor:
    """fp32 uniforms that are exact multiples of 2^-24 in [0, 1)."""
    m = torch.randint(0, 1 << 24, shape, generator=_gen(seed, name, device), device=device,
                      dtype=torch.int32)
    return m.to(torch.float32) * (1.0 / (1 << 24))


def storage_dtype(shape: DecoderShape):
    return torch.bfloat16 if shape.dtype == "bf16" else torch.float32


def layer_weights(shape: DecoderShape, seed: int, layer: int, device="cpu") -> dict:
    """One decoder layer: wq, wk, wv, wo [d,d]; wg, wu [F,d]; wd [d,F]; g1, g2 [d] (fp32 gains)."""
    d, F = shape.d_model, shape.d_ff
    dt = storage_dtype(shape)
    hd_all = shape.n_heads * shape.head_dim
    pre = f"layer{layer}."
    w = {}
    for nm, shp in (("wq", (hd_all, d)), ("wk", (hd_all, d)), ("wv", (hd_all, d)),
                    ("wo", (d, hd_all)), ("wg", (F, d)), ("wu", (F, d)), ("wd", (d, F))):
        w[nm] = normal(seed, pre + nm, shp, 0.02, device=device, dtype=dt)
    for nm in ("g1", "g2"):
        w[nm] = normal(seed, pre + nm, (d,), 0.02, mean=1.0, device=device)
    return w


def decoder_weights(shape: DecoderShape, seed: int, device="cpu") -> dict:
    """Whole decoder: 'embed' [V,d], 'layers' list, 'gf' [d] final gain, 'lm_head' [V,d]."""
    dt = storage_dtype(shape)
    return {
        "embed": normal(seed, "embed", (shape.vocab, shape.d_model), 0.02, device=device, dtype=dt),
        "layers": [layer_weights(shape, seed, l, device) for l in range(shape.n_layers)],
        "gf": normal(seed, "gf", (shape.d_model,), 0.02, mean=1.0, device=device),
        "lm_head": normal(seed, "lm_head", (shape.vocab, shape.d_model), 0.02, device=device, dtype=dt),
    }


def packed_decoder(shape: DecoderShape, seed: int, device="cpu"):
    """The same decoder as decoder_weights(), layer by layer, with q|k|v and gate|up concatenated into the
    fused matrices a weight-streaming forward reads ([3*H*hd, d] and [2*F, d]); only one layer's separate
    matrices exist at a time, so a 7B-shaped model can be drawn directly in device memory.
    Returns (shape, packed layers [{wqkv, wo, wgu, wd, g1, g2}], {embed, gf, lm_head})."""
    packed = []
    for l in range(shape.n_layers):
        lw = layer_weights(shape, seed, l, device=device)
        packed.append({"wqkv": torch.cat([lw["wq"], lw["wk"], lw["wv"]], 0), "wo": lw["wo"],
                       "wgu": torch.cat([lw["wg"], lw["wu"]], 0), "wd": lw["wd"], "g1": lw["g1"], "g2": lw["g2"]})
        del lw
    dt = storage_dtype(shape)
    io = {"embed": normal(seed, "embed", (shape.vocab, shape.d_model), 0.02, device=device, dtype=dt),
          "gf": normal(seed, "gf", (shape.d_model,), 0.02, mean=1.0, device=device),
          "lm_head": normal(seed, "lm_head", (shape.vocab, shape.d_model), 0.02, device=device, dtype=dt)}
    return shape, packed, io


def packed_7b(seed: int, n_layers: int, device="cpu"):
    """packed_decoder() of the 7B shape with the given depth."""
    return packed_decoder(DecoderShape(**{**FULL_7B.as_dict(), "n_layers": n_layers}), seed, device)


def damp_late_layers(packed, first: int, factor: float):
    """A second set of packed layers in which every layer from `first` on writes `factor` times as much into the residual
    stream (its O and down projections are scaled, rounded to the storage type again); all other tensors are shared.
    With a small factor the target's first `first` layers + final norm + LM head predict the whole target the way a
    trained draft predicts its target: a synthetic stand-in for a good draft."""
    out = []
    for l, p in enumerate(packed):
        if l < first:
            out.append(p)
        else:
            q = dict(p)
            for k in ("wo", "wd"):
                q[k] = (p[k].float() * factor).to(p[k].dtype)
            out.append(q)
    return out


def unpack_layers(shape: DecoderShape, packed):
    """Packed layers -> the separate host matrices {wq, wk, wv, wo, wg, wu, wd, g1, g2} (views, same bits)."""
    W = shape.n_heads * shape.head_dim
    return [{"wq": p["wqkv"][:W].cpu(), "wk": p["wqkv"][W:2 * W].cpu(), "wv": p["wqkv"][2 * W:].cpu(), "wo": p["wo"].cpu(),
             "wg": p["wgu"][:shape.d_ff].cpu(), "wu": p["wgu"][shape.d_ff:].cpu(), "wd": p["wd"].cpu(),
             "g1": p["g1"].cpu(), "g2": p["g2"].cpu()} for p in packed]


def early_exit_draft(target_shape: DecoderShape, target_weights: dict, n_layers: int):
    """Draft = the target's first `n_layers` layers + its final gain and LM head (same tensors)."""
    ds = DecoderShape(**{**target_shape.as_dict(), "n_layers": n_layers})
    dw = {"embed": target_weights["embed"], "layers": target_weights["layers"][:n_layers],
          "gf": target_weights["gf"], "lm_head": target_weights["lm_head"]}
    return ds, dw


def kv_context(shape: DecoderShape, seed: int, name: str, n_rows: int, device="cpu"):
    """Synthetic existing context for one sequence: per layer K and V rows [n_rows, H*hd] ~ N(0,1)
    in the storage type (K rows are taken as already rotated)."""
    dt = storage_dtype(shape)
    hd_all = shape.n_heads * shape.head_dim
    out = []
    for l in range(shape.n_layers):
        k = normal(seed, f"{name}.k{l}", (n_rows, hd_all), 1.0, device=device, dtype=dt)
        v = normal(seed, f"{name}.v{l}", (n_rows, hd_all), 1.0, device=device, dtype=dt)
        out.append((k, v))
    return out


def accept_workload(seed: int, batch: int, K: int, vocab: int, device="cpu"):
    """Standalone accept workload: q_logits [B,K,V] ~ N(0,2); p_logits [B,K+1,V] with rows 0..K-1 =
    q_logits + N(0,0.5) and row K ~ N(0,2); accept/sampling uniforms [B,K+1]; draft uniforms [B,K]."""
    q = normal(seed, "q_logits", (batch, K, vocab), 2.0, device=device)
    p = torch.empty((batch, K + 1, vocab), dtype=torch.float32, device=device)
    p[:, :K] = q + normal(seed, "p_noise", (batch, K, vocab), 0.5, device=device)
    p[:, K] = normal(seed, "p_bonus", (batch, vocab), 2.0, device=device)
    u = uniforms(seed, "u_accept", (batch, K + 1), device=device)
    ud = uniforms(seed, "u_draft", (batch, K), device=device)
    return p, q, u, ud
