"""ctypes front-end of the CPU oracle (oracle/spec_oracle.c) plus the host loops of Section 3
(autoregressive sampling) and Sections 3/4.3/4.4 (speculative sampling with two KV caches).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the bench's cpu_baseline
leg.  It shares nothing with the GPU library and never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "spec_oracle.c")
_LIB = os.path.join(_DIR, "libspec_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over independent outputs only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC",
                               "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, i32, f64, f32 = C.c_void_p, C.c_int, C.c_double, C.c_float
        L.orc_model_new.restype = vp
        L.orc_model_new.argtypes = [i32] * 6 + [f64, f64, i32]
        L.orc_model_set_layer.argtypes = [vp, i32] + [vp] * 9
        L.orc_model_set_io.argtypes = [vp, vp, vp, vp]
        L.orc_model_free.argtypes = [vp]
        L.orc_set_num_threads.argtypes = [i32]
        L.orc_kv_new.restype = vp
        L.orc_kv_new.argtypes = [vp, i32]
        L.orc_kv_free.argtypes = [vp]
        L.orc_kv_len.argtypes = [vp]
        L.orc_kv_set_len.argtypes = [vp, i32]
        L.orc_kv_write.argtypes = [vp, i32, i32, vp, vp, i32]
        L.orc_kv_advance.argtypes = [vp, i32]
        L.orc_layers_forward.argtypes = [vp, vp, vp, i32]
        L.orc_forward.argtypes = [vp, vp, vp, i32, vp]
        L.orc_embed.argtypes = [vp, vp, i32, vp]
        L.orc_head.argtypes = [vp, vp, i32, vp]
        L.orc_rmsnorm.argtypes = [vp, vp, i32, f64, vp]
        L.orc_linear.argtypes = [vp, i32, vp, i32, i32, vp]
        L.orc_rope.argtypes = [vp, i32, C.c_int64, f64]
        L.orc_softmax.argtypes = [vp, i32, f64, vp]
        L.orc_argmax.argtypes = [vp, i32]
        L.orc_accept.argtypes = [f32, f32, f32]
        L.orc_sample.argtypes = [vp, i32, f32]
        L.orc_sample_residual.argtypes = [vp, vp, i32, f32]
        L.orc_speculative_accept.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp]
        L.orc_greedy_accept.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        L.orc_quantize_rows_int8.argtypes = [vp, i32, i32, i32, vp, vp]
        L.orc_linear_w8.argtypes = [vp, vp, vp, i32, i32, vp]
        L.orc_model_set_scales.argtypes = [vp, i32, C.POINTER(vp)]
        L.orc_quantize_rows_int4.argtypes = [vp, i32, i32, i32, i32, vp, vp]
        L.orc_linear_w4.argtypes = [vp, vp, vp, i32, i32, i32, vp]
        L.orc_model_set_wbits.argtypes = [vp, i32]
        L.orc_top_p_filter.argtypes = [vp, i32, f32, vp]
        L.orc_top_k_filter.argtypes = [vp, i32, i32, vp]
        L.orc_f32_to_bf16.restype = C.c_uint16
        L.orc_f32_to_bf16.argtypes = [f32]
        L.orc_bf16_to_f32.restype = f32
        L.orc_bf16_to_f32.argtypes = [C.c_uint16]
        _lib = L
    return _lib


def num_threads() -> int:
    return lib().orc_num_threads()


def set_num_threads(n: int) -> None:
    """Threads the row loops use from now on (for timing on one core; results do not depend on it)."""
    lib().orc_set_num_threads(int(n))


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _storage(t, is_bf16: bool) -> np.ndarray:
    """torch tensor or ndarray -> contiguous ndarray in the storage type (bf16 as uint16 bits)."""
    if hasattr(t, "detach"):
        import torch
        t = t.detach().cpu().contiguous()
        if is_bf16:
            assert t.dtype == torch.bfloat16
            return t.view(torch.int16).numpy().view(np.uint16)
        assert t.dtype == torch.float32
        return t.numpy()
    a = np.ascontiguousarray(t)
    assert a.dtype == (np.uint16 if is_bf16 else np.float32)
    return a


# ------------------------------------------------------------------ small pieces

def rmsnorm(x, g, eps=1e-5):
    x, g = _f32(x), _f32(g)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(g), x.size, eps, _p(out))
    return out


def linear(W, x, is_bf16=False):
    W = _storage(W, is_bf16)
    x = _f32(x)
    y = np.empty(W.shape[0], dtype=np.float32)
    lib().orc_linear(_p(W), int(is_bf16), _p(x), W.shape[0], W.shape[1], _p(y))
    return y


def quantize_rows_int8(W, is_bf16=False):
    """Weight-only int8 of a matrix [N, K] in the storage type -> (q int8 [N, K], scale fp32 [N])."""
    Ws = _storage(W, is_bf16)
    N, K = Ws.shape
    q = np.empty((N, K), dtype=np.int8)
    s = np.empty(N, dtype=np.float32)
    lib().orc_quantize_rows_int8(_p(Ws), int(is_bf16), N, K, _p(q), _p(s))
    return q, s


W4_GROUP = 128


def quantize_rows_int4(W, is_bf16=False, group=W4_GROUP):
    """Weight-only int4 with group scales of a matrix [N, K] in the storage type -> (packed uint8 [N, K/2],
    scale fp32 [K/group, N])."""
    Ws = _storage(W, is_bf16)
    N, K = Ws.shape
    assert K % group == 0 and group % 2 == 0
    q = np.zeros((N, K // 2), dtype=np.uint8)
    s = np.empty((K // group, N), dtype=np.float32)
    lib().orc_quantize_rows_int4(_p(Ws), int(is_bf16), N, K, group, _p(q), _p(s))
    return q, s


def linear_w4(q, scale, x, group=W4_GROUP):
    q = np.ascontiguousarray(q, dtype=np.uint8)
    scale, x = _f32(scale), _f32(x)
    y = np.empty(q.shape[0], dtype=np.float32)
    lib().orc_linear_w4(_p(q), _p(scale), _p(x), q.shape[0], q.shape[1] * 2, group, _p(y))
    return y


def linear_w8(q, scale, x):
    q = np.ascontiguousarray(q, dtype=np.int8)
    scale, x = _f32(scale), _f32(x)
    y = np.empty(q.shape[0], dtype=np.float32)
    lib().orc_linear_w8(_p(q), _p(scale), _p(x), q.shape[0], q.shape[1], _p(y))
    return y


def rope(v, pos, base=10000.0):
    v = _f32(v).copy()
    lib().orc_rope(_p(v), v.size, int(pos), base)
    return v


def softmax(logits, temperature=1.0):
    logits = _f32(logits)
    flat = logits.reshape(-1, logits.shape[-1])
    out = np.empty_like(flat)
    for r in range(flat.shape[0]):
        lib().orc_softmax(_p(flat[r]), flat.shape[1], float(temperature), _p(out[r]))
    return out.reshape(logits.shape)


def argmax(x):
    x = _f32(x)
    return lib().orc_argmax(_p(x), x.size)


def accept(u, p, q) -> bool:
    return bool(lib().orc_accept(float(u), float(p), float(q)))


def sample(p, u) -> int:
    p = _f32(p)
    return lib().orc_sample(_p(p), p.size, float(u))


def sample_residual(p, q, u) -> int:
    p, q = _f32(p), _f32(q)
    return lib().orc_sample_residual(_p(p), _p(q), p.size, float(u))


def top_p_filter(p, top_p):
    """Rows of probabilities [..., V] -> the rows restricted to their top-p nucleus and renormalised
    (top_p >= 1: returned unchanged)."""
    p = _f32(p)
    if top_p >= 1.0:
        return p.copy()
    flat = p.reshape(-1, p.shape[-1])
    out = np.empty_like(flat)
    for r in range(flat.shape[0]):
        lib().orc_top_p_filter(_p(flat[r]), flat.shape[1], float(top_p), _p(out[r]))
    return out.reshape(p.shape)


def top_k_filter(p, top_k):
    """Rows of probabilities [..., V] -> the rows restricted to their top_k most probable tokens (ties: lowest
    index first) and renormalised (top_k >= V or top_k < 1: returned unchanged)."""
    p = _f32(p)
    flat = p.reshape(-1, p.shape[-1])
    out = np.empty_like(flat)
    for r in range(flat.shape[0]):
        lib().orc_top_k_filter(_p(flat[r]), flat.shape[1], int(top_k), _p(out[r]))
    return out.reshape(p.shape)


def select(p, top_k=0, top_p=1.0):
    """The selection rules in the order they apply: top-k (top_k >= 1), then top-p (top_p < 1)."""
    if top_k and top_k >= 1:
        p = top_k_filter(p, top_k)
    return top_p_filter(p, top_p)


def speculative_accept(p, q, draft, u):
    """p [B,K+1,V], q [B,K,V] probabilities, draft [B,K] int32, u [B,K+1] -> (n_accepted[B], next[B])."""
    p, q, u = _f32(p), _f32(q), _f32(u)
    draft = np.ascontiguousarray(draft, dtype=np.int32)
    B, K1, V = p.shape
    K = K1 - 1
    assert q.shape == (B, K, V) and draft.shape == (B, K) and u.shape == (B, K + 1)
    na = np.empty(B, dtype=np.int32)
    nx = np.empty(B, dtype=np.int32)
    rc = lib().orc_speculative_accept(_p(p), _p(q), _p(draft), _p(u), B, K, V, _p(na), _p(nx))
    if rc != 0:
        raise ValueError("draft token out of range")
    return na, nx


def greedy_accept(p_logits, draft):
    p_logits = _f32(p_logits)
    draft = np.ascontiguousarray(draft, dtype=np.int32)
    B, K1, V = p_logits.shape
    na = np.empty(B, dtype=np.int32)
    nx = np.empty(B, dtype=np.int32)
    lib().orc_greedy_accept(_p(p_logits), _p(draft), B, K1 - 1, V, _p(na), _p(nx))
    return na, nx


# ------------------------------------------------------------------ model + cache

class Model:
    """A decoder held by the oracle.  `shape` has n_layers, d_model, n_heads, head_dim, d_ff,
    vocab, rope_base, rms_eps, dtype ("bf16" | "f32"); `weights` is the dict layout of
    seeded_inputs.decoder_weights (torch tensors or ndarrays; bf16 as uint16 bits)."""

    def __init__(self, shape, weights, int8_weights=False, int4_weights=False):
        """int8_weights / int4_weights: the seven matrices of every layer and the LM head are quantised
        (quantize_rows_int8: one scale per row; quantize_rows_int4: groups of 128 along K) from the given
        weights; embedding, gains and cache keep the storage type."""
        self.shape = shape
        assert not (int8_weights and int4_weights)
        self.int4_weights = bool(int4_weights)
        self.int8_weights = bool(int8_weights) or self.int4_weights   # "quantised": the code below is shared
        quant = quantize_rows_int4 if self.int4_weights else quantize_rows_int8
        self.is_bf16 = shape.dtype == "bf16"
        L = lib()
        self._keep = []
        self.h = L.orc_model_new(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim,
                                 shape.d_ff, shape.vocab, shape.rope_base, shape.rms_eps,
                                 int(self.is_bf16))
        if self.int4_weights:
            L.orc_model_set_wbits(self.h, 4)
        for l, lw in enumerate(weights["layers"]):
            ws = [self._hold(_storage(lw[n], self.is_bf16)) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")]
            gs = [self._hold(_f32(lw[n].detach().cpu().numpy() if hasattr(lw[n], "detach") else lw[n]))
                  for n in ("g1", "g2")]
            if self.int8_weights:
                qs = [quant(w, self.is_bf16) for w in ws]
                ws = [self._hold(q) for q, _ in qs]
                sc = [self._hold(s_) for _, s_ in qs]
            L.orc_model_set_layer(self.h, l, *[_p(a) for a in ws + gs])
            if self.int8_weights:
                L.orc_model_set_scales(self.h, l, (C.c_void_p * 7)(*[a.ctypes.data for a in sc]))
        if weights.get("embed") is not None:
            gf = weights["gf"]
            gf = self._hold(_f32(gf.detach().cpu().numpy() if hasattr(gf, "detach") else gf))
            emb = self._hold(_storage(weights["embed"], self.is_bf16))
            head = self._hold(_storage(weights["lm_head"], self.is_bf16))
            if self.int8_weights:
                hq, hs = quant(head, self.is_bf16)
                head = self._hold(hq)
                self._hold(hs)
                L.orc_model_set_scales(self.h, -1, (C.c_void_p * 1)(hs.ctypes.data))
            L.orc_model_set_io(self.h, _p(emb), _p(gf), _p(head))

    def _hold(self, a):
        self._keep.append(a)
        return a

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_model_free(self.h)
            self.h = None

    def new_kv(self, max_seq: int) -> "KVCache":
        return KVCache(self, max_seq)

    def forward(self, kv: "KVCache", tokens, want_logits=True):
        """Append the rows of `tokens` to the cache; return logits [M, vocab] (or None)."""
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        M = tokens.size
        logits = np.empty((M, self.shape.vocab), dtype=np.float32) if want_logits else None
        rc = lib().orc_forward(self.h, kv.h, _p(tokens), M, _p(logits) if want_logits else None)
        if rc != 0:
            raise ValueError("oracle forward failed (token out of range or cache full)")
        return logits

    def layers_forward(self, kv: "KVCache", hidden):
        """All decoder layers over hidden rows [M, d]; returns the new hidden rows."""
        h = _f32(hidden).copy()
        rc = lib().orc_layers_forward(self.h, kv.h, _p(h), h.shape[0])
        if rc != 0:
            raise ValueError("cache full")
        return h

    def head(self, hidden):
        h = _f32(hidden)
        out = np.empty((h.shape[0], self.shape.vocab), dtype=np.float32)
        lib().orc_head(self.h, _p(h), h.shape[0], _p(out))
        return out


class KVCache:
    def __init__(self, model: Model, max_seq: int):
        self.model = model
        self.h = lib().orc_kv_new(model.h, max_seq)

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_kv_free(self.h)
            self.h = None

    def __len__(self):
        return lib().orc_kv_len(self.h)

    def set_len(self, n: int):
        if lib().orc_kv_set_len(self.h, int(n)) != 0:
            raise ValueError("truncation only: new length must be within [0, len]")

    def append_raw(self, per_layer_kv):
        """per_layer_kv: list over layers of (k_rows, v_rows) [n, H*hd] in the storage type."""
        n = None
        pos0 = len(self)
        for l, (k, v) in enumerate(per_layer_kv):
            k = _storage(k, self.model.is_bf16)
            v = _storage(v, self.model.is_bf16)
            n = k.shape[0]
            if lib().orc_kv_write(self.h, l, pos0, _p(k), _p(v), n) != 0:
                raise ValueError("cache full")
        lib().orc_kv_advance(self.h, n)


# ------------------------------------------------------------------ host loops

def autoregressive_generate(target: Model, prompt, n_new: int, temperature: float, u=None,
                            max_seq=None, top_p=1.0, top_k=0):
    """Section 3, Eq. (1) with a KV cache (Section 4.2).  temperature == 0 selects argmax;
    otherwise token ~ softmax(logits / T), restricted to its top_k most probable tokens when top_k >= 1 and
    then to its top-p nucleus when top_p < 1, by the integer inverse CDF with uniforms u[n_new]."""
    x = [int(t) for t in prompt]
    kv = target.new_kv(max_seq or (len(x) + n_new + 1))
    logits = target.forward(kv, x)[-1]
    out = []
    for i in range(n_new):
        if temperature == 0:
            t = argmax(logits)
        else:
            t = sample(select(softmax(logits, temperature), top_k, top_p), u[i])
        out.append(t)
        if i + 1 < n_new:
            logits = target.forward(kv, [t])[-1]
    return out


def speculative_generate(target: Model, draft: Model, prompt, n_new: int, K: int,
                         temperature: float, u_draft=None, u_accept=None, max_seq=None, shared_kv=False, top_p=1.0, top_k=0):
    """Speculative sampling with two KV caches (Sections 3, 4.3, 4.4).

    shared_kv (the other answer to the question Section 4.4 leaves open, whether the two models need separate caches; for a draft made of
    the target's first layers): the draft reads and writes the leading layers of the target's cache.
    Its K calls leave the cache at n-1+K positions; the length is set back to n-1 and the verify call
    rewrites those positions for every layer, so afterwards the cache is complete up to n+K for both
    models and no catch-up call is ever needed.

    State at the start of a step: n committed tokens, both caches hold positions of the first n-1.
    Draft phase: K one-token draft calls (after a fully accepted step the first call feeds the two
    tokens the draft cache is missing).  Verify: one target call over [x_n, d_1..d_K].  Accept:
    the modified rejection rule.  Fix-up: both caches are truncated to n + a positions.
    top_k >= 1 / top_p < 1: the draft's and the target's rows are both restricted (top-k first, then top-p)
    before anything is sampled or compared, so the run emits the filtered target distribution.
    u_draft [steps, K], u_accept [steps, K+1].  Returns (tokens[n_new], stats dict)."""
    x = [int(t) for t in prompt]
    n0 = len(x)
    cap = max_seq or (n0 + n_new + K + 2)
    tkv = target.new_kv(cap)
    dkv = tkv if shared_kv else draft.new_kv(cap)
    if n0 > 1:
        target.forward(tkv, x[:-1], want_logits=False)
        if not shared_kv:
            draft.forward(dkv, x[:-1], want_logits=False)
    pending = [x[-1]]
    step = 0
    accepted_hist = []
    greedy = temperature == 0
    V = target.shape.vocab
    while len(x) - n0 < n_new:
        n = len(x)
        d, q_rows = [], np.zeros((K, V), dtype=np.float32)
        feed = pending
        for i in range(K):
            ql = draft.forward(dkv, feed)[-1]
            if greedy:
                tok = argmax(ql)
            else:
                q_rows[i] = select(softmax(ql, temperature), top_k, top_p)
                tok = sample(q_rows[i], u_draft[step][i])
            d.append(tok)
            feed = [tok]
        if shared_kv:
            tkv.set_len(n - 1)   # the draft's rows of the leading layers are rewritten by the verify call
        pl = target.forward(tkv, [x[-1]] + d)
        if greedy:
            na, nx = greedy_accept(pl[None], np.asarray([d], dtype=np.int32))
        else:
            p_rows = select(softmax(pl, temperature), top_k, top_p)
            na, nx = speculative_accept(p_rows[None], q_rows[None], np.asarray([d], dtype=np.int32),
                                        np.asarray([u_accept[step]], dtype=np.float32))
        a, y = int(na[0]), int(nx[0])
        x += d[:a] + [y]
        tkv.set_len(n + a)
        if shared_kv or a < K:
            if not shared_kv:
                dkv.set_len(n + a)
            pending = [y]
        else:
            pending = [d[K - 1], y]
        accepted_hist.append(a)
        step += 1
    return x[n0:n0 + n_new], {"steps": step, "accepted": accepted_hist}
