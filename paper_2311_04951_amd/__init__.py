"""Python binding of libspecverify.so (C ABI in include/specverify.h).

Argument marshalling only: every function here has the name of the C entry point it calls, takes
torch tensors (device memory) where the C call takes device pointers, and raises SpecVerifyError
on a negative return code.  PyTorch is used for device memory and streams, nothing else; there is
no CPU fallback - importing works without a GPU, calling does not.
"""
from __future__ import annotations

import atexit
import weakref
import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libspecverify.so")

SS_OK, SS_EINVAL, SS_ECAPACITY, SS_EHIP, SS_EABORTED = 0, -1, -2, -3, -4
SS_DTYPE_F32, SS_DTYPE_BF16 = 0, 1
SS_MAX_ROWS_PER_SEQ = 16
SS_QUANT_NONE, SS_QUANT_INT8, SS_QUANT_INT4_G128 = 0, 1, 2

EXPORTS = [
    "ss_last_error", "ss_device_status", "ss_model_create", "ss_model_destroy", "ss_kv_cache_alloc",
    "ss_kv_cache_free", "ss_kv_cache_bytes", "ss_kv_cache_append", "ss_kv_cache_set_len",
    "ss_kv_cache_get_len", "ss_kv_cache_rollback", "ss_verify_forward", "ss_decoder_layers_forward",
    "ss_draft_step", "ss_softmax", "ss_speculative_accept", "ss_speculative_accept_logits",
    "ss_greedy_accept", "ss_profile_enable", "ss_profile_read", "ss_model_set_persistent", "ss_model_set_persistent_options",
    "ss_speculative_step", "ss_speculative_step_batched", "ss_probe_read_bandwidth", "ss_quantize_rows_int8", "ss_top_p_filter", "ss_top_k_filter",
    "ss_model_set_wait_limit", "ss_quantize_rows_int4", "ss_shutdown", "ss_kv_cache_create", "ss_kv_cache_truncate",
    "ss_workspace_bytes", "ss_workspace_init", "ss_workspace_status", "ss_model_set_timeline", "ss_freeze_allocations",
    "ss_speculative_accept_noalloc",
]

PROFILE_CLASSES = ["rmsnorm", "qkv_gemm", "attention", "oproj_gemm", "gateup_gemm", "down_gemm", "head_gemm", "other",
                   "verify_persistent"]


class SpecVerifyError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"specverify error {code}: {msg}")
        self.code = code


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ff", "vocab")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32),
                ("max_rows", C.c_int32), ("max_pos", C.c_int32), ("weight_quant", C.c_int32)]


class _LayerW(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wqkv", "wo", "wgu", "wd", "g1", "g2", "sqkv", "so", "sgu", "sd")]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("layers", C.POINTER(_LayerW)), ("gf", C.c_void_p), ("lm_head", C.c_void_p),
                ("s_head", C.c_void_p)]


_lib = None


def lib():
    """Loads the built library; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        L.ss_last_error.restype = C.c_char_p
        L.ss_kv_cache_bytes.restype = C.c_size_t
        L.ss_workspace_bytes.restype = C.c_size_t
        sz = C.c_size_t
        sig = {
            "ss_device_status": [vp, vp, vp],
            "ss_model_create": [C.POINTER(_Cfg), C.POINTER(_Weights), C.POINTER(vp)],
            "ss_model_destroy": [vp],
            "ss_kv_cache_alloc": [vp, i32, i32, C.POINTER(vp)],
            "ss_kv_cache_create": [vp, i32, i32, vp, sz, vp, C.POINTER(vp)],
            "ss_kv_cache_truncate": [vp, vp, vp, vp, vp],
            "ss_workspace_bytes": [i64, i32],
            "ss_workspace_init": [vp, sz, vp],
            "ss_workspace_status": [vp, sz, vp, vp],
            "ss_model_set_timeline": [vp, vp, sz],
            "ss_shutdown": [],
            "ss_freeze_allocations": [i32],
            "ss_kv_cache_free": [vp],
            "ss_kv_cache_bytes": [vp, i32, i32],
            "ss_kv_cache_append": [vp, i32, i32, i32, vp, vp, i32, vp],
            "ss_kv_cache_set_len": [vp, vp, vp],
            "ss_kv_cache_get_len": [vp, vp, vp],
            "ss_kv_cache_rollback": [vp, vp, vp, i32, vp],
            "ss_verify_forward": [vp, vp, vp, i32, i32, vp, vp],
            "ss_decoder_layers_forward": [vp, vp, vp, i32, i32, vp],
            "ss_draft_step": [vp, vp, vp, i32, i32, f32, f32, i32, vp, vp, i64, vp, vp],
            "ss_top_p_filter": [vp, i32, i32, f32, vp, vp],
            "ss_top_k_filter": [vp, i32, i32, i32, vp, vp],
            "ss_softmax": [vp, i32, i32, f32, vp, vp, sz, vp],
            "ss_speculative_accept": [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp],
            "ss_speculative_accept_noalloc": [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp],
            "ss_speculative_accept_logits": [vp, vp, f32, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp],
            "ss_greedy_accept": [vp, vp, i32, i32, i32, vp, vp, vp, sz, vp],
            "ss_profile_enable": [vp, i32],
            "ss_model_set_persistent": [vp, i32],
            "ss_model_set_persistent_options": [vp, i32, i32],
            "ss_model_set_wait_limit": [vp, C.c_uint32],
            "ss_speculative_step": [vp, vp, vp, vp, i32, C.c_float, C.c_float, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp],
            "ss_speculative_step_batched": [vp, vp, vp, vp, i32, i32, C.c_float, C.c_float, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp],
            "ss_profile_read": [vp, i32, vp, vp],
            "ss_probe_read_bandwidth": [vp, C.c_size_t, i32, vp, vp, vp],
            "ss_quantize_rows_int8": [vp, i32, i64, i64, vp, vp, vp],
            "ss_quantize_rows_int4": [vp, i32, i64, i64, vp, vp, vp],
        }
        for name, args in sig.items():
            getattr(L, name).argtypes = args
        _lib = L
        atexit.register(ss_shutdown)     # releases what is still alive while the HIP runtime is up
    return _lib


def ss_freeze_allocations(on: bool):
    _check(lib().ss_freeze_allocations(int(bool(on))))


_live = weakref.WeakSet()   # Model and KVCache objects that hold a handle


def ss_shutdown():
    """Destroys every live model and cache of the library.  The Python objects that held them forget their handles:
    a later close() or garbage collection must not release a handle value that a new object has received since."""
    if _lib is not None:
        _lib.ss_shutdown()
    for obj in list(_live):
        obj.handle = None
    _workspaces.clear()


def _check(rc):
    if rc != 0:
        raise SpecVerifyError(rc, lib().ss_last_error().decode())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev(t, dtype=None):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _host_i32(seq):
    import numpy as np
    a = np.ascontiguousarray(seq, dtype=np.int32)
    return a, a.ctypes.data_as(C.c_void_p)


# ---------------------------------------------------------------------------------- handles

class Model:
    """Owner of an ss_model handle.  `shape` carries n_layers, d_model, n_heads, head_dim, d_ff, vocab,
    rope_base, rms_eps, dtype ("bf16" | "f32"); `weights` is a dict
    {embed, layers: [{wq, wk, wv, wo, wg, wu, wd, g1, g2}], gf, lm_head} of device tensors.  Packing
    q|k|v and gate|up into the fused matrices the library streams is a one-off copy done here
    (memory plumbing; pass `packed_layers` = [{wqkv, wo, wgu, wd, g1, g2}] to skip it).
    int8_weights / int4_weights: the library quantises the packed matrices and the LM head
    (ss_quantize_rows_int8: one scale per row; ss_quantize_rows_int4: groups of 128 along K) and the model
    streams the quantised copies; packed layers that already carry quantised matrices with their scales
    ({..., sqkv, so, sgu, sd}) and weights["s_head"] are taken as they are."""

    def __init__(self, shape, weights=None, max_rows=16, max_pos=4096, packed_layers=None, int8_weights=False,
                 int4_weights=False):
        self.shape = shape
        self.max_rows, self.max_pos = int(max_rows), int(max_pos)
        if int8_weights and int4_weights:
            raise ValueError("one quantisation at a time")
        self.int4_weights = bool(int4_weights)
        self.int8_weights = bool(int8_weights) or self.int4_weights     # "quantised": the code below is shared
        quantise = ss_quantize_rows_int4 if self.int4_weights else ss_quantize_rows_int8
        st = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        if packed_layers is None:
            packed_layers = []
            for lw in weights["layers"]:
                packed_layers.append({
                    "wqkv": torch.cat([lw["wq"], lw["wk"], lw["wv"]], 0).contiguous(),
                    "wo": lw["wo"].contiguous(),
                    "wgu": torch.cat([lw["wg"], lw["wu"]], 0).contiguous(),
                    "wd": lw["wd"].contiguous(), "g1": lw["g1"].contiguous(), "g2": lw["g2"].contiguous()})
        self.embed = weights.get("embed") if weights else None
        self.gf = weights.get("gf") if weights else None
        self.lm_head = weights.get("lm_head") if weights else None
        self.s_head = weights.get("s_head") if weights else None
        wt = st
        if self.int8_weights:
            wt = torch.uint8 if self.int4_weights else torch.int8
            quantised = []
            for pl in packed_layers:
                if pl["wqkv"].dtype == wt:
                    quantised.append(pl)
                    continue
                ql = {"g1": pl["g1"], "g2": pl["g2"]}
                for n, sn in (("wqkv", "sqkv"), ("wo", "so"), ("wgu", "sgu"), ("wd", "sd")):
                    ql[n], ql[sn] = quantise(pl[n])
                quantised.append(ql)
            packed_layers = quantised
            if self.lm_head is not None and self.lm_head.dtype != wt:
                self.lm_head, self.s_head = quantise(self.lm_head)
        self.layers = packed_layers
        arr = (_LayerW * max(1, len(packed_layers)))()
        for i, pl in enumerate(packed_layers):
            for n in ("wqkv", "wo", "wgu", "wd"):
                setattr(arr[i], n, _dev(pl[n], wt).value)
            for n in ("g1", "g2") + (("sqkv", "so", "sgu", "sd") if self.int8_weights else ()):
                setattr(arr[i], n, _dev(pl[n], torch.float32).value)
        w = _Weights(_dev(self.embed, st if self.embed is not None else None), arr,
                     _dev(self.gf, torch.float32 if self.gf is not None else None),
                     _dev(self.lm_head, wt if self.lm_head is not None else None),
                     _dev(self.s_head, torch.float32 if self.s_head is not None else None))
        cfg = _Cfg(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ff, shape.vocab,
                   shape.rope_base, shape.rms_eps, SS_DTYPE_BF16 if shape.dtype == "bf16" else SS_DTYPE_F32,
                   max_rows, max_pos, SS_QUANT_INT4_G128 if self.int4_weights else (SS_QUANT_INT8 if self.int8_weights else SS_QUANT_NONE))
        h = C.c_void_p()
        _check(lib().ss_model_create(C.byref(cfg), C.byref(w), C.byref(h)))
        self.handle = h
        _live.add(self)

    def close(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ss_model_destroy(self.handle)
            self.handle = None

    __del__ = close


class KVCache:
    """Owner of an ss_kv_cache handle over a buffer allocated here with torch (the caller-owned buffer of
    ss_kv_cache_create); `buf` may be given to place the cache in existing device memory."""

    def __init__(self, model: Model, batch: int, max_seq: int, buf=None, stream=None):
        self.model, self.batch, self.max_seq = model, batch, max_seq
        need = lib().ss_kv_cache_bytes(model.handle, batch, max_seq)
        h = C.c_void_p()
        if isinstance(buf, str) and buf == "library":     # the convenience call: the library allocates (and frees) the buffer
            self.buf = None
            _check(lib().ss_kv_cache_alloc(model.handle, batch, max_seq, C.byref(h)))
            self.handle = h
            return
        if buf is None:
            buf = torch.empty(max(need, 16), dtype=torch.uint8, device=torch.device("cuda", torch.cuda.current_device()))
        self.buf = buf
        _check(lib().ss_kv_cache_create(model.handle, batch, max_seq, _dev(buf), buf.numel() * buf.element_size(), _stream(stream),
                                        C.byref(h)))
        self.handle = h
        _live.add(self)

    def close(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ss_kv_cache_free(self.handle)
            self.handle = None
        self.buf = None

    __del__ = close


# ---------------------------------------------------------------------------------- workspaces

_workspaces = {}


def ss_workspace_bytes(rows: int, vocab: int) -> int:
    return lib().ss_workspace_bytes(int(rows), int(vocab))


def ss_workspace_init(ws, stream=None):
    _check(lib().ss_workspace_init(_dev(ws), ws.numel() * ws.element_size(), _stream(stream)))
    return ws


def ss_workspace_status(ws, stream=None) -> int:
    out = C.c_int32(0)
    _check(lib().ss_workspace_status(_dev(ws), ws.numel() * ws.element_size(), _stream(stream), C.byref(out)))
    return out.value


def workspace(device, rows: int, vocab: int):
    """A device workspace for the calls without a handle: one per (device, stream), kept between calls and
    replaced by a larger one when a call needs more (memory plumbing: the C calls never allocate)."""
    need = ss_workspace_bytes(rows, vocab)
    key = (str(device), torch.cuda.current_stream().cuda_stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < need:
        ws = torch.empty(max(need, 1 << 20), dtype=torch.uint8, device=device)
        ss_workspace_init(ws)
        _workspaces[key] = ws
    return ws


def _ws_args(ws, device, rows, vocab):
    if ws is None:
        ws = workspace(device, rows, vocab)
    return _dev(ws), ws.numel() * ws.element_size()


# ---------------------------------------------------------------------------------- entry points

def ss_kv_cache_alloc(model: Model, batch: int, max_seq: int) -> KVCache:
    return KVCache(model, batch, max_seq)


def ss_kv_cache_create(model: Model, batch: int, max_seq: int, buf, stream=None) -> KVCache:
    """A cache over the caller's device buffer `buf` (at least ss_kv_cache_bytes bytes; the call clears it)."""
    return KVCache(model, batch, max_seq, buf=buf, stream=stream)


def ss_kv_cache_bytes(model: Model, batch: int, max_seq: int) -> int:
    return lib().ss_kv_cache_bytes(model.handle, batch, max_seq)


def ss_kv_cache_append(kv: KVCache, layer: int, seq: int, pos0: int, k, v, stream=None):
    _check(lib().ss_kv_cache_append(kv.handle, layer, seq, pos0, _dev(k), _dev(v), k.shape[0], _stream(stream)))


def ss_kv_cache_set_len(kv: KVCache, lens, stream=None):
    a, p = _host_i32(lens)
    if a.size != kv.batch:
        raise ValueError("one length per sequence")
    _check(lib().ss_kv_cache_set_len(kv.handle, p, _stream(stream)))


def ss_kv_cache_truncate(kv: KVCache, new_len, new_len_host=None, status=None, stream=None):
    """Device-side truncation: len[b] = min(len[b], new_len[b]) (new_len: device int32 [batch])."""
    hp = C.c_void_p(0)
    if new_len_host is not None:
        keep, hp = _host_i32(new_len_host)
    _check(lib().ss_kv_cache_truncate(kv.handle, _dev(new_len, torch.int32), hp, _dev(status, torch.int32 if status is not None else None),
                                      _stream(stream)))


def ss_kv_cache_get_len(kv: KVCache, stream=None):
    import numpy as np
    a = np.zeros(kv.batch, dtype=np.int32)
    _check(lib().ss_kv_cache_get_len(kv.handle, a.ctypes.data_as(C.c_void_p), _stream(stream)))
    return a


def ss_kv_cache_rollback(kv: KVCache, n_accepted, M: int, n_accepted_host=None, stream=None):
    hp = C.c_void_p(0)
    if n_accepted_host is not None:
        keep, hp = _host_i32(n_accepted_host)
    _check(lib().ss_kv_cache_rollback(kv.handle, _dev(n_accepted, torch.int32), hp, M, _stream(stream)))


def ss_verify_forward(model: Model, kv: KVCache, tokens, M: int, logits=None, stream=None):
    """tokens int32 [batch, M] -> logits fp32 [batch, M, vocab] (allocated when not given; pass
    logits=False to skip the LM head)."""
    batch = tokens.numel() // M
    if logits is None:
        logits = torch.empty((batch, M, model.shape.vocab), dtype=torch.float32, device=tokens.device)
    lp = None if logits is False else logits
    _check(lib().ss_verify_forward(model.handle, kv.handle, _dev(tokens, torch.int32), batch, M,
                                   _dev(lp, torch.float32 if lp is not None else None), _stream(stream)))
    return lp


def ss_decoder_layers_forward(model: Model, kv: KVCache, h, batch: int, M: int, stream=None):
    _check(lib().ss_decoder_layers_forward(model.handle, kv.handle, _dev(h, torch.float32), batch, M, _stream(stream)))
    return h


def ss_draft_step(draft: Model, kv: KVCache, tokens, m: int, temperature: float, u, q_rows, ldq: int,
                  token_out, stream=None, top_p: float = 1.0, top_k: int = 0):
    batch = tokens.numel() // m
    qp = C.c_void_p(0) if q_rows is None else C.c_void_p(q_rows.data_ptr())
    _check(lib().ss_draft_step(draft.handle, kv.handle, _dev(tokens, torch.int32), batch, m, float(temperature), float(top_p), int(top_k),
                               _dev(u, torch.float32 if u is not None else None), qp, int(ldq),
                               _dev(token_out, torch.int32), _stream(stream)))
    return token_out


def ss_softmax(logits, temperature: float, probs=None, stream=None, ws=None):
    V = logits.shape[-1]
    rows = logits.numel() // V
    if probs is None:
        probs = torch.empty_like(logits)
    _check(lib().ss_softmax(_dev(logits, torch.float32), rows, V, float(temperature), _dev(probs, torch.float32),
                            *_ws_args(ws, logits.device, rows, V), _stream(stream)))
    return probs


def ss_top_p_filter(probs, top_p: float, out=None, stream=None):
    """Rows [..., V] of probabilities -> restricted to their top-p nucleus and renormalised (out may be probs)."""
    V = probs.shape[-1]
    if out is None:
        out = torch.empty_like(probs)
    _check(lib().ss_top_p_filter(_dev(probs, torch.float32), probs.numel() // V, V, float(top_p), _dev(out, torch.float32),
                                 _stream(stream)))
    return out


def ss_top_k_filter(probs, top_k: int, out=None, stream=None):
    """Rows [..., V] of probabilities -> restricted to their top_k most probable tokens and renormalised (out may be probs)."""
    V = probs.shape[-1]
    if out is None:
        out = torch.empty_like(probs)
    _check(lib().ss_top_k_filter(_dev(probs, torch.float32), probs.numel() // V, V, int(top_k), _dev(out, torch.float32),
                                 _stream(stream)))
    return out


def _accept_out(batch, device, n_accepted, next_token):
    if n_accepted is None:
        n_accepted = torch.empty(batch, dtype=torch.int32, device=device)
    if next_token is None:
        next_token = torch.empty(batch, dtype=torch.int32, device=device)
    return n_accepted, next_token


def ss_speculative_accept(p, q, draft_tokens, uniforms, n_accepted=None, next_token=None, stream=None, ws=None):
    B, K1, V = p.shape
    n_accepted, next_token = _accept_out(B, p.device, n_accepted, next_token)
    _check(lib().ss_speculative_accept(_dev(p, torch.float32), _dev(q, torch.float32) if K1 > 1 else C.c_void_p(0),
                                       _dev(draft_tokens, torch.int32) if K1 > 1 else C.c_void_p(0),
                                       _dev(uniforms, torch.float32), B, K1 - 1, V, _dev(n_accepted), _dev(next_token),
                                       *_ws_args(ws, p.device, B * (2 * K1 - 1), V), _stream(stream)))
    return n_accepted, next_token


def ss_speculative_accept_noalloc(p, q, draft_tokens, uniforms, n_accepted, next_token, status=None, stream=None):
    """The rejection step with the library's built-in scratch array: every tensor, outputs included, is the caller's."""
    B, K1, V = p.shape
    _check(lib().ss_speculative_accept_noalloc(_dev(p, torch.float32), _dev(q, torch.float32) if K1 > 1 else C.c_void_p(0),
                                               _dev(draft_tokens, torch.int32) if K1 > 1 else C.c_void_p(0),
                                               _dev(uniforms, torch.float32), B, K1 - 1, V, _dev(n_accepted, torch.int32),
                                               _dev(next_token, torch.int32), _dev(status, torch.int32 if status is not None else None),
                                               _stream(stream)))
    return n_accepted, next_token


def ss_speculative_accept_logits(p_logits, q_logits, temperature, draft_tokens, uniforms, n_accepted=None,
                                 next_token=None, p_out=None, q_out=None, stream=None, ws=None):
    B, K1, V = p_logits.shape
    n_accepted, next_token = _accept_out(B, p_logits.device, n_accepted, next_token)
    _check(lib().ss_speculative_accept_logits(
        _dev(p_logits, torch.float32), _dev(q_logits, torch.float32) if K1 > 1 else C.c_void_p(0), float(temperature),
        _dev(draft_tokens, torch.int32) if K1 > 1 else C.c_void_p(0), _dev(uniforms, torch.float32), B, K1 - 1, V,
        _dev(n_accepted), _dev(next_token), _dev(p_out), _dev(q_out), *_ws_args(ws, p_logits.device, B * (2 * K1 - 1), V),
        _stream(stream)))
    return n_accepted, next_token


def ss_greedy_accept(p_logits, draft_tokens, n_accepted=None, next_token=None, stream=None, ws=None):
    B, K1, V = p_logits.shape
    n_accepted, next_token = _accept_out(B, p_logits.device, n_accepted, next_token)
    _check(lib().ss_greedy_accept(_dev(p_logits, torch.float32),
                                  _dev(draft_tokens, torch.int32) if K1 > 1 else C.c_void_p(0), B, K1 - 1, V,
                                  _dev(n_accepted), _dev(next_token), *_ws_args(ws, p_logits.device, B * K1, V), _stream(stream)))
    return n_accepted, next_token


class StepBuffers:
    """Device and host buffers of ss_speculative_step for one sequence (allocated once per decode loop)."""

    def __init__(self, K: int, vocab: int, first_token: int, device):
        self.K, self.V = K, vocab
        i32, f32 = torch.int32, torch.float32
        self.feed = torch.tensor([first_token, 0], dtype=i32, device=device)
        self.n_feed = C.c_int32(1)
        self.verify_tokens = torch.zeros(K + 1, dtype=i32, device=device)
        self.q = torch.zeros((K, vocab), dtype=f32, device=device)
        self.logits = torch.empty((K + 1, vocab), dtype=f32, device=device)
        self.p = torch.empty((K + 1, vocab), dtype=f32, device=device)
        self.result = torch.zeros(2, dtype=i32, device=device)
        self.out = (C.c_int32 * (K + 2))()


def ss_speculative_step(target: Model, target_kv: KVCache, draft: Model, draft_kv: KVCache, buf: StepBuffers,
                        temperature: float, u_draft=None, u_accept=None, stream=None, top_p: float = 1.0, top_k: int = 0):
    """One speculative step; returns (n_accepted, next_token, [d_1..d_K]) as host integers."""
    _check(lib().ss_speculative_step(
        target.handle, target_kv.handle, draft.handle, draft_kv.handle, buf.K, float(temperature), float(top_p), int(top_k),
        _dev(buf.feed, torch.int32),
        C.byref(buf.n_feed), _dev(u_draft, torch.float32), _dev(u_accept, torch.float32), _dev(buf.verify_tokens, torch.int32),
        _dev(buf.q), _dev(buf.logits), _dev(buf.p), _dev(buf.result, torch.int32), buf.out, _stream(stream)))
    return buf.out[0], buf.out[1], list(buf.out[2:2 + buf.K])


class BatchedStepBuffers:
    """Device and host buffers of ss_speculative_step_batched (allocated once per decode loop).
    last_two: [batch][2], every sequence's last two committed tokens."""

    def __init__(self, batch: int, K: int, vocab: int, last_two, device):
        self.B, self.K, self.V = batch, K, vocab
        i32, f32 = torch.int32, torch.float32
        self.feed = torch.as_tensor(last_two, dtype=i32).reshape(batch, 2).to(device).contiguous()
        self.draft_tokens = torch.zeros((2, K, batch), dtype=i32, device=device)
        self.verify_tokens = torch.zeros((batch, K + 1), dtype=i32, device=device)
        self.q = torch.zeros((batch, K, vocab), dtype=f32, device=device)
        self.logits = torch.empty((batch, K + 1, vocab), dtype=f32, device=device)
        self.p = torch.empty((batch, K + 1, vocab), dtype=f32, device=device)
        self.result = torch.zeros((2, batch), dtype=i32, device=device)
        self.out = (C.c_int32 * (batch * (K + 2)))()


def ss_speculative_step_batched(target: Model, target_kv: KVCache, draft: Model, draft_kv: KVCache, buf: BatchedStepBuffers,
                                temperature: float, u_draft=None, u_accept=None, stream=None, top_p: float = 1.0, top_k: int = 0):
    """One speculative step of every sequence; u_draft [K][batch], u_accept [batch][K+1].
    Returns a list over sequences of (n_accepted, next_token, [d_1..d_K]) as host integers."""
    _check(lib().ss_speculative_step_batched(
        target.handle, target_kv.handle, draft.handle, draft_kv.handle, buf.B, buf.K, float(temperature), float(top_p), int(top_k),
        _dev(buf.feed, torch.int32), _dev(u_draft, torch.float32), _dev(u_accept, torch.float32), _dev(buf.draft_tokens, torch.int32),
        _dev(buf.verify_tokens, torch.int32), _dev(buf.q), _dev(buf.logits), _dev(buf.p), _dev(buf.result, torch.int32), buf.out,
        _stream(stream)))
    w = buf.K + 2
    return [(buf.out[b * w], buf.out[b * w + 1], list(buf.out[b * w + 2:b * w + w])) for b in range(buf.B)]


def ss_device_status(model: Model, stream=None) -> int:
    out = C.c_int32(0)
    _check(lib().ss_device_status(model.handle, _stream(stream), C.byref(out)))
    return out.value


def ss_model_set_persistent(model: Model, on: bool):
    _check(lib().ss_model_set_persistent(model.handle, int(bool(on))))


def ss_quantize_rows_int8(w, stream=None):
    """Row-wise int8 of a device matrix [rows, K] (fp32 or bf16) -> (q int8 [rows, K], scale fp32 [rows])."""
    if w.dim() != 2 or w.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("expected a 2-d fp32 or bf16 matrix")
    q = torch.empty(w.shape, dtype=torch.int8, device=w.device)
    s = torch.empty(w.shape[0], dtype=torch.float32, device=w.device)
    _check(lib().ss_quantize_rows_int8(_dev(w), SS_DTYPE_BF16 if w.dtype == torch.bfloat16 else SS_DTYPE_F32, w.shape[0], w.shape[1],
                                       _dev(q), _dev(s), _stream(stream)))
    return q, s


def ss_quantize_rows_int4(w, stream=None):
    """int4 with group scales of a device matrix [rows, K] (fp32 or bf16, K % 128 == 0) ->
    (packed uint8 [rows, K/2], scale fp32 [K/128, rows])."""
    if w.dim() != 2 or w.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("expected a 2-d fp32 or bf16 matrix")
    q = torch.empty((w.shape[0], w.shape[1] // 2), dtype=torch.uint8, device=w.device)
    s = torch.empty((max(1, w.shape[1] // 128), w.shape[0]), dtype=torch.float32, device=w.device)
    _check(lib().ss_quantize_rows_int4(_dev(w), SS_DTYPE_BF16 if w.dtype == torch.bfloat16 else SS_DTYPE_F32, w.shape[0], w.shape[1],
                                       _dev(q), _dev(s), _stream(stream)))
    return q, s


def ss_probe_read_bandwidth(buf, iters=20, stream=None):
    """GB/s a dependency-free read kernel reaches over the device tensor `buf` (read once per launch)."""
    sink = torch.zeros(1, dtype=torch.int32, device=buf.device)
    out = C.c_double(0.0)
    _check(lib().ss_probe_read_bandwidth(_dev(buf), buf.numel() * buf.element_size(), int(iters), _dev(sink), C.byref(out),
                                         _stream(stream)))
    return out.value


def ss_model_set_persistent_options(model: Model, workgroups: int = 0, data_sync: bool = True):
    _check(lib().ss_model_set_persistent_options(model.handle, int(workgroups), int(bool(data_sync))))


def ss_model_set_timeline(model: Model, buf):
    """Development aid: device clock samples of the persistent kernel into `buf` (int64 device tensor, zero-filled)."""
    if buf is None:
        _check(lib().ss_model_set_timeline(model.handle, C.c_void_p(0), 0))
    else:
        _check(lib().ss_model_set_timeline(model.handle, _dev(buf, torch.int64), buf.numel()))


def ss_model_set_wait_limit(model: Model, polls: int):
    _check(lib().ss_model_set_wait_limit(model.handle, int(polls)))


def ss_profile_enable(model: Model, on: bool):
    _check(lib().ss_profile_enable(model.handle, int(bool(on))))


def ss_profile_read(model: Model):
    """-> {class name: (total_ms, launches)} for the launches recorded since profiling was enabled."""
    n = len(PROFILE_CLASSES)
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(lib().ss_profile_read(model.handle, n, ms, cnt))
    return {PROFILE_CLASSES[i]: (ms[i], cnt[i]) for i in range(n)}
