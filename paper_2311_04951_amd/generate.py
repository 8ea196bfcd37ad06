"""Host loops over the C-ABI calls: autoregressive decoding (Section 3, Eq. 1) and speculative
sampling with two KV caches (Sections 3, 4.3, 4.4).  Control flow and buffer plumbing only - every
number is produced by the library's kernels.

Cache bookkeeping of the speculative loop (the answer to Section 4.4's two-caches question): with n
committed tokens both caches hold the first n-1 positions.  K draft calls bring the draft cache to
n-1+K, one verify call brings the target cache to n+K, and after a tokens are accepted both are
rolled back (a length write on the device) to n+a.  When all K are accepted the draft cache is one
row short, so its next call feeds two tokens.
"""
from __future__ import annotations

import time

import torch

from . import (BatchedStepBuffers, KVCache, Model, SpecVerifyError, StepBuffers, ss_device_status, ss_draft_step, ss_greedy_accept, ss_kv_cache_get_len, ss_kv_cache_rollback, ss_kv_cache_set_len, ss_softmax, ss_top_k_filter, ss_top_p_filter,
               ss_speculative_accept, ss_speculative_step, ss_speculative_step_batched, ss_verify_forward)


def _check_status(*models):
    """A decode loop's results are only valid if no kernel flagged anything (a clamped token id, a wait of the
    persistent kernel that gave up): read the status words once, after the loop."""
    for m in models:
        st = ss_device_status(m)
        if st:
            raise SpecVerifyError(-4 if st & 2 else -1, f"device status {st} after a decode loop (bit 0: token id clamped, bit 1: wait gave up)")


def prefill(model: Model, kv: KVCache, tokens, chunk: int = 16):
    """Feeds `tokens` (list of ids, one sequence, batch 1) through the model in chunks of <= 16 rows."""
    dev = torch.device("cuda")
    for i in range(0, len(tokens), chunk):
        t = torch.tensor([tokens[i:i + chunk]], dtype=torch.int32, device=dev)
        ss_verify_forward(model, kv, t, t.shape[1], logits=False)


def autoregressive_generate(target: Model, prompt, n_new: int, temperature: float, u=None, max_seq=None,
                            stats=None, top_p: float = 1.0, top_k: int = 0):
    """One target call per token; the sampled token never leaves the device between steps.  `stats`
    (a dict, optional) receives loop_seconds: the wall time of the decode loop without the prefill.
    top_p < 1: tokens are drawn from the top-p nucleus of every row; top_k >= 1: from its top_k most probable
    tokens (top-k first when both are set; Section 3)."""
    dev = torch.device("cuda")
    V = target.shape.vocab
    kv = KVCache(target, 1, max_seq or (len(prompt) + n_new + 1))
    prefill(target, kv, list(prompt[:-1]))
    buf = torch.empty(n_new + 1, dtype=torch.int32, device=dev)
    buf[0] = int(prompt[-1])
    q = torch.empty(V, dtype=torch.float32, device=dev) if temperature > 0 else None
    ud = None
    if temperature > 0:
        ud = torch.as_tensor(u, dtype=torch.float32).to(dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n_new):
        ss_draft_step(target, kv, buf[i:i + 1], 1, temperature, ud[i:i + 1] if ud is not None else None, q, V,
                      buf[i + 1:i + 2], top_p=top_p, top_k=top_k)
    torch.cuda.synchronize()
    if stats is not None:
        stats["loop_seconds"] = time.perf_counter() - t0
    _check_status(target)
    out = buf[1:].tolist()
    kv.close()
    return out


def speculative_generate(target: Model, draft: Model, prompt, n_new: int, K: int, temperature: float,
                         u_draft=None, u_accept=None, max_seq=None, observer=None, shared_kv=False, top_p: float = 1.0,
                         top_k: int = 0):
    """Returns (tokens[n_new], stats).  u_draft [steps, K], u_accept [steps, K+1] (temperature > 0).
    `observer(dict)` (optional) sees each step's device tensors: draft tokens, q rows, target logits,
    n_accepted, next token; with an observer the step is issued call by call from here, without one
    it is a single ss_speculative_step per step (same calls, same results).
    shared_kv (Section 4.4, for a draft made of the target's first layers): one cache; the draft works in
    its leading layers, the verify pass rewrites the draft's positions, no catch-up call exists.
    top_p < 1 / top_k >= 1: the draft's and the target's rows are both restricted (top-k first, then the top-p
    nucleus; Section 3 names both selection rules) before anything is drawn or compared: the run emits the
    filtered target distribution."""
    if observer is None:
        return _speculative_generate_native(target, draft, prompt, n_new, K, temperature, u_draft, u_accept, max_seq, shared_kv, top_p, top_k)
    dev = torch.device("cuda")
    V = target.shape.vocab
    M = K + 1
    greedy = temperature == 0
    cap = max_seq or (len(prompt) + n_new + K + 2)
    tkv = KVCache(target, 1, cap)
    dkv = tkv if shared_kv else KVCache(draft, 1, cap)
    prefill(target, tkv, list(prompt[:-1]))
    if not shared_kv:
        prefill(draft, dkv, list(prompt[:-1]))
    x = [int(t) for t in prompt]
    n0 = len(x)
    pending = [x[-1]]
    vt = torch.empty((1, M), dtype=torch.int32, device=dev)       # verify rows [x_n, d_1..d_K]
    q = torch.zeros((1, K, V), dtype=torch.float32, device=dev)
    logits = torch.empty((1, M, V), dtype=torch.float32, device=dev)
    p = torch.empty_like(logits)
    na = torch.empty(1, dtype=torch.int32, device=dev)
    nx = torch.empty(1, dtype=torch.int32, device=dev)
    if not greedy:
        ud_all = torch.as_tensor(u_draft, dtype=torch.float32).to(dev)
        ua_all = torch.as_tensor(u_accept, dtype=torch.float32).to(dev)
    accepted = []
    step = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while len(x) - n0 < n_new:
        feed = torch.tensor([pending], dtype=torch.int32, device=dev)
        for i in range(K):
            ss_draft_step(draft, dkv, feed, feed.shape[1], temperature,
                          None if greedy else ud_all[step, i:i + 1], None if greedy else q[0, i], K * V,
                          vt[0, i + 1:i + 2], top_p=top_p, top_k=top_k)
            feed = vt[:, i + 1:i + 2]
        vt[0, 0] = x[-1]
        if shared_kv:
            ss_kv_cache_set_len(tkv, [len(x) - 1])   # the verify pass rewrites the draft's K positions
        ss_verify_forward(target, tkv, vt, M, logits)
        d = vt[:, 1:].contiguous()
        if greedy:
            ss_greedy_accept(logits, d, na, nx)
        else:
            ss_softmax(logits, temperature, p)
            if 1 <= top_k < V:
                ss_top_k_filter(p, top_k, p)
            if top_p < 1.0:
                ss_top_p_filter(p, top_p, p)
            ss_speculative_accept(p, q, d, ua_all[step:step + 1].contiguous(), na, nx)
        if observer is not None:
            observer({"step": step, "draft": d, "q": q, "logits": logits, "p": p, "n_accepted": na, "next": nx})
        host = torch.cat([na, nx, d[0]]).tolist()   # one device-to-host copy per step
        a, y, dl = host[0], host[1], host[2:]
        ss_kv_cache_rollback(tkv, na, M, n_accepted_host=[a])
        if not shared_kv:
            ss_kv_cache_rollback(dkv, na, K, n_accepted_host=[a])   # a = K leaves the draft cache one row short
        x += dl[:a] + [y]
        pending = [y] if (a < K or shared_kv) else [dl[K - 1], y]
        accepted.append(a)
        step += 1
    torch.cuda.synchronize()
    loop_s = time.perf_counter() - t0
    _check_status(target, draft)
    tkv.close()
    if not shared_kv:
        dkv.close()
    return x[n0:n0 + n_new], {"steps": step, "accepted": accepted, "loop_seconds": loop_s,
                              "generated": len(x) - n0}


def _speculative_generate_native(target, draft, prompt, n_new, K, temperature, u_draft, u_accept, max_seq, shared_kv=False,
                                 top_p=1.0, top_k=0):
    dev = torch.device("cuda")
    greedy = temperature == 0
    cap = max_seq or (len(prompt) + n_new + K + 2)
    tkv = KVCache(target, 1, cap)
    dkv = tkv if shared_kv else KVCache(draft, 1, cap)
    prefill(target, tkv, list(prompt[:-1]))
    if not shared_kv:
        prefill(draft, dkv, list(prompt[:-1]))
    buf = StepBuffers(K, target.shape.vocab, int(prompt[-1]), dev)
    ud_all = ua_all = None
    if not greedy:
        ud_all = torch.as_tensor(u_draft, dtype=torch.float32).to(dev).contiguous()
        ua_all = torch.as_tensor(u_accept, dtype=torch.float32).to(dev).contiguous()
    out, accepted = [], []
    step = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while len(out) < n_new:
        a, y, d = ss_speculative_step(target, tkv, draft, dkv, buf, temperature,
                                      None if greedy else ud_all[step], None if greedy else ua_all[step], top_p=top_p, top_k=top_k)
        out += d[:a] + [y]
        accepted.append(a)
        step += 1
    torch.cuda.synchronize()
    loop_s = time.perf_counter() - t0
    _check_status(target, draft)
    tkv.close()
    if not shared_kv:
        dkv.close()
    return out[:n_new], {"steps": step, "accepted": accepted, "loop_seconds": loop_s, "generated": len(out)}


def speculative_generate_batched(target: Model, draft: Model, prompts, n_new: int, K: int, temperature: float,
                                 u_draft=None, u_accept=None, max_seq=None, observer=None, top_p: float = 1.0, top_k: int = 0):
    """Speculative sampling for a batch of sequences that accept different numbers of tokens per step (ragged cache
    lengths, Section 4.4's bookkeeping per sequence): one ss_speculative_step_batched per step until every sequence
    has n_new tokens.  prompts: list of token lists (>= 2 tokens each, any lengths).  u_draft [batch][steps][K],
    u_accept [batch][steps][K+1] (temperature > 0): sequence b consumes row s in its step s, as a single-sequence run
    would.  Returns (list of token lists, stats).  `observer(step, buf, results)` (optional) sees the step's device
    buffers after each step."""
    dev = torch.device("cuda")
    B = len(prompts)
    greedy = temperature == 0
    cap = max_seq or (max(len(p) for p in prompts) + n_new + 2 * K + 20)   # (room for the padding rows of the ragged prefill)
    tkv, dkv = KVCache(target, B, cap), KVCache(draft, B, cap)
    # ragged prefill: sequence by sequence into its own slot of the batched caches (one-sequence views share the buffers)
    for b, pr in enumerate(prompts):
        if len(pr) < 2:
            raise ValueError("a prompt needs at least two tokens")
        for model, kv, upto in ((target, tkv, len(pr) - 1), (draft, dkv, len(pr) - 2)):
            _prefill_slot(model, kv, b, list(pr[:upto]))
    buf = BatchedStepBuffers(B, K, target.shape.vocab, [list(p[-2:]) for p in prompts], dev)
    ud_all = ua_all = None
    if not greedy:
        ud_all = torch.as_tensor(u_draft, dtype=torch.float32).to(dev)      # [B][steps][K]
        ua_all = torch.as_tensor(u_accept, dtype=torch.float32).to(dev)     # [B][steps][K+1]
    out = [[] for _ in range(B)]
    accepted = [[] for _ in range(B)]
    step = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while min(len(o) for o in out) < n_new:
        ud = None if greedy else ud_all[:, step].transpose(0, 1).contiguous()      # [K][B]
        ua = None if greedy else ua_all[:, step].contiguous()                      # [B][K+1]
        res = ss_speculative_step_batched(target, tkv, draft, dkv, buf, temperature, ud, ua, top_p=top_p, top_k=top_k)
        if observer is not None:
            observer(step, buf, res)
        for b, (a, y, d) in enumerate(res):
            out[b] += d[:a] + [y]
            accepted[b].append(a)
        step += 1
    torch.cuda.synchronize()
    loop_s = time.perf_counter() - t0
    _check_status(target, draft)
    tkv.close()
    dkv.close()
    return [o[:n_new] for o in out], {"steps": step, "accepted": accepted, "loop_seconds": loop_s, "generated": [len(o) for o in out]}


def _prefill_slot(model: Model, kv: KVCache, b: int, tokens, chunk: int = 16):
    """Feeds `tokens` of sequence b through the model into slot b of a batched cache: the other sequences take part with
    a padding token and are set back to their lengths afterwards (a length write; their rows are overwritten later)."""
    dev = torch.device("cuda")
    B = kv.batch
    lens = [int(x) for x in ss_kv_cache_get_len(kv).tolist()]
    chunk = max(1, min(chunk, model.max_rows // B))       # every sequence takes part in a call
    for i in range(0, len(tokens), chunk):
        part = tokens[i:i + chunk]
        t = torch.zeros((B, len(part)), dtype=torch.int32, device=dev)
        t[b] = torch.tensor(part, dtype=torch.int32, device=dev)
        ss_verify_forward(model, kv, t, len(part), logits=False)
        lens[b] += len(part)
        ss_kv_cache_set_len(kv, lens)
