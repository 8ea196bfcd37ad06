#!/usr/bin/env python3
"""Benchmark of the verify pass of speculative sampling on one MI355X.

Workload (default): the full 7B-shaped bf16 target (32 layers, d 4096, 32 heads x 128, FFN 11008,
vocab 32000, random init), batch 1, K = 4 draft tokens (5 query rows), prompt of 128 random ids.
A timed "step" is one verify pass: ss_verify_forward over the 5 rows against the KV cache, softmax
of the 5 logit rows, the modified rejection step against the draft's q rows, and the device-side
cache roll-back.  Inputs (weights, cache, draft rows) are resident in HBM before timing starts.
The same run also times the end-to-end speculative loop (K draft steps + verify + accept per
step, draft = the target's first 2 layers + shared norm and head), an autoregressive baseline, a
per-kernel-class event profile for the roofline figure, and the CPU oracle on a bounded sample.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12  # B/s, MI355X published peak
# HBM bytes per launch of the persistent kernel on the default workload: a stored measurement (two rocprofv3 --pmc runs,
# FETCH_SIZE then WRITE_SIZE, each scaled by what the counter reads for a plain 1 GiB device copy), valid for the kernel
# source it was taken on; bench.py reports it only on that workload and names the file it comes from
PERSISTENT_7B_TRAFFIC_BYTES = 13.601e9  # 13.465 GB fetched + 0.136 GB written
PERSISTENT_7B_TRAFFIC_SOURCE = "profiles/verify_pass_7b_persistent_hbm_traffic.txt"
# the same kind of stored measurement for the stand-alone accept workload (the kernels stop reading a sequence's rows at
# its first rejection, so they fetch less than "every logit once") and for the batched long-context pass
ACCEPT_TRAFFIC_BYTES, ACCEPT_TRAFFIC_SOURCE = 366.5e6, "profiles/standalone_accept_hbm_traffic.txt"
GATEUP_TRAFFIC_BYTES, GATEUP_TRAFFIC_SOURCE = 181.4e6, "profiles/verify_pass_7b_per_phase_hbm_traffic.txt"
PER_PHASE_PASS_TRAFFIC_BYTES = 13.495e9  # 13.463 GB fetched + 0.032 GB written over the launches of one pass (same file)
BATCHED_TRAFFIC_BYTES, BATCHED_TRAFFIC_SOURCE = 37.412e9, "profiles/batched_long_context_pass_hbm_traffic.txt"
STORED = " (stored counter measurement of this workload, not taken in this run)"


def check_status(sv, *models):
    """No timing below counts unless the kernels flagged nothing (a clamped token id, a bounded wait that gave up)."""
    for m in models:
        st = sv.ss_device_status(m)
        if st:
            raise RuntimeError(f"device status {st} after a timed loop (bit 0: token id clamped, bit 1: a wait of the persistent kernel gave up)")


def layer_bytes(shape):
    d, F, W = shape.d_model, shape.d_ff, shape.n_heads * shape.head_dim
    return 2 * (3 * W * d + d * W + 3 * d * F)


def verify_pass_bytes(shape, L, M):
    """Algorithmic HBM bytes of one verify pass: every weight once, the KV context once, the new K/V
    rows, the logits."""
    W = shape.n_heads * shape.head_dim
    kv_read = shape.n_layers * 2 * (L + M) * W * 2
    kv_write = shape.n_layers * 2 * M * W * 2
    head = shape.vocab * shape.d_model * 2
    return shape.n_layers * layer_bytes(shape) + head + kv_read + kv_write + M * shape.vocab * 4


def cpu_baseline(si, torch, shape, packed, io, prompt_len, M, seconds_target=10.0):
    """The oracle, as it stands, on bounded samples of the workloads (about 25 s of host time in all):
    whole M-row verify passes of the named model on every host thread (the reported value), the same pass on
    one thread (first layers + LM head, extrapolated by weight bytes), one layer of the single-layer
    workload, and a slice of the stand-alone accept workload."""
    import numpy as np
    import oracle
    d, W = shape.d_model, shape.n_heads * shape.head_dim
    threads = oracle.num_threads()

    def model(n_layers):
        s = si.DecoderShape(**{**shape.as_dict(), "n_layers": n_layers})
        w = {"embed": io["embed"].cpu(), "gf": io["gf"].cpu(), "lm_head": io["lm_head"].cpu(),
             "layers": si.unpack_layers(shape, packed[:n_layers])}
        return s, oracle.Model(s, w)

    def run(n_layers, ctx=prompt_len, rows=M, reps=1):
        s, om = model(n_layers)
        kv = om.new_kv(ctx + rows * reps + 1)
        kv.append_raw(si.kv_context(s, 1, "cpu_ctx", ctx))
        toks = si.token_ids(1, "cpu_toks", (rows,), s.vocab).numpy()
        t0 = time.perf_counter()
        for _ in range(reps):
            om.forward(kv, toks)
        return (time.perf_counter() - t0) / reps

    head_b = shape.vocab * d * 2
    full_b = shape.n_layers * layer_bytes(shape) + head_b

    def sampled(seconds, what):
        """tokens/s of the full pass from a sample that takes about `seconds`"""
        t1 = run(1)
        n = int(max(1, min(shape.n_layers, round(seconds / max(t1, 1e-3)))))
        if n < shape.n_layers:
            t = run(n) if n > 1 else t1
            frac = (n * layer_bytes(shape) + head_b) / full_b
            return M / (t / frac), (f"first {n} of {shape.n_layers} layers + LM head of one {M}-row verify pass against {prompt_len} cached "
                                    f"positions ({t:.1f} s {what}), extrapolated by weight bytes to the full pass")
        t_one = run(shape.n_layers)
        reps = int(max(1, min(20, round(seconds / max(t_one, 1e-3)))))
        t_tot = t_one + sum(run(shape.n_layers) for _ in range(reps - 1))
        return M * reps / t_tot, (f"{reps} full {M}-row verify passes (all {shape.n_layers} layers + LM head) against {prompt_len} cached "
                                  f"positions, {t_tot:.1f} s {what}")

    value, sample = sampled(seconds_target, f"on {threads} threads")
    out = {"value": value, "unit": "tokens/s", "cores": threads, "kind": "oracle", "sample": sample}
    oracle.set_num_threads(1)
    try:
        v1, s1 = sampled(5.0, "on 1 thread")
    finally:
        oracle.set_num_threads(threads)
    out["single_thread"] = {"value": v1, "unit": "tokens/s", "cores": 1, "sample": s1}
    # a draft step of the early-exit draft (first 2 layers + LM head, one row), the call a speculative step makes K times
    nd = min(2, shape.n_layers)
    out["draft_step"] = {"ms": 1e3 * run(nd, rows=1, reps=3), "cores": threads, "sample": f"3 one-row passes of the first {nd} layers + LM head"}
    # the single-layer workload: one layer, M rows against 1024 cached positions (layers_forward: no embedding, no head)
    s1l, om = model(1)
    kv = om.new_kv(1024 + M + 1)
    kv.append_raw(si.kv_context(s1l, 1, "cpu_ctx1024", 1024))
    h = si.normal(7, "cpu_lp_h", (M, d), 1.0).numpy()
    reps, t0 = 0, time.perf_counter()
    while reps < 3 or (time.perf_counter() - t0 < 2.0 and reps < 50):
        kv.set_len(1024)
        om.layers_forward(kv, h)
        reps += 1
    t_layer = (time.perf_counter() - t0) / reps
    out["layer_pass"] = {"us_per_layer": t_layer * 1e6, "cores": threads,
                         "sample": f"{reps} passes of one 7B-shaped layer, {M} rows against 1024 cached positions"}
    # the stand-alone accept workload, a slice of its batch: softmax of every row at the temperature, then the rejection step
    Bs, K, V, T = 4, 8, 128256, 0.8
    pl, ql, u, ud = si.accept_workload(41, Bs, K, V)
    t0 = time.perf_counter()
    p = oracle.softmax(pl.numpy(), T)
    q = oracle.softmax(ql.numpy(), T)
    dtok = np.array([[oracle.sample(q[b, i], float(ud[b, i])) for i in range(K)] for b in range(Bs)], dtype=np.int32)
    t_q = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.speculative_accept(p, q, dtok, u.numpy())
    t_acc = time.perf_counter() - t0
    # the tiny fp32 pair end to end: 64 tokens, K = 4, temperature 1 and greedy (the configuration the oracle finishes in seconds)
    tw = si.decoder_weights(si.TINY_TARGET, 0)
    ot, od = oracle.Model(si.TINY_TARGET, tw), oracle.Model(si.TINY_DRAFT, si.decoder_weights(si.TINY_DRAFT, 100))
    tp = si.token_ids(0, "prompt", (32,), si.TINY_TARGET.vocab).numpy().tolist()
    t0 = time.perf_counter()
    _, st_s = oracle.speculative_generate(ot, od, tp, 64, 4, 1.0, si.uniforms(0, "ud", (64, 4)).numpy(), si.uniforms(0, "ua", (64, 5)).numpy())
    t_s = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.speculative_generate(ot, od, tp, 64, 4, 0.0)
    t_g = time.perf_counter() - t0
    out["tiny_pair"] = {"sampled_tokens_per_s": 64 / t_s, "greedy_tokens_per_s": 64 / t_g, "cores": threads,
                        "sample": f"speculative loop of the tiny fp32 pair, prompt 32, 64 tokens, K 4: {t_s:.2f} s at temperature 1 "
                                  f"({st_s['steps']} steps), {t_g:.2f} s greedy"}
    out["standalone_accept"] = {"us_per_sequence": (t_q + t_acc) / Bs * 1e6, "cores": threads,
                                "sample": f"{Bs} of the workload's 64 sequences (K {K}, vocab {V}): softmax of the {2 * K + 1} rows per sequence, "
                                          f"the draft's samples and the rejection step; {t_q + t_acc:.1f} s"}
    return out


def standalone_accept(si, sv, torch, dev, iters=40):
    """The stand-alone accept workload (batch 64, K 8, vocab 128256, fp32 logits, temperature 0.8):
    time of ss_speculative_accept_logits against the algorithmic bytes of reading every logit once."""
    B, K, V, T = 64, 8, 128256, 0.8
    sets = []
    for s in range(2):  # two input sets, alternated (1.1 GB together: beyond the 256 MB last-level cache)
        pl, ql, u, ud = si.accept_workload(41 + s, B, K, V, device=dev)
        q = sv.ss_softmax(ql, T)
        d = torch.empty((B, K), dtype=torch.int32, device=dev)
        zf, zi = torch.zeros(1, device=dev), torch.zeros(1, dtype=torch.int32, device=dev)
        for i in range(K):  # draft tokens ~ q (the K = 0 case of the accept entry is a plain sample)
            _, tok = sv.ss_speculative_accept(q[:, i].contiguous()[:, None], zf, zi, ud[:, i:i + 1].contiguous())
            d[:, i] = tok
        del q
        sets.append((pl, ql, d, u))
    na = torch.empty(B, dtype=torch.int32, device=dev)
    nx = torch.empty(B, dtype=torch.int32, device=dev)

    def run(i):
        pl, ql, d, u = sets[i % len(sets)]
        sv.ss_speculative_accept_logits(pl, ql, T, d, u, n_accepted=na, next_token=nx)

    for i in range(4):
        run(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(iters):
        run(i)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / iters
    nbytes = (2 * K + 1) * B * V * 4
    return {"workload": f"batch {B}, K {K}, vocab {V}, fp32 logits, temperature {T}", "us_per_call": dt * 1e6,
            "algorithmic_bytes": nbytes, "GBps": nbytes / dt / 1e9, "frac_of_hbm_peak": nbytes / dt / HBM_PEAK,
            "algorithmic_bytes_note": "every logit of p and q once; the kernels read a sequence's rows only up to its first rejection",
            "traffic": ACCEPT_TRAFFIC_BYTES, "traffic_source": ACCEPT_TRAFFIC_SOURCE + STORED,
            "traffic_GBps": ACCEPT_TRAFFIC_BYTES / dt / 1e9, "mean_accepted": float(na.float().mean())}


def layer_pass(si, sv, torch, dev, target, shape, iters=20, L=1024, M=5):
    """The one-layer workload at full width (5 query rows against 1024 cached positions), measured over the
    target's distinct layers in turn (every layer has its own weights and cache, 13 GB in all, so
    nothing is served from the last-level cache): median time of ss_decoder_layers_forward per layer."""
    kv = sv.KVCache(target, 1, L + 64)
    W = shape.n_heads * shape.head_dim
    for l in range(shape.n_layers):
        k = si.normal(7, f"lp_k{l}", (L, W), 1.0, device=dev, dtype=torch.bfloat16)
        v = si.normal(7, f"lp_v{l}", (L, W), 1.0, device=dev, dtype=torch.bfloat16)
        sv.ss_kv_cache_append(kv, l, 0, 0, k, v)
    h0 = si.normal(7, "lp_h", (M, shape.d_model), 1.0, device=dev)
    times = []
    for it in range(iters + 3):
        sv.ss_kv_cache_set_len(kv, [L])
        h = h0.clone()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        sv.ss_decoder_layers_forward(target, kv, h, 1, M)
        torch.cuda.synchronize()
        if it >= 3:
            times.append((time.perf_counter() - t0) / shape.n_layers)
    kv.close()
    times.sort()
    t = times[len(times) // 2]
    nbytes = layer_bytes(shape) + 2 * (L + M) * W * 2 + 2 * M * W * 2
    return {"workload": f"one 7B-shaped bf16 layer, {M} query rows, {L} cached positions; median over {iters} passes through "
                        f"{shape.n_layers} distinct layers", "us_per_layer": t * 1e6, "algorithmic_bytes_per_layer": nbytes,
            "GBps": nbytes / t / 1e9, "frac_of_hbm_peak": nbytes / t / HBM_PEAK}


def int8_weights_leg(si, sv, torch, gen, dev, target, persistent, shape, packed, io, prompt, K, steps, bits=8):
    """The verify pass with weight-only quantised matrices (the quantised model the paper assumes; bits = 8: one
    scale per output row, bits = 4: one scale per group of 128 entries along K): the same 7B-shaped weights
    quantised by the library, K + 1 rows per pass, one launch per phase (the persistent kernel streams bf16
    matrices only), beside the bf16 model on the same per-phase path; then the speculative loop and the
    autoregressive baseline on the quantised pair."""
    M = K + 1
    qkw = {"int4_weights": True} if bits == 4 else {"int8_weights": True}
    t8 = sv.Model(shape, io, max_rows=16, max_pos=4096, packed_layers=packed, **qkw)
    d8 = sv.Model(si.DecoderShape(**{**shape.as_dict(), "n_layers": min(2, shape.n_layers)}),
                  {"embed": io["embed"], "gf": io["gf"], "lm_head": t8.lm_head, "s_head": t8.s_head},
                  max_rows=16, max_pos=4096, packed_layers=t8.layers[:min(2, shape.n_layers)], **qkw)
    vt = si.token_ids(3, "int8_rows", (1, M), shape.vocab).to(torch.int32).to(dev)
    zero = torch.zeros(1, dtype=torch.int32, device=dev)
    logits = torch.empty((1, M, shape.vocab), dtype=torch.float32, device=dev)

    def timed(model):
        kv = sv.KVCache(model, 1, len(prompt) + M * (steps + 3) + 16)   # the host's bound on the length grows by M per pass
        gen.prefill(model, kv, prompt[:-1])
        for it in range(steps + 3):
            if it == 3:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            sv.ss_verify_forward(model, kv, vt, M, logits)
            sv.ss_kv_cache_rollback(kv, zero, M)          # commits one row: the context grows by one per pass
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        kv.close()
        return dt

    t_int8 = timed(t8)
    sv.ss_model_set_persistent(target, False)
    t_bf16 = timed(target)
    sv.ss_model_set_persistent(target, persistent)
    W = shape.n_heads * shape.head_dim
    L = len(prompt) + steps // 2
    wbytes16 = shape.n_layers * layer_bytes(shape) + shape.vocab * shape.d_model * 2                # the matrices in bf16
    if bits == 4:
        nscale = wbytes16 // 2 // 128                                                                 # one fp32 scale per 128 entries
    else:
        nscale = shape.n_layers * (3 * W + 2 * shape.d_model + 2 * shape.d_ff) + shape.vocab         # one fp32 scale per matrix row
    nbytes = wbytes16 * bits // 16 + 4 * nscale + shape.n_layers * 2 * (L + 2 * M) * W * 2 + M * shape.vocab * 4
    out = {"workload": f"7B-shaped target with int{bits} matrices ({shape.n_layers} layers), batch 1, K={K}, KV context ~{L}, "
                       "one launch per phase",
           "ms_per_pass": 1e3 * t_int8, "verify_pass_tokens_per_s": M / t_int8, "algorithmic_bytes": nbytes,
           "GBps": nbytes / t_int8 / 1e9, "frac_of_hbm_peak": nbytes / t_int8 / HBM_PEAK,
           "bf16_same_path_ms_per_pass": 1e3 * t_bf16, "speedup_vs_bf16_same_path": t_bf16 / t_int8}
    n_new = 96
    ud, ua = si.uniforms(2, "ud8", (n_new, K)), si.uniforms(2, "ua8", (n_new, K + 1))
    _, st = gen.speculative_generate(t8, d8, prompt, n_new, K, 1.0, ud, ua)
    ar = {}
    gen.autoregressive_generate(t8, prompt, 48, 1.0, si.uniforms(2, "uar8", (48,)), stats=ar)
    out["end_to_end"] = {"accepted_tokens_per_s": st["generated"] / st["loop_seconds"],
                         "mean_accepted_per_step": sum(st["accepted"]) / max(1, st["steps"]),
                         "ms_per_step": 1e3 * st["loop_seconds"] / max(1, st["steps"]),
                         "autoregressive_tokens_per_s": 48 / ar["loop_seconds"]}
    d8.close()
    t8.close()
    return out


def paper_pair_leg(si, sv, torch, gen, dev, prompt_len=128, n_new=96, K=5):
    """The size ratio of the paper's own experiment (Section 6: a 12B target with a 3B draft, K = 5) on
    Llama-shaped stand-ins with random weights: a 13B-shaped target (40 layers, d 5120, 40 heads, FFN 13824)
    and a separate 3B-shaped draft (28 layers, d 3072, 24 heads, FFN 8192) with its own cache.  Random
    weights make the draft useless as a predictor, so the figures are costs per step, not the paper's speed-up."""
    ts = si.DecoderShape(40, 5120, 40, 128, 13824, 32000, dtype="bf16")
    ds = si.DecoderShape(28, 3072, 24, 128, 8192, 32000, dtype="bf16")
    _, tp, tio = si.packed_decoder(ts, 11, dev)
    _, dp, dio = si.packed_decoder(ds, 12, dev)
    target = sv.Model(ts, tio, max_rows=16, max_pos=1024, packed_layers=tp)
    draft = sv.Model(ds, dio, max_rows=16, max_pos=1024, packed_layers=dp)
    prompt = si.token_ids(11, "prompt", (prompt_len,), ts.vocab).tolist()
    ud, ua = si.uniforms(11, "ud", (n_new, K)), si.uniforms(11, "ua", (n_new, K + 1))
    gen.speculative_generate(target, draft, prompt, 8, K, 1.0, ud[:8], ua[:8])          # warm-up
    _, st = gen.speculative_generate(target, draft, prompt, n_new, K, 1.0, ud, ua)
    ar = {}
    n_ar = 32
    gen.autoregressive_generate(target, prompt, n_ar, 1.0, si.uniforms(11, "uar", (n_ar,)), stats=ar)
    dr = {}
    gen.autoregressive_generate(draft, prompt, n_ar, 1.0, si.uniforms(12, "uar", (n_ar,)), stats=dr)
    t_step = st["loop_seconds"] / max(1, st["steps"])
    t_target1, t_draft1 = ar["loop_seconds"] / n_ar, dr["loop_seconds"] / n_ar
    tb = ts.n_layers * layer_bytes(ts) + ts.vocab * ts.d_model * 2
    db = ds.n_layers * layer_bytes(ds) + ds.vocab * ds.d_model * 2
    out = {"workload": f"13B-shaped target ({tb / 1e9:.1f} GB) + separate 3B-shaped draft ({db / 1e9:.1f} GB), bf16, batch 1, K={K}, "
                       f"T=1, prompt {prompt_len}, {n_new} tokens, random weights",
           "accepted_tokens_per_s": st["generated"] / st["loop_seconds"], "ms_per_step": 1e3 * t_step,
           "mean_accepted_per_step": sum(st["accepted"]) / max(1, st["steps"]),
           "autoregressive_tokens_per_s": 1.0 / t_target1, "target_ms_per_token": 1e3 * t_target1,
           "draft_ms_per_token": 1e3 * t_draft1,
           "target_GBps": tb / t_target1 / 1e9, "draft_GBps": db / t_draft1 / 1e9,
           # accepted draft tokens per step at which a step (K draft tokens + one verify pass) yields as many tokens per second as one target token per pass
           "break_even_accepted_per_step": t_step / t_target1 - 1.0,
           "parity_note": "timing only at this depth: these two widths are compared with the oracle on one layer each "
                          "(tests/test_gpu_forward.py, reduced depth), not as 40- and 28-layer models"}
    for obj in (target, draft):
        obj.close()
    return out


def batched_workload(si, sv, torch, dev, shape, packed, io, iters=5, B=8, L=4096, M=9, int8=True):
    """The batched long-context workload: 8 sequences with 4096 cached positions each, K = 8 (72 rows per
    verify pass, one launch per phase: wide GEMMs and split-KV attention)."""
    m = sv.Model(shape, io, max_rows=B * M, max_pos=L + 512, packed_layers=packed)
    kv = sv.KVCache(m, B, L + 512)
    W = shape.n_heads * shape.head_dim
    for l in range(shape.n_layers):
        k = si.normal(5, f"bw_k{l}", (L, W), 1.0, device=dev, dtype=torch.bfloat16)
        v = si.normal(5, f"bw_v{l}", (L, W), 1.0, device=dev, dtype=torch.bfloat16)
        for b in range(B):
            sv.ss_kv_cache_append(kv, l, b, 0, k, v)
    toks = si.token_ids(0, "bw_t", (B, M), shape.vocab).to(dev).int()
    logits = torch.empty((B, M, shape.vocab), device=dev)

    def run():
        sv.ss_kv_cache_set_len(kv, [L] * B)
        sv.ss_verify_forward(m, kv, toks, M, logits)

    for _ in range(2):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        run()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / iters
    sv.ss_profile_enable(m, True)
    for _ in range(3):
        run()
    torch.cuda.synchronize()
    prof = sv.ss_profile_read(m)
    nbytes = shape.n_layers * layer_bytes(shape) + shape.vocab * shape.d_model * 2 + shape.n_layers * B * 2 * (L + M) * W * 2
    check_status(sv, m)
    out = {"workload": f"batch {B}, context {L}, K {M - 1} ({B * M} rows per pass), {shape.n_layers} layers, one launch per phase", "ms_per_pass": dt * 1e3,
           "rows_per_s": B * M / dt, "algorithmic_bytes": nbytes, "GBps": nbytes / dt / 1e9, "frac_of_hbm_peak": nbytes / dt / HBM_PEAK,
           "roofline": {"bound": "hbm", "achieved": nbytes / dt / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": nbytes / dt / HBM_PEAK,
                        "traffic": BATCHED_TRAFFIC_BYTES if (shape.n_layers == 32 and B == 8 and L == 4096 and M == 9) else None,
                        "traffic_source": BATCHED_TRAFFIC_SOURCE + STORED,
                        "note": "whole pass (weights once, every sequence's KV context once) over its host-timed duration"},
           "class_ms_per_pass": {k: round(ms / 3, 3) for k, (ms, n) in prof.items() if n}}
    # end to end on this workload: speculative steps of all sequences at once (ss_speculative_step_batched), early-exit draft,
    # T = 1; the sequences start at ragged lengths and accept different numbers of tokens per step
    K = M - 1
    dshape = si.DecoderShape(**{**shape.as_dict(), "n_layers": min(2, shape.n_layers)})
    dm = sv.Model(dshape, io, max_rows=2 * B, max_pos=L + 512, packed_layers=packed[:dshape.n_layers])
    dkv = sv.KVCache(dm, B, L + 512)
    for l in range(dshape.n_layers):
        k = si.normal(5, f"bw_k{l}", (L, W), 1.0, device=dev, dtype=torch.bfloat16)
        v = si.normal(5, f"bw_v{l}", (L, W), 1.0, device=dev, dtype=torch.bfloat16)
        for b in range(B):
            sv.ss_kv_cache_append(dkv, l, b, 0, k, v)
    lens = [L - 7 * b for b in range(B)]
    n_steps = 12
    buf = sv.BatchedStepBuffers(B, K, shape.vocab, si.token_ids(2, "bw_feed", (B, 2), shape.vocab).tolist(), dev)
    ud = si.uniforms(2, "bw_ud", (n_steps + 2, K, B)).to(dev)
    ua = si.uniforms(2, "bw_ua", (n_steps + 2, B, K + 1)).to(dev)
    sv.ss_kv_cache_set_len(kv, lens)
    sv.ss_kv_cache_set_len(dkv, [x - 1 for x in lens])
    tokens = accepted = 0
    for it in range(n_steps + 2):
        if it == 2:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        res = sv.ss_speculative_step_batched(m, kv, dm, dkv, buf, 1.0, ud[it], ua[it])
        if it >= 2:
            tokens += sum(a + 1 for a, _, _ in res)
            accepted += sum(a for a, _, _ in res)
    torch.cuda.synchronize()
    dts = (time.perf_counter() - t0) / n_steps
    check_status(sv, m, dm)
    out["end_to_end"] = {"workload": f"{n_steps} speculative steps of {B} sequences at once (K {K}, T 1, early-exit draft of {dshape.n_layers} layers, ragged lengths from {lens[-1]} to {lens[0]})",
                         "ms_per_step": dts * 1e3, "accepted_tokens_per_s": tokens / (dts * n_steps),
                         "mean_accepted_per_step_and_sequence": accepted / (n_steps * B),
                         "final_lengths": [int(x) for x in sv.ss_kv_cache_get_len(kv).tolist()]}
    dkv.close()
    dm.close()
    m.close()
    if int8:
        # the same pass with quantised matrices (the KV cache stays bf16: it is most of this workload's bytes); int4 streams
        # its matrices once per 16 rows (five times here)
        wb16 = shape.n_layers * layer_bytes(shape) + shape.vocab * shape.d_model * 2
        for name, kw, wbytes in (("int8_weights", {"int8_weights": True}, wb16 // 2), ("int4_weights", {"int4_weights": True}, wb16 // 4 + wb16 // 2 // 128 * 4)):
            m = sv.Model(shape, io, max_rows=B * M, max_pos=L + 512, packed_layers=packed, **kw)
            for _ in range(2):
                run()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(iters):
                run()
            torch.cuda.synchronize()
            dtq = (time.perf_counter() - t0) / iters
            sv.ss_profile_enable(m, True)
            for _ in range(3):
                run()
            torch.cuda.synchronize()
            prof = sv.ss_profile_read(m)
            check_status(sv, m)
            nbq = nbytes - wb16 + wbytes
            out[name] = {"ms_per_pass": dtq * 1e3, "rows_per_s": B * M / dtq, "algorithmic_bytes": nbq, "GBps": nbq / dtq / 1e9,
                         "frac_of_hbm_peak": nbq / dtq / HBM_PEAK,
                         "class_ms_per_pass": {k: round(ms / 3, 3) for k, (ms, n) in prof.items() if n}}
            m.close()
    kv.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--K", type=int, default=4)
    ap.add_argument("--layers", type=int, default=32, help="decoder layers (32 = the named workload)")
    ap.add_argument("--gen-tokens", type=int, default=256)
    ap.add_argument("--persistent", type=int, default=0,
                    help="0 (the library's default): one launch per phase, 1: the forward as the persistent single-launch kernel")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-e2e", action="store_true")
    ap.add_argument("--no-accept-workload", action="store_true", help="skip the stand-alone accept workload leg")
    ap.add_argument("--no-int8-leg", action="store_true", help="skip the weight-only int8 and int4 legs")
    ap.add_argument("--no-paper-pair", action="store_true", help="skip the 13B/3B-shaped target/draft pair (the paper's size ratio)")
    ap.add_argument("--no-layer-pass", action="store_true", help="skip the one-layer leg (5 rows, 1024 cached positions)")
    ap.add_argument("--no-batched-workload", action="store_true",
                    help="skip the batched long-context workload (8 x 4096 positions, 72 rows per pass; 20 GB more)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of 1 GiB five times (a kernel of known traffic, for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2311_04951_amd as sv
    import seeded_inputs as si
    from paper_2311_04951_amd import generate as gen

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, M, T = args.K, args.K + 1, 1.0
    prompt_len = 128
    shape, packed, io = si.packed_7b(0, args.layers, dev)
    max_pos = 4096
    target = sv.Model(shape, io, max_rows=16, max_pos=max_pos, packed_layers=packed)
    dshape = si.DecoderShape(**{**shape.as_dict(), "n_layers": min(2, args.layers)})
    draft = sv.Model(dshape, io, max_rows=16, max_pos=max_pos, packed_layers=packed[:dshape.n_layers])
    sv.ss_model_set_persistent(target, bool(args.persistent))
    sv.ss_model_set_persistent(draft, bool(args.persistent))
    V = shape.vocab
    prompt = si.token_ids(0, "prompt", (prompt_len,), V).tolist()

    # ---- end-to-end speculative loop and autoregressive baseline (also warms everything up)
    e2e = None
    if not args.no_e2e:
        n_new = args.gen_tokens
        ud = si.uniforms(0, "ud", (n_new, K))
        ua = si.uniforms(0, "ua", (n_new, K + 1))
        toks, st = gen.speculative_generate(target, draft, prompt, n_new, K, T, ud, ua)
        ar_stats = {}
        n_ar = min(64, n_new)
        gen.autoregressive_generate(target, prompt, n_ar, T, si.uniforms(0, "uar", (n_ar,)), stats=ar_stats)
        e2e = {"accepted_tokens_per_s": st["generated"] / st["loop_seconds"], "generated": st["generated"],
               "steps": st["steps"], "mean_accepted_per_step": sum(st["accepted"]) / max(1, st["steps"]),
               "ms_per_step": 1e3 * st["loop_seconds"] / max(1, st["steps"]),
               "autoregressive_tokens_per_s": n_ar / ar_stats["loop_seconds"],
               "speedup_vs_autoregressive": (st["generated"] / st["loop_seconds"]) / (n_ar / ar_stats["loop_seconds"]),
               "temperature": T, "K": K, "draft": f"first {dshape.n_layers} target layers + shared norm and LM head"}
        # the other draft lengths of the workload (K = 2, 4, 8), sampled and greedy, on a shorter run
        sweep = {}
        n_sw = min(96, n_new)
        for k2 in (2, 4, 8):
            for t2 in (1.0, 0.0):
                _, s2 = gen.speculative_generate(target, draft, prompt, n_sw, k2, t2, si.uniforms(1, f"ud{k2}", (n_sw, k2)),
                                                 si.uniforms(1, f"ua{k2}", (n_sw, k2 + 1)))
                sweep[f"K{k2}_{'greedy' if t2 == 0.0 else 'T1'}"] = {
                    "accepted_tokens_per_s": round(s2["generated"] / s2["loop_seconds"], 1),
                    "mean_accepted_per_step": round(sum(s2["accepted"]) / max(1, s2["steps"]), 3),
                    "ms_per_step": round(1e3 * s2["loop_seconds"] / max(1, s2["steps"]), 3)}
        e2e["by_draft_length"] = sweep
        # top-p selection (nucleus 0.9) on both models' rows
        n_tp = min(96, n_new)
        _, s4 = gen.speculative_generate(target, draft, prompt, n_tp, K, T, ud[:n_tp], ua[:n_tp], top_p=0.9)
        e2e["top_p_0.9"] = {"accepted_tokens_per_s": s4["generated"] / s4["loop_seconds"],
                            "mean_accepted_per_step": sum(s4["accepted"]) / max(1, s4["steps"]),
                            "ms_per_step": 1e3 * s4["loop_seconds"] / max(1, s4["steps"])}
        # the same loop with one cache shared by both models (the draft works in the target's first layers' cache)
        _, s3 = gen.speculative_generate(target, draft, prompt, n_new, K, T, ud, ua, shared_kv=True)
        e2e["shared_kv_cache"] = {"accepted_tokens_per_s": s3["generated"] / s3["loop_seconds"], "steps": s3["steps"],
                                  "mean_accepted_per_step": sum(s3["accepted"]) / max(1, s3["steps"]),
                                  "ms_per_step": 1e3 * s3["loop_seconds"] / max(1, s3["steps"])}

        # The same loop against a target whose layers behind the draft's two write only a tenth as much into the residual
        # stream: the early-exit draft then predicts its target about as well as a trained draft does, which random
        # weights cannot show (same shapes, same kernels, same bytes per pass; only the acceptance changes).
        damped = si.damp_late_layers(packed, dshape.n_layers, 0.1)
        t2 = sv.Model(shape, io, max_rows=16, max_pos=max_pos, packed_layers=damped)
        sv.ss_model_set_persistent(t2, bool(args.persistent))
        good = {}
        n_gd = min(128, n_new)
        ar2 = {}
        gen.autoregressive_generate(t2, prompt, 48, T, si.uniforms(4, "uar", (48,)), stats=ar2)
        for k2, t2v in ((4, 1.0), (8, 1.0), (4, 0.0)):
            _, s5 = gen.speculative_generate(t2, draft, prompt, n_gd, k2, t2v, si.uniforms(4, f"ud{k2}", (n_gd, k2)), si.uniforms(4, f"ua{k2}", (n_gd, k2 + 1)))
            good[f"K{k2}_{'greedy' if t2v == 0.0 else 'T1'}"] = {
                "accepted_tokens_per_s": round(s5["generated"] / s5["loop_seconds"], 1),
                "mean_accepted_per_step": round(sum(s5["accepted"]) / max(1, s5["steps"]), 3),
                "ms_per_step": round(1e3 * s5["loop_seconds"] / max(1, s5["steps"]), 3),
                "speedup_vs_autoregressive": round((s5["generated"] / s5["loop_seconds"]) / (48 / ar2["loop_seconds"]), 3)}
        good["autoregressive_tokens_per_s"] = round(48 / ar2["loop_seconds"], 1)
        good["workload"] = ("the 7B-shaped target with the O and down projections of layers 2..31 scaled by 0.1 (synthetic stand-in for a "
                            "draft that predicts its target), same early-exit draft")
        e2e["good_draft"] = good
        check_status(sv, t2, draft)
        t2.close()
        del damped

    # ---- state for the verify-pass legs: prompt in the cache, real draft rows from the draft model
    total_steps = args.warmup + 2 * args.steps + 4
    tkv = sv.KVCache(target, 1, prompt_len + M * total_steps + 16)
    dkv = sv.KVCache(draft, 1, prompt_len + K + 16)
    gen.prefill(target, tkv, prompt[:-1])
    gen.prefill(draft, dkv, prompt[:-1])
    vt = torch.empty((1, M), dtype=torch.int32, device=dev)
    vt[0, 0] = prompt[-1]
    q = torch.zeros((1, K, V), dtype=torch.float32, device=dev)
    udd = si.uniforms(0, "bench_ud", (K,)).to(dev)
    feed = vt[:, 0:1]
    for i in range(K):
        sv.ss_draft_step(draft, dkv, feed, 1, T, udd[i:i + 1], q[0, i], K * V, vt[0, i + 1:i + 2])
        feed = vt[:, i + 1:i + 2]
    d = vt[:, 1:].contiguous()
    u = si.uniforms(0, "bench_ua", (total_steps, K + 1)).to(dev)
    logits = torch.empty((1, M, V), dtype=torch.float32, device=dev)
    p = torch.empty_like(logits)
    na = torch.empty(1, dtype=torch.int32, device=dev)
    nx = torch.empty(1, dtype=torch.int32, device=dev)
    counter = [0]

    def verify_step():
        i = counter[0]
        counter[0] += 1
        sv.ss_verify_forward(target, tkv, vt, M, logits)
        sv.ss_softmax(logits, T, p)
        sv.ss_speculative_accept(p, q, d, u[i:i + 1], na, nx)
        sv.ss_kv_cache_rollback(tkv, na, M)

    for _ in range(args.warmup):
        verify_step()
    torch.cuda.synchronize()
    L_start = int(sv.ss_kv_cache_get_len(tkv)[0])
    t0 = time.perf_counter()
    for _ in range(args.steps):
        verify_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    L_end = int(sv.ss_kv_cache_get_len(tkv)[0])
    check_status(sv, target, draft)
    ms_per_step = 1e3 * dt / args.steps
    value = M * args.steps / dt
    L_mean = 0.5 * (L_start + L_end)
    pass_bytes = verify_pass_bytes(shape, L_mean, M)

    # ---- the same steps again with an event pair around every forward-path launch
    sv.ss_profile_enable(target, True)
    for _ in range(args.steps):
        verify_step()
    torch.cuda.synchronize()
    prof = sv.ss_profile_read(target)
    sv.ss_profile_enable(target, False)
    check_status(sv, target)
    classes = {k: {"avg_us": 1e3 * ms / max(1, n), "launches_per_step": n / args.steps} for k, (ms, n) in prof.items() if n}
    if "verify_persistent" in classes:
        # the whole forward of a verify pass is one launch of the persistent kernel
        vp = classes["verify_persistent"]
        k_bytes = pass_bytes
        k_name = f"verify_persistent_kernel<bf16> (embedding, {shape.n_layers} layers, LM head: one launch per verify pass)"
        k_us = vp["avg_us"]
    else:
        gu = classes["gateup_gemm"]
        k_bytes = 2 * shape.d_ff * shape.d_model * 2          # W_gate | W_up streamed once per launch
        k_name = "gemm_kernel<bf16, SWIGLU> (gate/up projection, 42.8% of the pass's bytes)"
        k_us = gu["avg_us"]
    achieved = k_bytes / (k_us * 1e-6) / 1e9
    # HBM bytes per launch from the FETCH_SIZE and WRITE_SIZE counters of two rocprofv3 --pmc runs, each scaled by
    # what the same counter reads for a plain 1 GiB device copy (profiles/verify_pass_7b_persistent_hbm_traffic.txt,
    # profiles/verify_pass_7b_per_phase_hbm_traffic.txt); measurements of the default workload only
    named = args.layers == 32 and K == 4
    if "verify_persistent" in classes:
        traffic, traffic_src = (PERSISTENT_7B_TRAFFIC_BYTES, PERSISTENT_7B_TRAFFIC_SOURCE) if named else (None, None)
    else:
        traffic, traffic_src = (GATEUP_TRAFFIC_BYTES, GATEUP_TRAFFIC_SOURCE) if named else (None, None)
    roofline = {"bound": "hbm", "kernel": k_name, "achieved": achieved, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "frac": achieved / (HBM_PEAK / 1e9), "traffic": traffic,
                "traffic_source": (traffic_src + STORED) if traffic else None,
                "algorithmic_bytes_per_launch": k_bytes, "avg_launch_us": k_us,
                # the whole verify pass (every launch of it) over its host-timed duration: the figure to set beside the
                # dominant kernel's, and the one that compares with a single-launch pass
                "whole_pass": {"algorithmic_bytes": pass_bytes, "ms": 1e3 * dt / args.steps,
                               "GBps": pass_bytes / (dt / args.steps) / 1e9, "frac": pass_bytes / (dt / args.steps) / HBM_PEAK,
                               "traffic": ((PERSISTENT_7B_TRAFFIC_BYTES if "verify_persistent" in classes else PER_PHASE_PASS_TRAFFIC_BYTES) if named else None),
                               "traffic_source": (((PERSISTENT_7B_TRAFFIC_SOURCE if "verify_persistent" in classes else GATEUP_TRAFFIC_SOURCE) + STORED) if named else None),
                               "note": "the timed step also holds softmax, the rejection step and the roll-back (about 40 us)"}}
    # what a dependency-free read kernel reaches on this machine over a 2 GiB buffer (beyond the last-level cache):
    # the practical ceiling beside the nominal peak
    probe_buf = torch.empty(1 << 29, dtype=torch.float32, device=dev).fill_(1.0)
    stream_GBps = sv.ss_probe_read_bandwidth(probe_buf, iters=20)
    del probe_buf
    roofline["read_stream_GBps"] = stream_GBps
    roofline["frac_of_read_stream"] = achieved / stream_GBps

    # The paper's premise (Section 2): the pass is memory-bound, so K + 1 rows cost about what one row costs.  The
    # forward alone, same cache length, M rows against one row.
    def forward_ms(rows, iters=20):
        Lp = int(sv.ss_kv_cache_get_len(tkv)[0])
        t_in = vt[:, :rows].contiguous()
        lg = logits[:, :rows]
        ts = []
        for it in range(iters + 2):
            sv.ss_kv_cache_set_len(tkv, [Lp])
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            sv.ss_verify_forward(target, tkv, t_in, rows, lg.contiguous() if rows != M else logits)
            torch.cuda.synchronize()
            if it >= 2:
                ts.append(time.perf_counter() - t1)
        sv.ss_kv_cache_set_len(tkv, [Lp])
        ts.sort()
        return 1e3 * ts[len(ts) // 2]
    t_m, t_1 = forward_ms(M), forward_ms(1)
    check_status(sv, target)
    # the other forward path on the same model and cache, for comparison (ss_model_set_persistent)
    other = None
    try:
        sv.ss_model_set_persistent(target, not bool(args.persistent))
        o_m, o_1 = forward_ms(M), forward_ms(1)
        other = {"forward_path": "one launch per phase" if args.persistent else "persistent kernel",
                 "t_verify_ms_rows_K_plus_1": o_m, "t_verify_ms_rows_1": o_1,
                 "hbm_frac_of_peak_rows_K_plus_1": pass_bytes / (o_m * 1e-3) / HBM_PEAK,
                 "note": "host-timed ss_verify_forward alone, as in `premise`"}
    except sv.SpecVerifyError as e:            # the persistent kernel is not available on every device
        other = {"forward_path": "persistent kernel", "unavailable": str(e)}
    finally:
        sv.ss_model_set_persistent(target, bool(args.persistent))
    check_status(sv, target)
    premise = {"t_verify_ms_rows_K_plus_1": t_m, "t_verify_ms_rows_1": t_1, "premise_ratio": t_m / t_1,
               "note": f"host-timed ss_verify_forward alone, {M} rows against 1 row, same cache length; 1.0 = K draft tokens verified for the price of one"}

    out = {
        "metric": "verify-pass tokens/s", "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"full 7B-shaped target ({shape.n_layers} layers, d 4096, 32x128 heads, FFN 11008, vocab 32000), "
                               f"bf16, batch 1, K={K} ({M} query rows), KV context {L_start}..{L_end}, random init",
                   "step": "ss_verify_forward + ss_softmax + ss_speculative_accept + ss_kv_cache_rollback",
                   "forward_path": "persistent kernel" if args.persistent else "one launch per phase"},
        "verify_pass": {"algorithmic_bytes": pass_bytes, "hbm_frac_of_peak": pass_bytes / (dt / args.steps) / HBM_PEAK,
                        "hbm_GBps": pass_bytes / (dt / args.steps) / 1e9, "kernel_classes": classes},
        "roofline": roofline,
        "premise": premise,
        "other_forward_path": other,
        "end_to_end": e2e,
    }
    if not args.no_layer_pass:
        out["layer_pass"] = layer_pass(si, sv, torch, dev, target, shape)
    if not args.no_accept_workload:
        out["standalone_accept"] = standalone_accept(si, sv, torch, dev)
    if not args.no_int8_leg:
        out["int8_weights"] = int8_weights_leg(si, sv, torch, gen, dev, target, bool(args.persistent), shape, packed, io, prompt, K, args.steps)
        out["int4_weights"] = int8_weights_leg(si, sv, torch, gen, dev, target, bool(args.persistent), shape, packed, io, prompt, K, args.steps, bits=4)
    if not args.no_paper_pair:
        out["paper_size_pair"] = paper_pair_leg(si, sv, torch, gen, dev)
    if not args.no_batched_workload and args.layers == 32:
        out["batched_workload"] = batched_workload(si, sv, torch, dev, shape, packed, io, int8=not args.no_int8_leg)
    for leg in ("layer_pass", "standalone_accept", "batched_workload", "int8_weights", "int4_weights"):
        if leg in out and "GBps" in out[leg]:
            out[leg]["frac_of_read_stream"] = out[leg]["GBps"] / stream_GBps
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(si, torch, shape, packed, io, prompt_len, M)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    check_status(sv, target, draft)
    print(json.dumps(out), flush=True)
    # release every device object and the library's own state while the HIP runtime is still up (not at interpreter teardown)
    torch.cuda.synchronize()
    for obj in (tkv, dkv, target, draft):
        obj.close()
    sv.ss_shutdown()


if __name__ == "__main__":
    main()
