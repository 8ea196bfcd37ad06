"""The speculative step for a batch of sequences that accept different numbers of tokens (ragged cache lengths;
Sections 3, 4.3, 4.4): every sequence of the batched loop is followed on the oracle in lock step (its q rows and
logits by tolerance, draft sampling and accept / resample decisions bit for bit on the GPU's own rows), greedy
streams equal the autoregressive ones, and bad requests are refused before a cache changes."""
import numpy as np
import pytest
import torch

import oracle
import paper_2311_04951_amd as sv
import seeded_inputs as si
from paper_2311_04951_amd import generate as gen
from gpu_util import dev, maxabs, weights_to_device

pytestmark = pytest.mark.gpu


def _pair(seed, B, K, early=True):
    tw = si.decoder_weights(si.TINY_TARGET, seed)
    if early:
        dshape, dw = si.early_exit_draft(si.TINY_TARGET, tw, 1)
    else:
        dshape, dw = si.TINY_DRAFT, si.decoder_weights(si.TINY_DRAFT, seed + 100)
    gt = sv.Model(si.TINY_TARGET, weights_to_device(tw), max_rows=max(16, B * (K + 1)), max_pos=256)
    gd = sv.Model(dshape, weights_to_device(dw), max_rows=max(16, 2 * B), max_pos=256)
    return (oracle.Model(si.TINY_TARGET, tw), oracle.Model(dshape, dw)), (gt, gd)


def _prompts(seed, B):
    lens = [7, 32, 2, 19, 11, 3, 26, 14][:B]                       # ragged from the start; one prompt of the minimum length
    return [si.token_ids(seed, f"prompt{b}", (n,), 1024).numpy().tolist() for b, n in enumerate(lens)]


@pytest.mark.parametrize("B,K,top_k", [(3, 4, 0), (8, 3, 0), (4, 8, 12)])
def test_sampled_batched_run_in_lock_step_with_the_oracle(B, K, top_k):
    n_new, T = 40, 1.0
    (ot, od), (gt, gd) = _pair(5, B, K)
    prompts = _prompts(5, B)
    ud = si.uniforms(5, "ud", (B, n_new, K)).numpy()
    ua = si.uniforms(5, "ua", (B, n_new, K + 1)).numpy()
    seen = []

    def obs(step, buf, res):
        seen.append({"q": buf.q.cpu().numpy().copy(), "p": buf.p.cpu().numpy().copy(), "logits": buf.logits.cpu().numpy().copy(), "res": res})

    out, stats = gen.speculative_generate_batched(gt, gd, prompts, n_new, K, T, ud, ua, observer=obs, top_k=top_k)
    assert all(len(o) == n_new for o in out) and stats["steps"] == len(seen)
    ragged = False
    for b in range(B):
        # replay sequence b on the oracle, following the GPU's committed history; the oracle keeps the usual
        # bookkeeping (draft cache n - 1 positions), which must give the same rows as the batched one (n - 2, two-token feed)
        x = list(prompts[b])
        otkv, odkv = ot.new_kv(256), od.new_kv(256)
        ot.forward(otkv, x[:-1], want_logits=False)
        if len(x) > 2:
            od.forward(odkv, x[:-2], want_logits=False)
        for st, s in enumerate(seen):
            n = len(x)
            a, y, d = s["res"][b]
            feed = x[-2:]
            for i in range(K):
                ql = od.forward(odkv, feed)[-1]
                want_q = oracle.select(oracle.softmax(ql, T), top_k=top_k)
                assert maxabs(s["q"][b, i], want_q) < 1e-5, (b, st, i)
                assert d[i] == oracle.sample(s["q"][b, i], ud[b][st][i])          # draft sampling: bit-exact on the GPU's q
                feed = [d[i]]
            pl = ot.forward(otkv, [x[-1]] + d)
            assert maxabs(s["logits"][b], pl) < 1e-4, (b, st)
            ona, onx = oracle.speculative_accept(s["p"][b][None], s["q"][b][None], np.asarray([d], dtype=np.int32), ua[b][st][None])
            assert (int(ona[0]), int(onx[0])) == (a, y), (b, st)
            x += d[:a] + [y]
            otkv.set_len(n + a)
            odkv.set_len(n + a - 1)
        assert x[len(prompts[b]):len(prompts[b]) + n_new] == out[b]
        ragged = ragged or stats["accepted"][b] != stats["accepted"][0]
    assert ragged                                                    # the sequences did accept different numbers of tokens
    flat = [a for acc in stats["accepted"] for a in acc]
    assert 0 < sum(flat) < K * len(flat)                             # both accepts and rejections occurred


@pytest.mark.parametrize("early", [True, False])
def test_greedy_batched_streams_equal_autoregressive_and_the_oracle(early):
    B, K, n_new = 5, 4, 32
    (ot, od), (gt, gd) = _pair(6, B, K, early)
    prompts = _prompts(6, B)
    out, stats = gen.speculative_generate_batched(gt, gd, prompts, n_new, K, 0.0)
    for b in range(B):
        assert out[b] == gen.autoregressive_generate(gt, prompts[b], n_new, 0.0)
        assert out[b] == oracle.autoregressive_generate(ot, prompts[b], n_new, 0.0)
    # draft = target: everything is accepted in every sequence, the streams stay the autoregressive ones
    same, st = gen.speculative_generate_batched(gt, gt, prompts, n_new, K, 0.0)
    assert same == out and all(a == K for acc in st["accepted"] for a in acc)


def test_batched_step_refuses_bad_requests_before_touching_a_cache():
    B, K = 2, 3
    _, (gt, gd) = _pair(7, B, K)
    V = si.TINY_TARGET.vocab
    tkv, dkv = sv.KVCache(gt, B, 64), sv.KVCache(gd, B, 64)
    one = sv.KVCache(gd, 1, 64)
    buf = sv.BatchedStepBuffers(B, K, V, [[1, 2], [3, 4]], dev())
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_speculative_step_batched(gt, tkv, gd, one, buf, 0.0)                    # caches of different batch
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_speculative_step_batched(gt, tkv, gt, tkv, buf, 0.0)                    # one shared cache
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_speculative_step_batched(gt, tkv, gd, dkv, buf, 1.0)                    # sampling without uniforms
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_speculative_step_batched(gt, tkv, gd, dkv, buf, 0.0, top_k=-1)
    small = sv.KVCache(gd, B, 3)                                                      # no room for K + 1 draft rows
    with pytest.raises(sv.SpecVerifyError):
        sv.ss_speculative_step_batched(gt, tkv, gd, small, buf, 0.0)
    assert sv.ss_kv_cache_get_len(tkv).tolist() == [0, 0] and sv.ss_kv_cache_get_len(dkv).tolist() == [0, 0]
    assert sv.ss_kv_cache_get_len(small).tolist() == [0, 0]
    # and a good request on the same buffers goes through
    res = sv.ss_speculative_step_batched(gt, tkv, gd, dkv, buf, 0.0)
    lt, ld = sv.ss_kv_cache_get_len(tkv).tolist(), sv.ss_kv_cache_get_len(dkv).tolist()
    assert lt == [r[0] + 1 for r in res] and ld == lt
