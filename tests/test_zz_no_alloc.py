"""The rejection step through the entry point that allocates nothing (its scratch is a device array built into the
library) against the entry point that takes a workspace: same bits, call after call, the second call smaller
than the first."""
import ctypes as C

import pytest
import torch

import paper_2311_04951_amd as sv
import seeded_inputs as si

pytestmark = pytest.mark.gpu


def _case(seed, B, K, V, dev):
    pl, ql, u, ud = si.accept_workload(seed, B, K, V, device=dev)
    p, q = sv.ss_softmax(pl, 0.8), sv.ss_softmax(ql, 0.8)
    d = torch.empty((B, K), dtype=torch.int32, device=dev)
    zf, zi = torch.zeros(1, device=dev), torch.zeros(1, dtype=torch.int32, device=dev)
    for i in range(K):   # draft tokens ~ q (the K = 0 case of the rejection step is a plain sample)
        d[:, i] = sv.ss_speculative_accept(q[:, i].contiguous()[:, None], zf, zi, ud[:, i:i + 1].contiguous())[1]
    return p, q, d, u


def test_no_alloc_entry_point_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    i32 = dict(dtype=torch.int32, device=dev)
    cases = [_case(51, 64, 8, 128256, dev), _case(52, 3, 4, 1000, dev)]    # 64 x 16 segments of scratch, then 3 x 1
    p1, q1, d1, u1 = cases[1]
    cases.append((p1[:, :1].contiguous(), q1, d1, u1[:, :1].contiguous()))   # K = 0: a plain sample from p
    bad = d1.clone()
    bad[1, 0] = 1000 + 7
    cases.append((p1, q1, bad, u1))                                         # a token id out of range
    order = [0, 1, 0, 1, 2, 3]                                              # large, small, large, small, ...
    got = [(torch.full((64,), -1, **i32), torch.full((64,), -1, **i32)) for _ in order]
    want = [(torch.full((64,), -1, **i32), torch.full((64,), -1, **i32)) for _ in order]
    status = torch.zeros(len(order), **i32)
    ws = sv.ss_workspace_init(torch.empty(sv.ss_workspace_bytes(64 * 17, 128256), dtype=torch.uint8, device=dev))
    sv.ss_freeze_allocations(True)          # also the one-off set-up of the built-in scratch array on this device
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    try:
        # nothing but library calls between the two readings of free device memory: every tensor exists already
        for i, c in enumerate(order):
            p, q, d, u = cases[c]
            B = p.shape[0]
            sv.ss_speculative_accept_noalloc(p, q, d, u, got[i][0][:B], got[i][1][:B], status=status[i:i + 1])
            sv.ss_speculative_accept(p, q, d, u, want[i][0][:B], want[i][1][:B], ws=ws)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free0
    finally:
        sv.ss_freeze_allocations(False)
    for i, c in enumerate(order):
        B, K = cases[c][0].shape[0], cases[c][2].shape[1] if cases[c][0].shape[1] > 1 else 0
        assert torch.equal(got[i][0], want[i][0]) and torch.equal(got[i][1], want[i][1]), i
        assert int(got[i][0][:B].min()) >= 0 and int(got[i][0][:B].max()) <= K
        assert int(got[i][1][:B].min()) >= 0 and bool((got[i][0][B:] == -1).all())          # nothing written past the batch
    assert status.tolist() == [0, 0, 0, 0, 0, 1]
    assert int(got[5][0][1]) == 0                                           # the bad token counts as rejected
    assert sv.ss_workspace_status(ws) == 1


def test_no_alloc_entry_point_refuses_what_does_not_fit_its_scratch():
    dev = torch.device("cuda:0")
    z = torch.zeros(16, device=dev)
    zi = torch.zeros(16, dtype=torch.int32, device=dev)
    rc = sv.lib().ss_speculative_accept_noalloc(C.c_void_p(z.data_ptr()), C.c_void_p(z.data_ptr()), C.c_void_p(zi.data_ptr()),
                                               C.c_void_p(z.data_ptr()), 8161, 4, 128256, C.c_void_p(zi.data_ptr()),
                                               C.c_void_p(zi.data_ptr()), None, None)
    assert rc == sv.SS_ECAPACITY and b"scratch" in sv.lib().ss_last_error()
