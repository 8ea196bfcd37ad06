"""No-GPU checks of the boundary: the built library loads and exports every symbol the header
declares, and the binding names match."""
import ctypes
import os
import re

import paper_2311_04951_amd as sv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "specverify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ss_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert "ss_verify_forward" in names and "ss_speculative_accept" in names and len(names) >= 18
    assert os.path.exists(sv.LIB_PATH), "build the library first (__graft_entry__.build())"
    L = ctypes.CDLL(sv.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert sorted(sv.EXPORTS) == names


def test_binding_has_one_function_per_compute_entry_point():
    for n in _declared():
        if n in ("ss_last_error", "ss_model_create", "ss_model_destroy", "ss_kv_cache_free"):
            continue          # wrapped by the Model / KVCache handle classes
        assert callable(getattr(sv, n)), n


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2311_04951_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("oracle-free", ""), f


def test_bench_refuses_more_than_one_gpu_before_touching_a_device():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode != 0 and r.stdout.strip() == ""
    assert "one GPU" in r.stderr


def test_bench_algorithmic_bytes_are_the_documented_sums():
    """The roofline figure divides these bytes by a measured time: every weight once (bf16), the KV context
    once, the new K/V rows, the logits."""
    import bench
    import seeded_inputs as si
    s = si.FULL_7B
    layer = 2 * (4 * 4096 * 4096 + 3 * 4096 * 11008)                 # q, k, v, o + gate, up, down in bf16
    assert bench.layer_bytes(s) == layer == 404_750_336
    L, M = 145, 5
    want = 32 * layer + 32000 * 4096 * 2 + 32 * 2 * (L + M) * 4096 * 2 + 32 * 2 * M * 4096 * 2 + M * 32000 * 4
    assert bench.verify_pass_bytes(s, L, M) == want
    assert abs(want - 13.296e9) < 0.01e9                              # the figure the committed profile summaries quote
    assert bench.HBM_PEAK == 8e12


def test_calls_without_a_handle_refuse_a_workspace_that_is_too_small_on_the_host():
    """Argument validation happens before anything is launched, so it can be exercised without a GPU: made-up
    (aligned, never dereferenced) device addresses, a workspace one byte short of what the call needs."""
    L = sv.lib()
    vp = ctypes.c_void_p
    fake = [vp(0x10000 * (i + 1)) for i in range(8)]
    rows, V, B, K = 9, 32000, 1, 4
    assert sv.ss_workspace_bytes(rows, V) > 0 and sv.ss_workspace_bytes(0, V) > 0 and sv.ss_workspace_bytes(4, 0) == 0
    assert sv.ss_workspace_bytes(64 * 17, 128256) >= sv.ss_workspace_bytes(17, 128256)
    small = 1024
    assert L.ss_softmax(fake[0], rows, V, 1.0, fake[1], fake[2], small, None) == sv.SS_ECAPACITY
    assert b"workspace" in L.ss_last_error()
    assert L.ss_speculative_accept(fake[0], fake[1], fake[2], fake[3], B, K, V, fake[4], fake[5], fake[6], small, None) == sv.SS_ECAPACITY
    assert L.ss_speculative_accept_logits(fake[0], fake[1], 0.8, fake[2], fake[3], B, K, V, fake[4], fake[5], None, None,
                                          fake[6], small, None) == sv.SS_ECAPACITY
    assert L.ss_greedy_accept(fake[0], fake[1], B, K, V, fake[2], fake[3], fake[4], small, None) == sv.SS_ECAPACITY
    assert L.ss_workspace_init(fake[0], small, None) == sv.SS_ECAPACITY
    # a NULL or misaligned workspace is a bad argument, not a capacity problem
    big = sv.ss_workspace_bytes(rows, V)
    assert L.ss_softmax(fake[0], rows, V, 1.0, fake[1], None, big, None) == sv.SS_EINVAL
    assert L.ss_softmax(fake[0], rows, V, 1.0, fake[1], vp(0x10004), big, None) == sv.SS_EINVAL
    # the device-array truncation and the cache creation validate on the host as well
    assert L.ss_kv_cache_truncate(None, fake[0], None, None, None) == sv.SS_EINVAL
    out = vp()
    assert L.ss_kv_cache_create(None, 1, 64, fake[0], 1 << 20, None, ctypes.byref(out)) == sv.SS_EINVAL
    assert L.ss_shutdown() == 0 and L.ss_shutdown() == 0      # nothing alive: a no-op, twice
