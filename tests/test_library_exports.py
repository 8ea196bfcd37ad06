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
