"""Helpers shared by the GPU parity tests: the same seeded inputs for the oracle and the library."""
import numpy as np
import torch

import oracle
import paper_2311_04951_amd as sv
import seeded_inputs as si


def dev():
    return torch.device("cuda:0")


def weights_to_device(w):
    d = dev()
    out = {k: (v.to(d) if v is not None and hasattr(v, "to") else v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: v.to(d) for k, v in lw.items()} for lw in w["layers"]]
    return out


def model_pair(shape, seed, max_rows=16, max_pos=256, persistent=False):
    """(oracle model, GPU model, host weights) over identical seeded weights."""
    w = si.decoder_weights(shape, seed)
    gm = sv.Model(shape, weights_to_device(w), max_rows=max_rows, max_pos=max_pos)
    set_path(gm, persistent)
    return oracle.Model(shape, w), gm, w


# Forward paths under test: per-phase launches (the default); the persistent kernel on its default grid (on these
# small shapes a grid of one workgroup per compute unit leaves workgroups without a share of some
# phase, so every phase boundary is a barrier); the persistent kernel on a grid of 8 workgroups, where
# every workgroup owns part of every GEMM phase and the activations synchronise themselves.
PATHS = [False, True, "grid8"]


def set_path(gm, path):
    sv.ss_model_set_persistent(gm, bool(path))
    if isinstance(path, str):
        sv.ss_model_set_persistent_options(gm, int(path[4:]), True)


def tol(shape):
    """logits tolerance: max-abs 2e-2 with bf16 storage, 1e-4 with fp32 storage."""
    return 2e-2 if shape.dtype == "bf16" else 1e-4


def maxabs(a, b):
    if hasattr(a, "detach"):
        a = a.detach().float().cpu().numpy()
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64))))
