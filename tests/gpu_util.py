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
    sv.ss_model_set_persistent(gm, persistent)
    return oracle.Model(shape, w), gm, w


PATHS = [False, True]   # per-phase launches, persistent kernel


def tol(shape):
    """logits tolerance: max-abs 2e-2 with bf16 storage, 1e-4 with fp32 storage."""
    return 2e-2 if shape.dtype == "bf16" else 1e-4


def maxabs(a, b):
    if hasattr(a, "detach"):
        a = a.detach().float().cpu().numpy()
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64))))
