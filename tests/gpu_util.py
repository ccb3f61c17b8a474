"""Helpers for the GPU parity tests: host <-> device conversion and error norms."""
import os
import sys

import numpy as np
import torch

TOL = {"bf16": 2e-2, "f32": 1e-5}   # relative L2 bound per output tensor (workload statement)


def to_dev(a, dtype):
    """float32 numpy array (already representable in dtype) -> device tensor."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t.contiguous()


def to_f64(t):
    """device tensor -> float64 numpy (exact)."""
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def empty(shape, dtype):
    return torch.empty(shape, device="cuda", dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)


MEASURED = {}   # (test function, line) -> largest relative L2 error seen there in this session


def rel_l2(got, ref, depth=1, tag=""):
    """Relative L2 distance; every value is also noted under the calling test and line (the
    session's worst cases are written to measured_errors.json in the run's output folder by conftest.py)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    den = np.linalg.norm(ref.reshape(-1))
    num = np.linalg.norm((got - ref).reshape(-1))
    e = num / den if den > 0 else num
    f = sys._getframe(depth)
    key = (os.path.basename(f.f_code.co_filename), f.f_code.co_name + ("[" + tag + "]" if tag else ""), f.f_lineno)
    MEASURED[key] = max(MEASURED.get(key, 0.0), float(e))
    return e


def packed_for(w):
    from paper_1811_12174_amd import k3
    nb = k3.conv3d_packed_bytes(w.shape[3], w.shape[4], k3.BF16 if w.dtype == torch.bfloat16 else k3.F32)
    if nb == 0:
        return None
    p = torch.empty(nb, device="cuda", dtype=torch.uint8)
    k3.conv3d_pack_weights(w, p)
    return p
