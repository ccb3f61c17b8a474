"""The built C-ABI library loads and exports every entry point that include/k3.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    import torch  # noqa: F401  (brings in the HIP runtime the library links against)
    from paper_1811_12174_amd import k3
    header = open(os.path.join(ROOT, "include", "k3.h")).read()
    names = sorted(set(re.findall(r"\b(k3_[a-z0-9_]+)\s*\(", header)))
    assert len(names) >= 30
    lib = k3.lib()
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, missing
    assert k3.version() == 104
    assert k3.status_string(k3.E_STATE) == "illegal swap-state transition"


def test_binding_covers_every_entry_point():
    from paper_1811_12174_amd import k3
    header = open(os.path.join(ROOT, "include", "k3.h")).read()
    names = sorted(set(re.findall(r"\bk3_([a-z0-9_]+)\s*\(", header)))
    missing = [n for n in names if not hasattr(k3, n)]
    assert not missing, missing


def test_argument_errors_need_no_gpu():
    from paper_1811_12174_amd import k3
    out = ctypes.c_size_t(7)
    assert k3.lib().k3_conv3d_packed_bytes(ctypes.c_int64(32), ctypes.c_int64(64), 1, ctypes.byref(out)) == 0
    assert out.value == 2 * 27 * 32 * 64 * 2
    assert k3.lib().k3_conv3d_packed_bytes(ctypes.c_int64(4), ctypes.c_int64(8), 2, ctypes.byref(out)) == 0 and out.value == 0
    assert k3.lib().k3_conv3d_packed_bytes(ctypes.c_int64(0), ctypes.c_int64(8), 2, ctypes.byref(out)) == k3.E_BADARG
    bad = k3.TensorDesc(1, 3, 4, 4, 8, k3.BF16, 0)
    y = k3.TensorDesc(1, 1, 2, 2, 8, k3.BF16, 0)
    assert k3.lib().k3_pool3d_fwd(ctypes.byref(bad), ctypes.c_void_p(16), ctypes.byref(y), ctypes.c_void_p(16), None) == k3.E_SHAPE


def test_argument_errors_of_the_later_entry_points_need_no_gpu():
    """Shape and argument checks happen before anything is launched."""
    from paper_1811_12174_amd import k3
    L = k3.lib()
    out = ctypes.c_size_t(7)
    y = k3.TensorDesc(1, 4, 4, 4, 32, k3.BF16, 0)
    assert L.k3_relu_bits_bytes(ctypes.byref(y), ctypes.byref(out)) == 0 and out.value == 64 * 2 * 2
    odd = k3.TensorDesc(1, 4, 4, 4, 24, k3.BF16, 0)
    assert L.k3_relu_bits_bytes(ctypes.byref(odd), ctypes.byref(out)) == k3.E_UNSUPPORTED
    assert L.k3_relu_bits_bytes(None, ctypes.byref(out)) == k3.E_BADARG
    small = k3.TensorDesc(1, 2, 2, 2, 8, k3.BF16, 0)
    big = k3.TensorDesc(1, 4, 4, 4, 8, k3.BF16, 0)
    wrong = k3.TensorDesc(1, 4, 4, 5, 8, k3.BF16, 0)
    p = ctypes.c_void_p(16)
    assert L.k3_upsample3d_fwd(ctypes.byref(small), p, ctypes.byref(wrong), p, None) == k3.E_SHAPE
    assert L.k3_upsample3d_fwd(ctypes.byref(small), None, ctypes.byref(big), p, None) == k3.E_BADARG
    assert L.k3_upsample3d_bwd(ctypes.byref(wrong), p, None, ctypes.byref(small), p, None) == k3.E_SHAPE
    assert L.k3_head_classify(ctypes.byref(big), None, p, None, p, None, None) == k3.E_BADARG
    assert L.k3_dice_coefficients(p, p, ctypes.c_int64(-1), p, None, None) == k3.E_BADARG
    assert L.k3_dice_coefficients(None, None, ctypes.c_int64(5), p, None, None) == k3.E_BADARG
    assert L.k3_sgd_momentum_step(ctypes.c_int64(-1), p, p, p, ctypes.c_float(0.1), ctypes.c_float(0), ctypes.c_float(0), None, None) == k3.E_BADARG
    assert L.k3_sgd_momentum_step(ctypes.c_int64(0), None, None, None, ctypes.c_float(0.1), ctypes.c_float(0), ctypes.c_float(0), None, None) == 0
    assert L.k3_sgd_momentum_step(ctypes.c_int64(4), p, p, p, ctypes.c_float(float("nan")), ctypes.c_float(0), ctypes.c_float(0), None, None) == k3.E_BADARG


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr
