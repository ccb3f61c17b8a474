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
    assert k3.version() == 101
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
