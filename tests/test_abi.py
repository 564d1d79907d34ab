"""The C-ABI library loads and exports every symbol include/ckpt.h declares;
host-only calls and host-side argument checks (nothing here launches a kernel)."""
import ctypes
import os
import re

import pytest

from paper_2502_12499_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    """Every function that a header under include/ declares."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(ckpt_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_three_calls():
    names = declared_functions()
    for want in ("ckpt_eval_peak", "ckpt_solve_cubic", "ckpt_solve_linear", "ckpt_workspace_bytes",
                 "ckpt_eval_timeline", "ckpt_select_baseline"):
        assert want in names


def test_library_exports_every_declared_symbol():
    lib = B.load()
    for name in declared_functions():
        assert getattr(lib, name) is not None, name
    assert set(B.EXPORTS) == set(declared_functions())


def test_host_only_helpers():
    assert B.cubic_cells(12) == (12 * 11 // 2 + 1) * 12 == 804
    assert B.cubic_cells(1001) == 500501 * 1001
    assert B.cubic_cells(4096) == 8386561 * 4096
    assert B.status_string(0) == "ok"
    assert "size" in B.status_string(3)


def test_workspace_bytes_and_layout_checks():
    good = B.Layout(1024, 64, 1, 1024)
    for which in (B.CALL_EVAL_PEAK, B.CALL_SOLVE_CUBIC, B.CALL_SOLVE_LINEAR):
        assert B.workspace_bytes(which, good) > 0
    assert B.workspace_bytes(7, good) == 0
    for bad in (B.Layout(-1, 64, 1, 1024), B.Layout(8, 0, 1, 8), B.Layout(8, 64, 0, 8),
                B.Layout(8, 64, 1, 0), B.Layout(8, 70000, 1, 8)):
        assert B.workspace_bytes(B.CALL_SOLVE_LINEAR, bad) == 0
    # the cubic solver has its own, smaller limit on n
    assert B.workspace_bytes(B.CALL_SOLVE_CUBIC, B.Layout(1, 8192, 1, 1)) == 0
    assert B.workspace_bytes(B.CALL_SOLVE_CUBIC, B.Layout(1, 8191, 1, 1)) > 0
    # grows with the problem
    assert B.workspace_bytes(B.CALL_SOLVE_LINEAR, B.Layout(2048, 64, 1, 2048)) > \
        B.workspace_bytes(B.CALL_SOLVE_LINEAR, good)


def test_host_detectable_errors_return_without_launching():
    lib = B.load()
    L = B.Layout(4, 8, 1, 4)
    fake = ctypes.c_void_p(4096)  # never dereferenced: every call below fails validation first
    assert lib.ckpt_eval_peak(fake, fake, None, 0, fake, None, None, 0, None) == 1
    assert lib.ckpt_eval_peak(None, fake, ctypes.byref(L), 0, fake, None, None, 0, None) == 1
    assert lib.ckpt_eval_peak(fake, fake, ctypes.byref(L), 3, fake, None, None, 0, None) == 2
    assert lib.ckpt_solve_linear(fake, ctypes.byref(B.Layout(4, 0, 1, 4)), fake, fake, None, fake, 1 << 20, None) == 2
    assert lib.ckpt_solve_linear(fake, ctypes.byref(L), fake, fake, None, None, 0, None) == 1
    assert lib.ckpt_solve_linear(fake, ctypes.byref(L), fake, fake, None, fake, 16, None) == 6      # too small
    assert lib.ckpt_solve_cubic(fake, ctypes.byref(L), fake, fake, None, None, ctypes.c_void_p(4100), 1 << 30, None) == 6  # misaligned
    assert lib.ckpt_solve_cubic(fake, ctypes.byref(L), None, fake, None, None, fake, 1 << 30, None) == 1
    # an empty batch is a successful no-op
    E = B.Layout(0, 8, 1, 1)
    assert lib.ckpt_solve_cubic(None, ctypes.byref(E), None, None, None, None, None, 0, None) == 0
    assert lib.ckpt_eval_peak(None, None, ctypes.byref(E), 1, None, None, None, 0, None) == 0


def test_timeline_and_baseline_host_checks():
    lib = B.load()
    L = B.Layout(4, 8, 1, 4)
    fake = ctypes.c_void_p(4096)        # never dereferenced: validation fails first
    assert lib.ckpt_eval_timeline(fake, fake, ctypes.byref(L), 1, fake, 0, 4, None, None) == 2
    assert lib.ckpt_eval_timeline(fake, fake, ctypes.byref(L), 3, fake, 1, 4, None, None) == 2
    assert lib.ckpt_eval_timeline(fake, fake, ctypes.byref(L), 1, None, 1, 4, None, None) == 1
    assert lib.ckpt_select_baseline(ctypes.byref(L), 3, fake, None) == 2
    assert lib.ckpt_select_baseline(ctypes.byref(L), 0, None, None) == 1


def test_binding_refuses_cpu_tensors():
    import torch
    d = torch.ones(5, 3, dtype=torch.int64)
    with pytest.raises(TypeError):
        B.ckpt_solve_linear(d)


def test_ragged_host_checks():
    import numpy as np
    lib = B.load()
    off = np.array([0, 16, 41, 43], dtype=np.int64)       # n = 15, 24, 1
    ptr = ctypes.c_void_p(off.ctypes.data)
    sizes = [lib.ckpt_ragged_workspace_bytes(w, ptr, 3) for w in
             (B.CALL_EVAL_PEAK, B.CALL_SOLVE_CUBIC, B.CALL_SOLVE_LINEAR, B.CALL_EVAL_TIMELINE)]
    assert all(s > 0 and s % 256 == 0 for s in sizes)
    assert sizes[3] > sizes[0]                              # the timeline stages 2n+2 phases per chain
    assert lib.ckpt_ragged_workspace_bytes(B.CALL_SOLVE_LINEAR, ptr, 0) == 0
    assert lib.ckpt_ragged_workspace_bytes(4, ptr, 3) == 0
    for bad in ([0, 16, 15, 43], [0, 1, 41, 43], [-2, 16, 41, 43]):
        b = np.array(bad, dtype=np.int64)
        assert lib.ckpt_ragged_workspace_bytes(B.CALL_SOLVE_LINEAR, ctypes.c_void_p(b.ctypes.data), 3) == 0
    # the cubic solver's limit on n applies per chain
    long = np.array([0, 8193], dtype=np.int64)
    assert lib.ckpt_ragged_workspace_bytes(B.CALL_SOLVE_CUBIC, ctypes.c_void_p(long.ctypes.data), 1) == 0
    assert lib.ckpt_ragged_workspace_bytes(B.CALL_SOLVE_LINEAR, ctypes.c_void_p(long.ctypes.data), 1) > 0
    fake = ctypes.c_void_p(4096)        # never dereferenced: validation fails first
    assert lib.ckpt_ragged_solve_linear(fake, ptr, None, 3, fake, fake, None, fake, 16, None) == 6
    assert lib.ckpt_ragged_solve_linear(fake, ptr, fake, 3, None, fake, None, fake, 1 << 30, None) == 1
    # offsets in neither place; the cubic solver plans on the host and needs them there
    assert lib.ckpt_ragged_solve_linear(fake, None, None, 3, fake, fake, None, fake, 1 << 30, None) == 1
    assert lib.ckpt_ragged_solve_cubic(fake, None, fake, 3, fake, fake, fake, None, fake, 1 << 30, None) == 1
    assert lib.ckpt_ragged_eval_peak(fake, fake, ptr, None, 3, 3, fake, None, fake, 1 << 30, None) == 2
    assert lib.ckpt_ragged_solve_cubic(None, ptr, None, 0, None, None, None, None, None, 0, None) == 0
