"""Python binding of the C ABI in include/ckpt.h: argument marshalling only.

Each function takes torch tensors that already live on the GPU, passes their
device pointers, the layout and the current HIP stream to the library call of
the same name, and returns the output tensors.  No step of the computation runs
here, and there is no fallback: if libckpt_hip.so has not been built the import
of the library fails loudly.

Tensor convention: ``d`` is int64 of shape (n+1, batch) ("position-major",
contiguous: the fast layout) or (batch, n+1) with ``chain_major=True``; masks
have the same shape, uint8.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libckpt_hip.so")

CKPT_OK = 0
OBJ_STATIC, OBJ_DYNAMIC, OBJ_BOTH = 0, 1, 2
CALL_EVAL_PEAK, CALL_SOLVE_CUBIC, CALL_SOLVE_LINEAR, CALL_EVAL_TIMELINE = 0, 1, 2, 3

SELECT_ENDS, SELECT_ALL, SELECT_SQRT = 0, 1, 2

EXPORTS = ("ckpt_workspace_bytes", "ckpt_eval_peak", "ckpt_eval_timeline", "ckpt_select_baseline",
           "ckpt_solve_cubic", "ckpt_solve_cubic_pruned", "ckpt_solve_cubic_costs", "ckpt_cubic_costs_len", "ckpt_solve_linear", "ckpt_solve_linear_noalloc",
           "ckpt_solve_quadratic", "ckpt_cubic_cells",
           "ckpt_status_string",
           "ckpt_ragged_workspace_bytes", "ckpt_ragged_eval_peak", "ckpt_ragged_eval_timeline",
           "ckpt_ragged_solve_linear", "ckpt_ragged_solve_cubic",
           # include/ckpt_probe.h
           "ckpt_probe_hbm_read", "ckpt_probe_hbm_copy", "ckpt_probe_valu", "ckpt_probe_lds")


class Layout(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int64), ("n_layers", ctypes.c_int32),
                ("chain_stride", ctypes.c_int64), ("pos_stride", ctypes.c_int64)]


_lib = None


def load():
    """dlopen the in-tree library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2502_12499_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, LP = ctypes.c_void_p, ctypes.POINTER(Layout)
        lib.ckpt_workspace_bytes.restype = ctypes.c_size_t
        lib.ckpt_workspace_bytes.argtypes = [ctypes.c_int, LP]
        lib.ckpt_eval_peak.restype = ctypes.c_int
        lib.ckpt_eval_peak.argtypes = [vp, vp, LP, ctypes.c_int, vp, vp, vp, ctypes.c_size_t, vp]
        lib.ckpt_eval_timeline.restype = ctypes.c_int
        lib.ckpt_eval_timeline.argtypes = [vp, vp, LP, ctypes.c_int, vp, ctypes.c_int64, ctypes.c_int64, vp, vp]
        lib.ckpt_select_baseline.restype = ctypes.c_int
        lib.ckpt_select_baseline.argtypes = [LP, ctypes.c_int, vp, vp]
        lib.ckpt_solve_cubic.restype = ctypes.c_int
        lib.ckpt_solve_cubic.argtypes = [vp, LP, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.ckpt_solve_cubic_pruned.restype = ctypes.c_int
        lib.ckpt_solve_cubic_pruned.argtypes = [vp, LP, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.ckpt_solve_cubic_costs.restype = ctypes.c_int
        lib.ckpt_solve_cubic_costs.argtypes = [vp, LP, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.ckpt_cubic_costs_len.restype = ctypes.c_int64
        lib.ckpt_cubic_costs_len.argtypes = [ctypes.c_int32]
        lib.ckpt_solve_linear.restype = ctypes.c_int
        lib.ckpt_solve_linear.argtypes = [vp, LP, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.ckpt_solve_linear_noalloc.restype = ctypes.c_int
        lib.ckpt_solve_linear_noalloc.argtypes = [vp, LP, vp, vp, vp, vp]
        lib.ckpt_solve_quadratic.restype = ctypes.c_int
        lib.ckpt_solve_quadratic.argtypes = [vp, LP, vp, vp, vp, vp, vp]
        lib.ckpt_cubic_cells.restype = ctypes.c_int64
        lib.ckpt_cubic_cells.argtypes = [ctypes.c_int32]
        lib.ckpt_status_string.restype = ctypes.c_char_p
        lib.ckpt_status_string.argtypes = [ctypes.c_int]
        i64 = ctypes.c_int64
        lib.ckpt_ragged_workspace_bytes.restype = ctypes.c_size_t
        lib.ckpt_ragged_workspace_bytes.argtypes = [ctypes.c_int, vp, i64]
        lib.ckpt_ragged_eval_peak.restype = ctypes.c_int
        lib.ckpt_ragged_eval_peak.argtypes = [vp, vp, vp, vp, i64, ctypes.c_int, vp, vp, vp, ctypes.c_size_t, vp]
        lib.ckpt_ragged_eval_timeline.restype = ctypes.c_int
        lib.ckpt_ragged_eval_timeline.argtypes = [vp, vp, vp, vp, i64, ctypes.c_int, vp, vp, vp, ctypes.c_size_t, vp]
        lib.ckpt_ragged_solve_linear.restype = ctypes.c_int
        lib.ckpt_ragged_solve_linear.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.ckpt_ragged_solve_cubic.restype = ctypes.c_int
        lib.ckpt_ragged_solve_cubic.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.ckpt_probe_hbm_read.restype = ctypes.c_int
        lib.ckpt_probe_hbm_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        lib.ckpt_probe_hbm_copy.restype = ctypes.c_int
        lib.ckpt_probe_hbm_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.ckpt_probe_valu.restype = ctypes.c_int
        lib.ckpt_probe_valu.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int32, vp, vp]
        lib.ckpt_probe_lds.restype = ctypes.c_int
        lib.ckpt_probe_lds.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int32, vp, vp]
        _lib = lib
    return _lib


class CkptError(RuntimeError):
    def __init__(self, call, code):
        self.code = code
        super().__init__(f"{call} failed: {status_string(code)} ({code})")


def status_string(code):
    return load().ckpt_status_string(int(code)).decode()


def cubic_cells(n_layers):
    return int(load().ckpt_cubic_cells(int(n_layers)))


def layout_of(t, chain_major=False):
    """ckpt_layout for a 2-D tensor of sizes or masks (strides in elements)."""
    if t.dim() != 2:
        raise ValueError("expected a 2-D tensor")
    if chain_major:
        batch, n1 = t.shape
        cs, ps = t.stride(0), t.stride(1)
    else:
        n1, batch = t.shape
        ps, cs = t.stride(0), t.stride(1)
    if batch == 1:      # a lone chain: any positive chain stride addresses it
        cs = max(cs, 1)
    return Layout(batch, n1 - 1, cs, ps)


def workspace_bytes(which, layout):
    return int(load().ckpt_workspace_bytes(int(which), ctypes.byref(layout)))


def _workspace(which, layout, device, workspace):
    need = workspace_bytes(which, layout)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, workspace.numel()


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _check_inputs(d, mask=None):
    if d.dtype != torch.int64 or not d.is_cuda:
        raise TypeError("d must be an int64 tensor on the GPU")
    if mask is not None:
        if mask.dtype != torch.uint8 or not mask.is_cuda:
            raise TypeError("mask must be a uint8 tensor on the GPU")
        if mask.shape != d.shape or mask.stride() != d.stride():
            raise ValueError("mask must have the shape and strides of d")


def ckpt_eval_peak(d, mask, objective, chain_major=False, want_status=True):
    """Peak memory of each chain's checkpoint set.  Returns (peak, status); with OBJ_BOTH peak has
    shape (2, batch): the static peaks, then the dynamic ones."""
    _check_inputs(d, mask)
    L = layout_of(d, chain_major)
    shape = (2, L.batch) if int(objective) == OBJ_BOTH else (L.batch,)
    peak = torch.empty(shape, dtype=torch.int64, device=d.device)
    status = torch.empty(L.batch, dtype=torch.int32, device=d.device) if want_status else None
    rc = load().ckpt_eval_peak(_ptr(d), _ptr(mask), ctypes.byref(L), int(objective), _ptr(peak), _ptr(status),
                               None, 0, _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_eval_peak", rc)
    return peak, status


def ckpt_eval_timeline(d, mask, objective, chain_major=False, want_status=True):
    """Memory per training phase index 0..2n+1 of each chain's set.  Returns
    (timeline, status); timeline has shape (2n+2, batch), or (batch, 2n+2) with
    ``chain_major``."""
    _check_inputs(d, mask)
    L = layout_of(d, chain_major)
    phases = 2 * L.n_layers + 2
    if chain_major:
        out = torch.empty((L.batch, phases), dtype=torch.int64, device=d.device)
        ocs, ops = phases, 1
    else:
        out = torch.empty((phases, L.batch), dtype=torch.int64, device=d.device)
        ocs, ops = 1, max(L.batch, 1)
    status = torch.empty(L.batch, dtype=torch.int32, device=d.device) if want_status else None
    rc = load().ckpt_eval_timeline(_ptr(d), _ptr(mask), ctypes.byref(L), int(objective), _ptr(out), ocs, ops,
                                   _ptr(status), _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_eval_timeline", rc)
    return out, status


def ckpt_select_baseline(like, kind, chain_major=False):
    """A size-independent checkpoint set for every chain; ``like`` is the sizes
    tensor (or a mask) whose shape and strides the result takes."""
    L = layout_of(like, chain_major)
    mask = torch.empty_strided(like.shape, like.stride(), dtype=torch.uint8, device=like.device)
    rc = load().ckpt_select_baseline(ctypes.byref(L), int(kind), _ptr(mask), _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_select_baseline", rc)
    return mask


def ckpt_solve_cubic(d, chain_major=False, workspace=None, want_status=True):
    """Optimal set under the static objective.  Returns (mask, peak, budget, status)."""
    _check_inputs(d)
    L = layout_of(d, chain_major)
    mask = torch.empty_strided(d.shape, d.stride(), dtype=torch.uint8, device=d.device)
    peak = torch.empty(L.batch, dtype=torch.int64, device=d.device)
    budget = torch.empty(L.batch, dtype=torch.int64, device=d.device)
    status = torch.empty(L.batch, dtype=torch.int32, device=d.device) if want_status else None
    ws, ws_bytes = _workspace(CALL_SOLVE_CUBIC, L, d.device, workspace)
    rc = load().ckpt_solve_cubic(_ptr(d), ctypes.byref(L), _ptr(mask), _ptr(peak), _ptr(budget), _ptr(status),
                                 _ptr(ws), ws_bytes, _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_solve_cubic", rc)
    return mask, peak, budget, status


def ckpt_solve_cubic_pruned(d, chain_major=False, workspace=None, want_status=True):
    """ckpt_solve_cubic without the budgets that cannot be optimal.  Returns
    (mask, peak, budget, evaluated, status); evaluated counts the budgets run."""
    _check_inputs(d)
    L = layout_of(d, chain_major)
    mask = torch.empty_strided(d.shape, d.stride(), dtype=torch.uint8, device=d.device)
    peak = torch.empty(L.batch, dtype=torch.int64, device=d.device)
    budget = torch.empty(L.batch, dtype=torch.int64, device=d.device)
    evaluated = torch.empty(L.batch, dtype=torch.int64, device=d.device)
    status = torch.empty(L.batch, dtype=torch.int32, device=d.device) if want_status else None
    ws, ws_bytes = _workspace(CALL_SOLVE_CUBIC, L, d.device, workspace)
    rc = load().ckpt_solve_cubic_pruned(_ptr(d), ctypes.byref(L), _ptr(mask), _ptr(peak), _ptr(budget),
                                        _ptr(evaluated), _ptr(status), _ptr(ws), ws_bytes, _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_solve_cubic_pruned", rc)
    return mask, peak, budget, evaluated, status


def ckpt_solve_cubic_costs(d, chain_major=False, workspace=None):
    """ckpt_solve_cubic plus the cost s + c_s of every candidate budget.  Returns
    (mask, peak, budget, budgets, costs, status); budgets and costs have shape
    (batch, ckpt_cubic_costs_len(n)), -1 in the unused places."""
    _check_inputs(d)
    L = layout_of(d, chain_major)
    per = int(load().ckpt_cubic_costs_len(L.n_layers))
    mask = torch.empty_strided(d.shape, d.stride(), dtype=torch.uint8, device=d.device)
    peak = torch.empty(L.batch, dtype=torch.int64, device=d.device)
    budget = torch.empty(L.batch, dtype=torch.int64, device=d.device)
    budgets = torch.empty((L.batch, per), dtype=torch.int64, device=d.device)
    costs = torch.empty((L.batch, per), dtype=torch.int64, device=d.device)
    status = torch.empty(L.batch, dtype=torch.int32, device=d.device)
    ws, ws_bytes = _workspace(CALL_SOLVE_CUBIC, L, d.device, workspace)
    rc = load().ckpt_solve_cubic_costs(_ptr(d), ctypes.byref(L), _ptr(mask), _ptr(peak), _ptr(budget),
                                       _ptr(budgets), _ptr(costs), _ptr(status), _ptr(ws), ws_bytes, _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_solve_cubic_costs", rc)
    return mask, peak, budget, budgets, costs, status


def ckpt_solve_linear(d, chain_major=False, workspace=None, want_status=True):
    """Optimal set under the dynamic objective.  Returns (mask, peak, status)."""
    _check_inputs(d)
    L = layout_of(d, chain_major)
    mask = torch.empty_strided(d.shape, d.stride(), dtype=torch.uint8, device=d.device)
    peak = torch.empty(L.batch, dtype=torch.int64, device=d.device)
    status = torch.empty(L.batch, dtype=torch.int32, device=d.device) if want_status else None
    ws, ws_bytes = _workspace(CALL_SOLVE_LINEAR, L, d.device, workspace)
    rc = load().ckpt_solve_linear(_ptr(d), ctypes.byref(L), _ptr(mask), _ptr(peak), _ptr(status),
                                  _ptr(ws), ws_bytes, _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_solve_linear", rc)
    return mask, peak, status


def ckpt_solve_linear_noalloc(d, mask, peak, status=None, chain_major=False):
    """ckpt_solve_linear into tensors the caller already holds, with the library's own
    scratch: nothing is allocated here or in the library.  Returns None."""
    _check_inputs(d)
    L = layout_of(d, chain_major)
    rc = load().ckpt_solve_linear_noalloc(_ptr(d), ctypes.byref(L), _ptr(mask), _ptr(peak), _ptr(status), _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_solve_linear_noalloc", rc)


def ckpt_solve_quadratic(d, chain_major=False, want_values=True, want_status=True):
    """Optimal set under the dynamic objective by the quadratic-time recurrence.
    Returns (mask, peak, values, status); values holds M(i) in the layout of d."""
    _check_inputs(d)
    L = layout_of(d, chain_major)
    mask = torch.empty_strided(d.shape, d.stride(), dtype=torch.uint8, device=d.device)
    peak = torch.empty(L.batch, dtype=torch.int64, device=d.device)
    values = torch.empty_strided(d.shape, d.stride(), dtype=torch.int64, device=d.device) if want_values else None
    status = torch.empty(L.batch, dtype=torch.int32, device=d.device) if want_status else None
    rc = load().ckpt_solve_quadratic(_ptr(d), ctypes.byref(L), _ptr(mask), _ptr(peak), _ptr(values), _ptr(status),
                                     _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_solve_quadratic", rc)
    return mask, peak, values, status


# ---- ragged batches: chains of different n in one flat array ------------------------------------

def _ragged_args(d, offsets, mask=None, offsets_dev=None):
    """(offsets as a contiguous host int64 array, its pointer, batch) after the type checks.
    offsets_dev, if given, is the caller's copy of the offsets on the GPU."""
    import numpy as np
    if d.dtype != torch.int64 or not d.is_cuda or d.dim() != 1 or not d.is_contiguous():
        raise TypeError("d must be a flat contiguous int64 tensor on the GPU")
    if mask is not None and (mask.dtype != torch.uint8 or not mask.is_cuda or mask.shape != d.shape
                             or not mask.is_contiguous()):
        raise TypeError("mask must be a flat uint8 tensor on the GPU, as long as d")
    off = np.ascontiguousarray(offsets.numpy() if isinstance(offsets, torch.Tensor) else offsets, dtype=np.int64)
    if off.ndim != 1 or off.size < 1:
        raise ValueError("offsets must hold batch + 1 values")
    if int(off[-1]) > d.numel():
        raise ValueError("offsets reach past the end of d")
    if offsets_dev is not None and (offsets_dev.dtype != torch.int64 or not offsets_dev.is_cuda
                                    or offsets_dev.numel() != off.size or not offsets_dev.is_contiguous()):
        raise TypeError("offsets_dev must be the offsets as a contiguous int64 tensor on the GPU")
    return off, ctypes.c_void_p(off.ctypes.data), off.size - 1


def _ragged_workspace(which, off_ptr, batch, device, workspace):
    """The caller's workspace as it is (the library checks its size), else one of the size the
    library asks for (a pass over the offsets on the host)."""
    if workspace is None:
        need = load().ckpt_ragged_workspace_bytes(int(which), off_ptr, batch)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, workspace.numel()


def ckpt_ragged_eval_peak(d, mask, offsets, objective, workspace=None, offsets_dev=None):
    """Peak memory of each chain's set; chain c is d[offsets[c]:offsets[c+1]].  Returns (peak, status);
    with OBJ_BOTH peak has shape (2, batch)."""
    off, off_ptr, batch = _ragged_args(d, offsets, mask, offsets_dev)
    shape = (2, batch) if int(objective) == OBJ_BOTH else (batch,)
    peak = torch.empty(shape, dtype=torch.int64, device=d.device)
    status = torch.empty(batch, dtype=torch.int32, device=d.device)
    ws, ws_bytes = _ragged_workspace(CALL_EVAL_PEAK, off_ptr, batch, d.device, workspace)
    rc = load().ckpt_ragged_eval_peak(_ptr(d), _ptr(mask), off_ptr, _ptr(offsets_dev), batch, int(objective), _ptr(peak), _ptr(status),
                                      _ptr(ws), ws_bytes, _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_ragged_eval_peak", rc)
    return peak, status


def ckpt_ragged_eval_timeline(d, mask, offsets, objective, workspace=None, offsets_dev=None):
    """Memory per phase of each chain, flat: chain c from element 2*offsets[c].  Returns (timeline, status)."""
    off, off_ptr, batch = _ragged_args(d, offsets, mask, offsets_dev)
    out = torch.empty(2 * d.numel(), dtype=torch.int64, device=d.device)
    status = torch.empty(batch, dtype=torch.int32, device=d.device)
    ws, ws_bytes = _ragged_workspace(CALL_EVAL_TIMELINE, off_ptr, batch, d.device, workspace)
    rc = load().ckpt_ragged_eval_timeline(_ptr(d), _ptr(mask), off_ptr, _ptr(offsets_dev), batch, int(objective), _ptr(out),
                                          _ptr(status), _ptr(ws), ws_bytes, _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_ragged_eval_timeline", rc)
    return out, status


def ckpt_ragged_solve_linear(d, offsets, workspace=None, offsets_dev=None):
    """Optimal sets under the dynamic objective.  Returns (flat mask, peak, status)."""
    off, off_ptr, batch = _ragged_args(d, offsets, None, offsets_dev)
    mask = torch.empty(d.numel(), dtype=torch.uint8, device=d.device)
    peak = torch.empty(batch, dtype=torch.int64, device=d.device)
    status = torch.empty(batch, dtype=torch.int32, device=d.device)
    ws, ws_bytes = _ragged_workspace(CALL_SOLVE_LINEAR, off_ptr, batch, d.device, workspace)
    rc = load().ckpt_ragged_solve_linear(_ptr(d), off_ptr, _ptr(offsets_dev), batch, _ptr(mask), _ptr(peak), _ptr(status),
                                         _ptr(ws), ws_bytes, _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_ragged_solve_linear", rc)
    return mask, peak, status


def ckpt_ragged_solve_cubic(d, offsets, workspace=None, offsets_dev=None):
    """Optimal sets under the static objective.  Returns (flat mask, peak, budget, status)."""
    off, off_ptr, batch = _ragged_args(d, offsets, None, offsets_dev)
    mask = torch.empty(d.numel(), dtype=torch.uint8, device=d.device)
    peak = torch.empty(batch, dtype=torch.int64, device=d.device)
    budget = torch.empty(batch, dtype=torch.int64, device=d.device)
    status = torch.empty(batch, dtype=torch.int32, device=d.device)
    ws, ws_bytes = _ragged_workspace(CALL_SOLVE_CUBIC, off_ptr, batch, d.device, workspace)
    rc = load().ckpt_ragged_solve_cubic(_ptr(d), off_ptr, _ptr(offsets_dev), batch, _ptr(mask), _ptr(peak), _ptr(budget), _ptr(status),
                                        _ptr(ws), ws_bytes, _stream())
    if rc != CKPT_OK:
        raise CkptError("ckpt_ragged_solve_cubic", rc)
    return mask, peak, budget, status


# ---- measurement probes (include/ckpt_probe.h) ------------------------------------------------

PROBE_VALU = {"v_add_u32": 0, "v_min_i32": 1, "v_max_u32": 2, "v_cndmask_b32": 3}
PROBE_LDS = {"ds_read_b32": 0, "ds_write_b32": 1, "ds_max_u32": 2}


def _probe(name, rc):
    if rc != CKPT_OK:
        raise CkptError(name, rc)


def ckpt_probe_hbm_read(src, sink):
    """Enqueues the read-only streaming kernel over the bytes of ``src``."""
    _probe("ckpt_probe_hbm_read",
           load().ckpt_probe_hbm_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream()))


def ckpt_probe_hbm_copy(src, dst):
    _probe("ckpt_probe_hbm_copy",
           load().ckpt_probe_hbm_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream()))


def ckpt_probe_valu(which, waves, iters, sink):
    """Returns the lane-operations the launch executes."""
    _probe("ckpt_probe_valu", load().ckpt_probe_valu(int(which), int(waves), int(iters), _ptr(sink), _stream()))
    return int(waves) * 64 * int(iters) * 256


def ckpt_probe_lds(which, waves, iters, sink):
    """Returns the LDS lane-accesses the launch executes."""
    _probe("ckpt_probe_lds", load().ckpt_probe_lds(int(which), int(waves), int(iters), _ptr(sink), _stream()))
    return int(waves) * 64 * int(iters) * 16
