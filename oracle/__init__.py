"""CPU oracle for checkpoint selection -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrappers over ``ckpt_oracle.c`` (the plain C reference, see its
header).  Only the tests, the smoke check and the benchmark's CPU-baseline leg
may import this package; the GPU library never does and shares no code with it.

Arrays here are chain-major: a batch is ``d[batch, n+1]`` (int64) and
``mask[batch, n+1]`` (uint8); a single chain is a 1-D array of n+1 entries.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ckpt_oracle.c")
_LIB = os.path.join(_HERE, "libckpt_oracle.so")
_lib = None

_i64p = ctypes.POINTER(ctypes.c_int64)
_u8p = ctypes.POINTER(ctypes.c_uint8)


def build(force=False):
    """Compile ckpt_oracle.c with gcc into libckpt_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-Wall", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        I, P, U, N = ctypes.c_int64, _i64p, _u8p, ctypes.c_int
        sig = {
            "orc_peak_static": (I, [P, U, N]),
            "orc_peak_dynamic": (I, [P, U, N]),
            "orc_sim_static": (I, [P, U, N]),
            "orc_sim_dynamic": (I, [P, U, N]),
            "orc_timeline": (None, [P, U, N, N, P]),
            "orc_select_baseline": (None, [N, N, U]),
            "orc_batch_timeline": (None, [P, U, I, N, N, P]),
            "orc_brute": (I, [P, N, N, P, P]),
            "orc_num_budgets": (I, [N]),
            "orc_budgets": (None, [P, N, P]),
            "orc_solve_static_literal": (I, [P, N, U, P]),
            "orc_solve_static_range": (I, [P, N, U, P, I, I]),
            "orc_solve_static": (I, [P, N, U, P]),
            "orc_static_cs": (I, [P, N, I]),
            "orc_solve_dynamic": (I, [P, N, U, P]),
            "orc_solve_dynamic_literal": (I, [P, N, P]),
            "orc_batch_peak": (None, [P, U, I, N, N, P]),
            "orc_batch_solve_dynamic": (None, [P, I, N, U, P]),
            "orc_batch_solve_static": (None, [P, I, N, U, P, P]),
            "orc_max_threads": (N, []),
            "orc_set_threads": (None, [N]),
            "orc_ragged_peak": (None, [P, U, P, I, N, P]),
            "orc_ragged_timeline": (None, [P, U, P, I, N, P]),
            "orc_ragged_solve_dynamic": (None, [P, P, I, U, P]),
            "orc_ragged_solve_static": (None, [P, P, I, U, P, P]),
            "orc_static_cs_list": (None, [P, N, P, I, P]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(_i64p)


def _m(a):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a, a.ctypes.data_as(_u8p)


def max_threads():
    return int(_load().orc_max_threads())


def set_threads(t):
    """Threads for the batch and budget loops from now on (t < 1: all processors)."""
    _load().orc_set_threads(int(t))


# ---- objective functions (single chain) ------------------------------------

def peak_static(d, mask):
    d, dp = _d(d); mask, mp = _m(mask)
    return int(_load().orc_peak_static(dp, mp, len(d) - 1))


def peak_dynamic(d, mask):
    d, dp = _d(d); mask, mp = _m(mask)
    return int(_load().orc_peak_dynamic(dp, mp, len(d) - 1))


def sim_static(d, mask):
    d, dp = _d(d); mask, mp = _m(mask)
    return int(_load().orc_sim_static(dp, mp, len(d) - 1))


def sim_dynamic(d, mask):
    d, dp = _d(d); mask, mp = _m(mask)
    return int(_load().orc_sim_dynamic(dp, mp, len(d) - 1))


def timeline(d, mask, objective):
    """Memory per training phase index 0..2n+1 (Algorithm 2 / Algorithm 3 events)."""
    d, dp = _d(d); mask, mp = _m(mask)
    n = len(d) - 1
    out = np.empty(2 * n + 2, dtype=np.int64)
    _load().orc_timeline(dp, mp, n, int(objective), out.ctypes.data_as(_i64p))
    return out


SELECT_NONE, SELECT_ALL, SELECT_SQRT = 0, 1, 2


def select_baseline(n, kind):
    """Size-independent checkpoint sets: ends only, every position, sqrt(n) rule."""
    mask = np.zeros(n + 1, dtype=np.uint8)
    _load().orc_select_baseline(int(n), int(kind), mask.ctypes.data_as(_u8p))
    return mask


# ---- brute force ---------------------------------------------------------------

def brute(d, objective):
    """(optimum, number of optimal sets, smallest max-segment among them)."""
    d, dp = _d(d)
    n = len(d) - 1
    assert 1 <= n <= 24
    cnt = ctypes.c_int64(0); seg = ctypes.c_int64(0)
    v = _load().orc_brute(dp, n, int(objective), ctypes.byref(cnt), ctypes.byref(seg))
    return int(v), int(cnt.value), int(seg.value)


# ---- static objective ------------------------------------------------------------

def num_budgets(n):
    return int(_load().orc_num_budgets(n))


def budgets(d):
    d, dp = _d(d)
    n = len(d) - 1
    out = np.empty(num_budgets(n), dtype=np.int64)
    _load().orc_budgets(dp, n, out.ctypes.data_as(_i64p))
    return out


def _solve_static(fn, d, *extra):
    d, dp = _d(d)
    n = len(d) - 1
    mask = np.zeros(n + 1, dtype=np.uint8)
    s = ctypes.c_int64(0)
    v = fn(dp, n, mask.ctypes.data_as(_u8p), ctypes.byref(s), *extra)
    return int(v), mask, int(s.value)


def solve_static_literal(d):
    """(optimum, canonical mask, s*) by the literal O(n^4) form."""
    return _solve_static(_load().orc_solve_static_literal, d)


def solve_static(d):
    """(optimum, canonical mask, s*) by Algorithm 4's queue over all budgets."""
    return _solve_static(_load().orc_solve_static, d)


def solve_static_range(d, first, num):
    """Best (cost, s) over budgets [first, first+num) only; no mask."""
    d, dp = _d(d)
    s = ctypes.c_int64(0)
    v = _load().orc_solve_static_range(dp, len(d) - 1, None, ctypes.byref(s), first, num)
    return int(v), int(s.value)


def static_cs(d, s):
    d, dp = _d(d)
    return int(_load().orc_static_cs(dp, len(d) - 1, int(s)))


# ---- dynamic objective -----------------------------------------------------------

def solve_dynamic(d):
    """(M(0), canonical mask, M[0..n]) by Algorithm 5."""
    d, dp = _d(d)
    n = len(d) - 1
    mask = np.zeros(n + 1, dtype=np.uint8)
    M = np.empty(n + 1, dtype=np.int64)
    v = _load().orc_solve_dynamic(dp, n, mask.ctypes.data_as(_u8p), M.ctypes.data_as(_i64p))
    return int(v), mask, M


def solve_dynamic_literal(d):
    d, dp = _d(d)
    n = len(d) - 1
    M = np.empty(n + 1, dtype=np.int64)
    v = _load().orc_solve_dynamic_literal(dp, n, M.ctypes.data_as(_i64p))
    return int(v), M


# ---- batches (chain-major [batch, n+1]) ---------------------------------------

def batch_peak(d, mask, objective):
    d, dp = _d(d); mask, mp = _m(mask)
    B, n1 = d.shape
    out = np.empty(B, dtype=np.int64)
    _load().orc_batch_peak(dp, mp, B, n1 - 1, int(objective), out.ctypes.data_as(_i64p))
    return out


def batch_timeline(d, mask, objective):
    d, dp = _d(d); mask, mp = _m(mask)
    B, n1 = d.shape
    out = np.empty((B, 2 * n1), dtype=np.int64)
    _load().orc_batch_timeline(dp, mp, B, n1 - 1, int(objective), out.ctypes.data_as(_i64p))
    return out


def batch_solve_dynamic(d, want_mask=True):
    d, dp = _d(d)
    B, n1 = d.shape
    mask = np.zeros((B, n1), dtype=np.uint8) if want_mask else None
    peak = np.empty(B, dtype=np.int64)
    _load().orc_batch_solve_dynamic(dp, B, n1 - 1,
                                    mask.ctypes.data_as(_u8p) if want_mask else None,
                                    peak.ctypes.data_as(_i64p))
    return peak, mask


def batch_solve_static(d, want_mask=True):
    d, dp = _d(d)
    B, n1 = d.shape
    mask = np.zeros((B, n1), dtype=np.uint8) if want_mask else None
    peak = np.empty(B, dtype=np.int64)
    s = np.empty(B, dtype=np.int64)
    _load().orc_batch_solve_static(dp, B, n1 - 1,
                                   mask.ctypes.data_as(_u8p) if want_mask else None,
                                   peak.ctypes.data_as(_i64p), s.ctypes.data_as(_i64p))
    return peak, mask, s


def static_cs_list(d, s_list):
    """c_s (Equation (T), literal recurrence) for every budget of a list."""
    d, dp = _d(d)
    sl = np.ascontiguousarray(s_list, dtype=np.int64)
    out = np.empty(len(sl), dtype=np.int64)
    _load().orc_static_cs_list(dp, len(d) - 1, sl.ctypes.data_as(_i64p), len(sl), out.ctypes.data_as(_i64p))
    return out


# ---- ragged batches: 1-D d (and mask) with offsets[batch+1]; chain c is d[off[c]:off[c+1]] ----

def _off(offsets):
    o = np.ascontiguousarray(offsets, dtype=np.int64)
    return o, o.ctypes.data_as(_i64p)


def ragged_peak(d, mask, offsets, objective):
    d, dp = _d(d); mask, mp = _m(mask); o, op = _off(offsets)
    out = np.empty(len(o) - 1, dtype=np.int64)
    _load().orc_ragged_peak(dp, mp, op, len(o) - 1, int(objective), out.ctypes.data_as(_i64p))
    return out


def ragged_timeline(d, mask, offsets, objective):
    """1-D array; the 2 n_c + 2 phases of chain c start at 2 * offsets[c]."""
    d, dp = _d(d); mask, mp = _m(mask); o, op = _off(offsets)
    out = np.empty(2 * len(d), dtype=np.int64)
    _load().orc_ragged_timeline(dp, mp, op, len(o) - 1, int(objective), out.ctypes.data_as(_i64p))
    return out


def ragged_solve_dynamic(d, offsets):
    d, dp = _d(d); o, op = _off(offsets)
    mask = np.zeros(len(d), dtype=np.uint8)
    peak = np.empty(len(o) - 1, dtype=np.int64)
    _load().orc_ragged_solve_dynamic(dp, op, len(o) - 1, mask.ctypes.data_as(_u8p), peak.ctypes.data_as(_i64p))
    return peak, mask


def ragged_solve_static(d, offsets):
    d, dp = _d(d); o, op = _off(offsets)
    mask = np.zeros(len(d), dtype=np.uint8)
    peak = np.empty(len(o) - 1, dtype=np.int64)
    s = np.empty(len(o) - 1, dtype=np.int64)
    _load().orc_ragged_solve_static(dp, op, len(o) - 1, mask.ctypes.data_as(_u8p), peak.ctypes.data_as(_i64p),
                                    s.ctypes.data_as(_i64p))
    return peak, mask, s
