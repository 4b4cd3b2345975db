"""ctypes binding of the host-side planner entry points declared in include/ss_plan.h (same shared
library).  Argument marshalling only: nothing is computed here."""
from __future__ import annotations

import ctypes as C

from . import binding as _b

EXPORTS = ("ss_plan_dependencies", "ss_plan_validate", "ss_rvd_search")
SS_PLAN_MAX_DIMS = 4
PRIMITIVE_NAMES = ("all-reduce", "all-gather", "reduce-scatter", "all-to-all", "schunk", "vchunk")


class ss_vtensor(C.Structure):
    _fields_ = [("op", C.c_int32), ("tensor", C.c_int32), ("ndim", C.c_int32), ("lo", C.c_int64 * SS_PLAN_MAX_DIMS),
                ("hi", C.c_int64 * SS_PLAN_MAX_DIMS)]


class ss_link_model(C.Structure):
    _fields_ = [("alpha_ns", C.c_int64), ("link_bytes_per_us", C.c_int64), ("local_ns", C.c_int64)]


class ss_rvd_step(C.Structure):
    _fields_ = [("primitive", C.c_int32), ("axis", C.c_int32), ("axis2", C.c_int32), ("group", C.c_int32),
                ("state", C.c_int32 * (2 + SS_PLAN_MAX_DIMS)), ("time_ns", C.c_int64)]


_ready = False


def lib():
    global _ready
    L = _b.lib()
    if not _ready:
        I32P = C.POINTER(C.c_int32)
        L.ss_plan_dependencies.argtypes = [C.POINTER(ss_vtensor), C.c_int32, C.POINTER(ss_vtensor), C.c_int32, I32P, C.c_int32, I32P]
        L.ss_plan_dependencies.restype = C.c_int
        L.ss_plan_validate.argtypes = [C.c_int32, I32P, C.c_int32, I32P, I32P, C.c_int32, I32P, I32P, I32P]
        L.ss_plan_validate.restype = C.c_int
        L.ss_rvd_search.argtypes = [I32P, I32P, C.c_int32, C.c_int64, C.POINTER(ss_link_model), C.POINTER(ss_rvd_step), C.c_int32,
                                    I32P, C.POINTER(C.c_int64)]
        L.ss_rvd_search.restype = C.c_int
        _ready = True
    return L


def _vt(items):
    arr = (ss_vtensor * max(1, len(items)))()
    for i, (op, tensor, lo, hi) in enumerate(items):
        arr[i].op, arr[i].tensor, arr[i].ndim = op, tensor, len(lo)
        for d in range(min(len(lo), SS_PLAN_MAX_DIMS)):
            arr[i].lo[d], arr[i].hi[d] = lo[d], hi[d]
    return arr


def _i32(values):
    flat = [int(x) for x in values]
    return (C.c_int32 * max(1, len(flat)))(*flat)


def ss_plan_dependencies(produced, consumed, capacity=None):
    """produced / consumed: lists of (op, tensor, lo tuple, hi tuple).  Returns the list of (producer, consumer)."""
    cap = len(produced) * len(consumed) if capacity is None else capacity
    edges, n = (C.c_int32 * max(1, 2 * cap))(), C.c_int32(0)
    rc = lib().ss_plan_dependencies(_vt(produced), len(produced), _vt(consumed), len(consumed), edges, cap, C.byref(n))
    if rc != _b.SS_OK:
        raise _b.SSAttnError(rc, "ss_plan_dependencies")
    return [(edges[2 * i], edges[2 * i + 1]) for i in range(n.value)]


def ss_plan_validate(n_ops, fixed_edges, alternatives=()):
    """Returns (feasible, choice tuple or None, order list or None)."""
    fixed = _i32([x for e in fixed_edges for x in e])
    alt = _i32([x for g in alternatives for e in g for x in e])
    sizes = _i32([len(g) for g in alternatives])
    feasible, choice, order = C.c_int32(0), (C.c_int32 * max(1, len(alternatives)))(), (C.c_int32 * max(1, n_ops))()
    rc = lib().ss_plan_validate(n_ops, fixed, len(fixed_edges), alt, sizes, len(alternatives), C.byref(feasible), choice, order)
    if rc != _b.SS_OK:
        raise _b.SSAttnError(rc, "ss_plan_validate")
    if not feasible.value:
        return False, None, None
    return True, tuple(choice[i] for i in range(len(alternatives))), [order[i] for i in range(n_ops)]


def ss_rvd_search(src, dst, tensor_bytes, alpha_ns=10000, link_bytes_per_us=153000, local_ns=1000, capacity=32):
    """src / dst: (r, v, d1, .., dn).  Returns (total_ns, [(primitive, axis, axis2, group, state_after, time_ns)])
    or None when dst cannot be reached."""
    ndim = len(src) - 2
    model = ss_link_model(alpha_ns, link_bytes_per_us, local_ns)
    steps, n, total = (ss_rvd_step * max(1, capacity))(), C.c_int32(0), C.c_int64(0)
    rc = lib().ss_rvd_search(_i32(src), _i32(dst), ndim, int(tensor_bytes), C.byref(model), steps, capacity, C.byref(n), C.byref(total))
    if rc == _b.SS_ERR_UNSUPPORTED:
        return None
    if rc != _b.SS_OK:
        raise _b.SSAttnError(rc, "ss_rvd_search")
    out = [(s.primitive, s.axis, s.axis2, s.group, tuple(s.state[i] for i in range(2 + ndim)), s.time_ns) for s in steps[:n.value]]
    return total.value, out
