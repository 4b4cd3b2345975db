"""ctypes binding of the feed-forward entry points declared in include/ss_ffn.h (same shared
library as the attention entry points).  Argument marshalling only: nothing is computed here."""
from __future__ import annotations

import ctypes as C

from . import binding as _b

SS_ACT_RELU, SS_ACT_GELU_TANH = 0, 1
SS_FFN_FLAG_EXACT_SUM = 1
EXPORTS = ("ss_ffn_workspace_bytes", "ss_ffn_chunk_range", "ss_ffn_fwd", "ss_ffn_bwd", "ss_ffn_profile_enable",
           "ss_ffn_profile_read")
KERNEL_NAMES = ("up", "down", "dh", "dw2", "dw1", "dx", "colsum")


class ss_ffn_desc(C.Structure):
    _fields_ = [
        ("T", C.c_int32), ("dm", C.c_int32), ("dh", C.c_int32), ("dtype", C.c_int32), ("act", C.c_int32),
        ("ld_x", C.c_int64), ("ld_w1", C.c_int64), ("ld_w2", C.c_int64),
        ("lo", C.c_int32), ("hi", C.c_int32), ("k", C.c_int32), ("flags", C.c_int32),
    ]


_ready = False


def lib():
    global _ready
    L = _b.lib()
    if not _ready:
        P, V = C.POINTER(ss_ffn_desc), C.c_void_p
        L.ss_ffn_workspace_bytes.argtypes = [P, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.ss_ffn_workspace_bytes.restype = C.c_int
        L.ss_ffn_chunk_range.argtypes = [P, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.ss_ffn_chunk_range.restype = C.c_int
        L.ss_ffn_fwd.argtypes = [P, V, V, V, V, V, V, V, C.c_size_t, V]
        L.ss_ffn_fwd.restype = C.c_int
        L.ss_ffn_bwd.argtypes = [P, V, V, V, V, V, V, V, V, V, V, V, C.c_size_t, V]
        L.ss_ffn_bwd.restype = C.c_int
        L.ss_ffn_profile_enable.argtypes = [C.c_int]
        L.ss_ffn_profile_enable.restype = C.c_int
        L.ss_ffn_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.ss_ffn_profile_read.restype = C.c_int
        _ready = True
    return L


def make_desc(T, dm, dh, lo, hi, k, *, act=SS_ACT_GELU_TANH, ld_x=None, ld_w1=None, ld_w2=None, dtype=_b.SS_BF16,
              flags=0) -> ss_ffn_desc:
    return ss_ffn_desc(T, dm, dh, dtype, act, dm if ld_x is None else ld_x, dh if ld_w1 is None else ld_w1,
                       dm if ld_w2 is None else ld_w2, lo, hi, k, flags)


def _check(rc, where):
    if rc != _b.SS_OK:
        raise _b.SSAttnError(rc, where)


def ss_ffn_workspace_bytes(desc):
    f, b = C.c_size_t(0), C.c_size_t(0)
    _check(lib().ss_ffn_workspace_bytes(C.byref(desc), C.byref(f), C.byref(b)), "ss_ffn_workspace_bytes")
    return f.value, b.value


def ss_ffn_chunk_range(desc, c):
    lo, hi = C.c_int32(0), C.c_int32(0)
    _check(lib().ss_ffn_chunk_range(C.byref(desc), c, C.byref(lo), C.byref(hi)), "ss_ffn_chunk_range")
    return lo.value, hi.value


def ss_ffn_fwd(desc, X, W1, b1, W2, b2, Y, workspace, workspace_bytes, stream):
    p = _b._ptr
    _check(lib().ss_ffn_fwd(C.byref(desc), p(X), p(W1), p(b1), p(W2), p(b2), p(Y), p(workspace), workspace_bytes,
                            stream), "ss_ffn_fwd")


def ss_ffn_bwd(desc, X, W1, b1, W2, dY, dX, dW1, db1, dW2, db2, workspace, workspace_bytes, stream):
    p = _b._ptr
    _check(lib().ss_ffn_bwd(C.byref(desc), p(X), p(W1), p(b1), p(W2), p(dY), p(dX), p(dW1), p(db1), p(dW2), p(db2),
                            p(workspace), workspace_bytes, stream), "ss_ffn_bwd")


def ss_ffn_profile_enable(on: bool):
    lib().ss_ffn_profile_enable(1 if on else 0)


def ss_ffn_profile_read(kernel: int):
    ms, n = C.c_double(0), C.c_int64(0)
    _check(lib().ss_ffn_profile_read(kernel, C.byref(ms), C.byref(n)), "ss_ffn_profile_read")
    return ms.value, n.value
