"""ctypes binding of libss_attn.so: argument marshalling only.

Functions carry the names of the C entry points declared in include/ss_attn.h.
Tensors are passed as objects with a `data_ptr()` method (torch tensors on the
GPU) or as raw integer addresses; nothing is computed here.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libss_attn.so")

SS_F32, SS_BF16 = 0, 1
SS_AXIS_HEAD, SS_AXIS_ROW = 0, 1
SS_MASK_NONE, SS_MASK_CAUSAL, SS_MASK_REGION = 0, 1, 2
SS_BIAS_NONE, SS_BIAS_DENSE, SS_BIAS_RELPOS = 0, 1, 2
SS_FLAG_GENERIC_KERNELS = 1
SS_OK = 0
SS_ERR_NULL, SS_ERR_BAD_SHAPE, SS_ERR_BAD_RANGE, SS_ERR_BAD_K = -1, -2, -3, -4
SS_ERR_UNSUPPORTED, SS_ERR_WORKSPACE, SS_ERR_HIP, SS_ERR_STATIC_SCRATCH = -5, -6, -7, -8
SS_ATTN_STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = ("ss_attn_workspace_bytes", "ss_attn_chunk_range", "ss_attn_fwd", "ss_attn_bwd", "ss_attn_bwd_static",
           "ss_strerror",
           "ss_attn_kernel_family", "ss_attn_profile_enable", "ss_attn_profile_read")
(SS_K_FWD, SS_K_RECOMPUTE, SS_K_DQ, SS_K_DKDV, SS_K_DBIAS, SS_K_TABLE_REDUCE, SS_K_DQ_DKDV, SS_K_DBIAS_FOLD,
 SS_K_RECOMPUTE_DQ, SS_K_COUNT) = range(10)
KERNEL_NAMES = ("fwd", "recompute", "dq", "dkdv", "dbias", "table_reduce", "dq_dkdv", "dbias_fold", "recompute_dq")


class ss_attn_desc(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("H", C.c_int32), ("S", C.c_int32), ("D", C.c_int32),
        ("dtype", C.c_int32), ("scale", C.c_float),
        ("stride_b", C.c_int64), ("stride_s", C.c_int64), ("stride_h", C.c_int64),
        ("bias_kind", C.c_int32), ("bias_dtype", C.c_int32),
        ("win_h", C.c_int32), ("win_w", C.c_int32),
        ("mask_kind", C.c_int32), ("mask_period", C.c_int32),
        ("gated", C.c_int32), ("shard_axis", C.c_int32),
        ("lo", C.c_int32), ("hi", C.c_int32), ("k", C.c_int32), ("flags", C.c_uint32),
    ]


class SSAttnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {ss_strerror(code)} ({code})")


_lib = None


def lib():
    """The loaded shared library.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2301_08984_amd.build` "
                "(there is no non-HIP fallback)")
        L = C.CDLL(LIB_PATH)
        P, V = C.POINTER(ss_attn_desc), C.c_void_p
        L.ss_attn_workspace_bytes.argtypes = [P, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.ss_attn_workspace_bytes.restype = C.c_int
        L.ss_attn_chunk_range.argtypes = [P, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.ss_attn_chunk_range.restype = C.c_int
        L.ss_attn_fwd.argtypes = [P, V, V, V, V, V, V, V, V, V, C.c_size_t, V]
        L.ss_attn_fwd.restype = C.c_int
        L.ss_attn_bwd.argtypes = [P, V, V, V, V, V, V, V, V, V, V, V, V, V, V, C.c_size_t, V]
        L.ss_attn_bwd.restype = C.c_int
        L.ss_attn_bwd_static.argtypes = [P, V, V, V, V, V, V, V, V, V, V, V, V, V, V]
        L.ss_attn_bwd_static.restype = C.c_int
        L.ss_attn_kernel_family.argtypes = [P]
        L.ss_attn_kernel_family.restype = C.c_char_p
        L.ss_attn_profile_enable.argtypes = [C.c_int]
        L.ss_attn_profile_enable.restype = C.c_int
        L.ss_attn_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.ss_attn_profile_read.restype = C.c_int
        L.ss_strerror.argtypes = [C.c_int]
        L.ss_strerror.restype = C.c_char_p
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def make_desc(B, H, S, D, dtype, scale, axis, lo, hi, k, *, stride_b=None, stride_s=None, stride_h=None,
              bias_kind=SS_BIAS_NONE, bias_dtype=None, win=(0, 0), mask_kind=SS_MASK_NONE, mask_period=0,
              gated=False, flags=0) -> ss_attn_desc:
    stride_h = D if stride_h is None else stride_h
    stride_s = H * D if stride_s is None else stride_s
    stride_b = S * H * D if stride_b is None else stride_b
    return ss_attn_desc(B, H, S, D, dtype, scale, stride_b, stride_s, stride_h, bias_kind,
                        dtype if bias_dtype is None else bias_dtype, win[0], win[1], mask_kind, mask_period,
                        1 if gated else 0, axis, lo, hi, k, flags)


def ss_strerror(code: int) -> str:
    return lib().ss_strerror(code).decode()


def ss_attn_workspace_bytes(desc: ss_attn_desc):
    """-> (fwd_bytes, bwd_bytes); raises SSAttnError on an invalid descriptor."""
    f, b = C.c_size_t(0), C.c_size_t(0)
    rc = lib().ss_attn_workspace_bytes(C.byref(desc), C.byref(f), C.byref(b))
    if rc != SS_OK:
        raise SSAttnError(rc, "ss_attn_workspace_bytes")
    return f.value, b.value


def ss_attn_chunk_range(desc: ss_attn_desc, c: int):
    lo, hi = C.c_int32(0), C.c_int32(0)
    rc = lib().ss_attn_chunk_range(C.byref(desc), c, C.byref(lo), C.byref(hi))
    if rc != SS_OK:
        raise SSAttnError(rc, "ss_attn_chunk_range")
    return lo.value, hi.value


def ss_attn_fwd(desc, Q, K, V, bias, region_ids, G, Y, lse, workspace, workspace_bytes, stream):
    rc = lib().ss_attn_fwd(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(bias), _ptr(region_ids), _ptr(G),
                           _ptr(Y), _ptr(lse), _ptr(workspace), workspace_bytes, stream)
    if rc != SS_OK:
        raise SSAttnError(rc, "ss_attn_fwd")


def ss_attn_bwd(desc, Q, K, V, bias, region_ids, G, dY, lse, dQ, dK, dV, dBias, dG, workspace,
                workspace_bytes, stream):
    rc = lib().ss_attn_bwd(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(bias), _ptr(region_ids), _ptr(G),
                           _ptr(dY), _ptr(lse), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dBias), _ptr(dG),
                           _ptr(workspace), workspace_bytes, stream)
    if rc != SS_OK:
        raise SSAttnError(rc, "ss_attn_bwd")


def ss_attn_bwd_static(desc, Q, K, V, bias, region_ids, G, dY, lse, dQ, dK, dV, dBias, dG, stream):
    rc = lib().ss_attn_bwd_static(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(bias), _ptr(region_ids), _ptr(G),
                                  _ptr(dY), _ptr(lse), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dBias), _ptr(dG), stream)
    if rc != SS_OK:
        raise SSAttnError(rc, "ss_attn_bwd_static")


def ss_attn_kernel_family(desc: ss_attn_desc):
    r = lib().ss_attn_kernel_family(C.byref(desc))
    return None if r is None else r.decode()


def ss_attn_profile_enable(on: bool):
    lib().ss_attn_profile_enable(1 if on else 0)


def ss_attn_profile_read(kernel: int):
    """-> (total_ms, launches) of one kernel id since the last read."""
    ms, n = C.c_double(0), C.c_int64(0)
    rc = lib().ss_attn_profile_read(kernel, C.byref(ms), C.byref(n))
    if rc != SS_OK:
        raise SSAttnError(rc, "ss_attn_profile_read")
    return ms.value, n.value
