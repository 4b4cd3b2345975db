"""Host-side checks of the C ABI that need no GPU: the library loads, exports what
include/ss_attn.h declares, the descriptor layout matches the header as a C compiler
sees it, validation returns the documented codes, and the chunk plan and workspace
sizes behave as the co-shard plan requires (Section 2; Section 4 uniform partition)."""
import ctypes as C
import os
import re
import subprocess

import pytest

from oracle import attention as orc
from paper_2301_08984_amd import binding as ss

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ss_attn.h")


def _desc(**kw):
    base = dict(B=4, H=8, S=64, D=32, dtype=ss.SS_BF16, scale=0.25, axis=ss.SS_AXIS_HEAD, lo=0, hi=8, k=2)
    base.update(kw)
    return ss.make_desc(**base)


def test_library_exports_every_declared_symbol():
    text = open(HEADER).read()
    declared = set(re.findall(r"\b(ss_[a-z_]+)\s*\(", text))
    assert declared == set(ss.EXPORTS)
    L = ss.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_descriptor_layout_matches_header(tmp_path):
    fields = " ".join(f'printf("%zu ", offsetof(ss_attn_desc, {n}));' for n, _ in ss.ss_attn_desc._fields_)
    src = tmp_path / "t.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "ss_attn.h"\n'
                   'int main(){ printf("%zu ", sizeof(ss_attn_desc)); ' + fields + ' return 0; }\n')
    exe = tmp_path / "t"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                           str(src), "-o", str(exe)])
    out = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    assert out[0] == C.sizeof(ss.ss_attn_desc)
    assert out[1:] == [getattr(ss.ss_attn_desc, n).offset for n, _ in ss.ss_attn_desc._fields_]


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), ss.SS_ERR_BAD_SHAPE),
    (dict(D=0), ss.SS_ERR_BAD_SHAPE),
    (dict(D=36), ss.SS_ERR_BAD_SHAPE),            # bf16 needs D % 8 == 0
    (dict(stride_h=16), ss.SS_ERR_BAD_SHAPE),     # stride shorter than a row
    (dict(dtype=7), ss.SS_ERR_UNSUPPORTED),
    (dict(D=512), ss.SS_ERR_UNSUPPORTED),
    (dict(lo=3, hi=3), ss.SS_ERR_BAD_RANGE),
    (dict(lo=-1), ss.SS_ERR_BAD_RANGE),
    (dict(hi=9), ss.SS_ERR_BAD_RANGE),
    (dict(axis=ss.SS_AXIS_ROW, hi=5), ss.SS_ERR_BAD_RANGE),
    (dict(k=0), ss.SS_ERR_BAD_K),
    (dict(k=9), ss.SS_ERR_BAD_K),
    (dict(lo=2, hi=5, k=4), ss.SS_ERR_BAD_K),
    (dict(bias_kind=ss.SS_BIAS_RELPOS, win=(7, 7)), ss.SS_ERR_BAD_SHAPE),   # S != 49
    (dict(mask_kind=ss.SS_MASK_REGION, mask_period=0), ss.SS_ERR_BAD_SHAPE),
    (dict(mask_kind=5), ss.SS_ERR_UNSUPPORTED),
    (dict(flags=1 << 9), ss.SS_ERR_UNSUPPORTED),
])
def test_validation_codes(kw, code):
    with pytest.raises(ss.SSAttnError) as e:
        ss.ss_attn_workspace_bytes(_desc(**kw))
    assert e.value.code == code


def test_null_and_workspace_errors_enqueue_nothing():
    d = _desc()
    L = ss.lib()
    # validation runs before any HIP call, so these return without touching a device
    assert L.ss_attn_fwd(C.byref(d), None, None, None, None, None, None, None, None, None, 0, None) == ss.SS_ERR_NULL
    one = 256  # a non-NULL, aligned fake address; never dereferenced because validation fails first
    assert L.ss_attn_bwd(C.byref(d), one, one, one, None, None, None, one, None, one, one, one, None, None,
                         None, 0, None) == ss.SS_ERR_WORKSPACE
    _, need = ss.ss_attn_workspace_bytes(d)
    assert L.ss_attn_bwd(C.byref(d), one, one, one, None, None, None, one, None, one, one, one, None, None,
                         one, need - 1, None) == ss.SS_ERR_WORKSPACE
    assert L.ss_attn_bwd(C.byref(d), one, one, one, None, None, None, one, None, one, one, one, None, None,
                         one + 8, need, None) == ss.SS_ERR_WORKSPACE
    g = _desc(gated=True)
    assert L.ss_attn_fwd(C.byref(g), one, one, one, None, None, None, one, None, None, 0, None) == ss.SS_ERR_NULL
    assert L.ss_attn_workspace_bytes(None, None, None) == ss.SS_ERR_NULL
    for code in range(-9, 1):
        assert ss.ss_strerror(code)


def test_share_beyond_the_built_in_buffer_is_rejected():
    """Validation only: nothing is enqueued, no pointer is dereferenced."""
    d = ss.make_desc(1024, 4, 1024, 32, ss.SS_BF16, 0.17, ss.SS_AXIS_ROW, 0, 1024, 4, bias_kind=ss.SS_BIAS_DENSE,
                     gated=True)
    _, need = ss.ss_attn_workspace_bytes(d)
    assert need > ss.SS_ATTN_STATIC_SCRATCH_BYTES
    one = 256
    rc = ss.lib().ss_attn_bwd_static(C.byref(d), one, one, one, one, None, one, one, None, one, one, one, None, one, None)
    assert rc == ss.SS_ERR_STATIC_SCRATCH
    assert "built-in" in ss.ss_strerror(rc)


def test_chunk_ranges_match_the_plan_rule():
    for axis, ext in ((ss.SS_AXIS_HEAD, 8), (ss.SS_AXIS_ROW, 4)):
        for lo in range(ext):
            for hi in range(lo + 1, ext + 1):
                for k in range(1, hi - lo + 1):
                    d = _desc(axis=axis, lo=lo, hi=hi, k=k)
                    got = [ss.ss_attn_chunk_range(d, c) for c in range(k)]
                    assert got == orc.chunk_ranges(lo, hi, k)
    with pytest.raises(ss.SSAttnError):
        ss.ss_attn_chunk_range(_desc(k=2), 2)


def test_workspace_shrinks_with_k():
    """The per-chunk scratch (softmax statistics, pre-gated dO) is proportional to the largest
    chunk; what does not depend on k (a transposed bias copy) stays constant."""
    for kw in (dict(gated=True, bias_kind=ss.SS_BIAS_DENSE, axis=ss.SS_AXIS_ROW, B=64, hi=64, S=128),
               dict(axis=ss.SS_AXIS_HEAD, S=128)):
        sizes = []
        for k in (1, 2, 4, 8):
            f, b = ss.ss_attn_workspace_bytes(_desc(k=k, **kw))
            assert f == 0 and b % 256 == 0 and b > 0
            sizes.append(b)
        assert all(a > b for a, b in zip(sizes, sizes[1:])), sizes
        B, H, S, D = kw.get("B", 4), 8, 128, 32
        per_chunk_k1 = 2 * B * H * S * 4 + (B * S * H * D * 2 if kw.get("gated") else 0)
        assert sizes[0] - sizes[3] >= 0.8 * per_chunk_k1 * (1 - 1 / 8), sizes


def test_workspace_of_the_workloads_scales_down_with_k():
    """The bias-gradient partial sums are folded into the result as their row groups complete, so they
    too are chunk-sized: the backward workspace is a constant (a transposed bias copy, one slice of
    group partials) plus a part proportional to the chunk.  Checked on the workload shapes:
    workspace(k) <= constant + workspace(1) / k * 1.25."""
    from paper_2301_08984_amd.workloads import WORKLOADS
    const = {"af2_msa_row": 16 << 20, "af2_triangle": 12 << 20, "af2_msa_col": 0, "gpt3_shard": 0}
    for name, c in const.items():
        w = WORKLOADS[name]
        ext = w["H"] if w["axis"] == "head" else w["B"]
        sizes = {}
        for k in (1,) + tuple(w["k"]):
            d = ss.make_desc(w["B"], w["H"], w["S"], w["D"], ss.SS_BF16, 0.1,
                             ss.SS_AXIS_HEAD if w["axis"] == "head" else ss.SS_AXIS_ROW, 0, ext, k,
                             bias_kind={None: 0, "dense": 1, "relpos": 2}[w["bias"]], gated=w["gated"],
                             mask_kind={None: 0, "causal": 1, "region": 2}[w["mask"]])
            sizes[k] = ss.ss_attn_workspace_bytes(d)[1]
        for k, b in sizes.items():
            assert b <= c + 1.25 * sizes[1] / k + 4096, (name, k, sizes)


def test_kernel_family_selection():
    assert ss.ss_attn_kernel_family(_desc(S=128)) == "mfma_bf16"
    assert ss.ss_attn_kernel_family(_desc(S=64)) == "mfma_bf16_short"
    assert ss.ss_attn_kernel_family(_desc(S=64, gated=True)) == "mfma_bf16"
    assert ss.ss_attn_kernel_family(_desc(D=128)) == "mfma_bf16"
    assert ss.ss_attn_kernel_family(_desc(D=48)) == "plain_fp32"
    assert ss.ss_attn_kernel_family(_desc(dtype=ss.SS_F32)) == "plain_fp32"
    assert ss.ss_attn_kernel_family(_desc(flags=ss.SS_FLAG_GENERIC_KERNELS)) == "plain_fp32"
    assert ss.ss_attn_kernel_family(_desc(k=0)) is None
    # the five workloads: only the fp32 one is served by the plain kernels
    from paper_2301_08984_amd.workloads import WORKLOADS
    for name, w in WORKLOADS.items():
        d = ss.make_desc(w["B"], w["H"], w["S"], w["D"], ss.SS_BF16 if w["dtype"] == "bf16" else ss.SS_F32, 0.1,
                         ss.SS_AXIS_HEAD if w["axis"] == "head" else ss.SS_AXIS_ROW, 0,
                         w["H"] if w["axis"] == "head" else w["B"], w["k"][0],
                         bias_kind={None: 0, "dense": 1, "relpos": 2}[w["bias"]], win=w.get("win", (0, 0)),
                         mask_kind={None: 0, "causal": 1, "region": 2}[w["mask"]], mask_period=256,
                         gated=w["gated"])
        want = "plain_fp32" if w["dtype"] == "f32" else ("mfma_bf16_short" if w["S"] <= 64 else "mfma_bf16")
        assert ss.ss_attn_kernel_family(d) == want, name
