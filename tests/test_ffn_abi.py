"""CPU checks of the feed-forward boundary: the library exports what include/ss_ffn.h declares, the
descriptor layout matches the header as a C compiler sees it, validation and the chunk plan."""
import os
import re
import subprocess

import pytest

from oracle import ffn as orc
from paper_2301_08984_amd import binding as ss
from paper_2301_08984_amd import ffn_binding as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ss_ffn.h")


def test_exports_match_header():
    text = open(HEADER).read()
    declared = set(re.findall(r"\b(ss_ffn_\w+)\s*\(", text))
    assert declared == set(fb.EXPORTS)
    L = fb.lib()
    for name in fb.EXPORTS:
        assert hasattr(L, name), name


def test_struct_layout_matches_c(tmp_path):
    import ctypes as C
    src = tmp_path / "layout.c"
    fields = [f for f, _ in fb.ss_ffn_desc._fields_]
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "ss_ffn.h"\nint main(void){\n'
                   + 'printf("%zu\\n", sizeof(ss_ffn_desc));\n'
                   + "".join(f'printf("%zu\\n", offsetof(ss_ffn_desc, {f}));\n' for f in fields) + "return 0;}\n")
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o",
                           str(exe)])
    out = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    assert out[0] == C.sizeof(fb.ss_ffn_desc)
    for f, off in zip(fields, out[1:]):
        assert getattr(fb.ss_ffn_desc, f).offset == off, f
    assert len(fb.KERNEL_NAMES) == 7


def test_validation_and_chunks():
    good = fb.make_desc(100, 64, 256, 0, 256, 4)
    assert fb.ss_ffn_workspace_bytes(good)[0] > 0
    bad = [(dict(T=0), ss.SS_ERR_BAD_SHAPE), (dict(dm=60), ss.SS_ERR_BAD_SHAPE), (dict(ld_x=32), ss.SS_ERR_BAD_SHAPE),
           (dict(lo=4), ss.SS_ERR_BAD_RANGE), (dict(hi=300), ss.SS_ERR_BAD_RANGE), (dict(lo=256), ss.SS_ERR_BAD_RANGE),
           (dict(k=0), ss.SS_ERR_BAD_K), (dict(k=17), ss.SS_ERR_BAD_K), (dict(dtype=ss.SS_F32), ss.SS_ERR_UNSUPPORTED),
           (dict(act=7), ss.SS_ERR_UNSUPPORTED), (dict(T=1, ld_x=1 << 22), ss.SS_ERR_UNSUPPORTED),
           (dict(T=1 << 20, ld_x=2048), ss.SS_ERR_UNSUPPORTED)]
    for change, code in bad:
        d = fb.make_desc(100, 64, 256, 0, 256, 4)
        for f, v in change.items():
            setattr(d, f, v)
        with pytest.raises(ss.SSAttnError) as e:
            fb.ss_ffn_workspace_bytes(d)
        assert e.value.code == code, change
    for lo, hi, k in ((0, 256, 4), (16, 200, 3), (0, 40, 3), (8, 248, 5)):
        d = fb.make_desc(10, 64, 256, lo, hi, k)
        # the library promises boundaries at multiples of 16 columns from lo (include/ss_ffn.h)
        assert [fb.ss_ffn_chunk_range(d, c) for c in range(k)] == orc.chunk_ranges(lo, hi, k, unit=16)
    # the workspace is one chunk's hidden activations and shrinks as 1/k; the fp32 accumulator appears only
    # when sums that are bit-identical for every k are asked for
    T, dm, dh = 2048, 512, 4096
    f1, b1 = fb.ss_ffn_workspace_bytes(fb.make_desc(T, dm, dh, 0, dh, 1))
    f4, b4 = fb.ss_ffn_workspace_bytes(fb.make_desc(T, dm, dh, 0, dh, 4))
    assert f1 == T * dh * 2 and b1 == 2 * T * dh * 2
    assert f4 == T * (dh // 4) * 2 and b4 == 2 * T * (dh // 4) * 2
    x = fb.SS_FFN_FLAG_EXACT_SUM
    assert fb.ss_ffn_workspace_bytes(fb.make_desc(T, dm, dh, 0, dh, 1, flags=x)) == (f1, b1)
    assert fb.ss_ffn_workspace_bytes(fb.make_desc(T, dm, dh, 0, dh, 4, flags=x)) == (f4 + T * dm * 4, b4 + T * dm * 4)
    with pytest.raises(ss.SSAttnError) as e:
        fb.ss_ffn_workspace_bytes(fb.make_desc(T, dm, dh, 0, dh, 4, flags=2))
    assert e.value.code == ss.SS_ERR_UNSUPPORTED
    # the GPT-3 share of the benchmark: peak memory must fall with k (Sections 2 and 6.3)
    from paper_2301_08984_amd.workloads import FFN_WORKLOADS
    w = FFN_WORKLOADS["gpt3_ffn"]
    sizes = [fb.ss_ffn_workspace_bytes(fb.make_desc(w["T"], w["dm"], w["dh"], w["lo"], w["hi"], k)) for k in w["k"]]
    assert all(a[0] > b[0] and a[1] > b[1] for a, b in zip(sizes, sizes[1:])), sizes
    assert sizes[-1][1] * w["k"][-1] == sizes[0][1] * w["k"][0], sizes
    # null pointers and workspace errors are reported before anything is launched
    d = fb.make_desc(16, 64, 64, 0, 64, 1)
    with pytest.raises(ss.SSAttnError) as e:
        fb.ss_ffn_fwd(d, None, 1, 1, 1, None, 1, 256, 1 << 20, None)
    assert e.value.code == ss.SS_ERR_NULL
    with pytest.raises(ss.SSAttnError) as e:
        fb.ss_ffn_fwd(d, 256, 256, 256, 256, None, 256, 256, 16, None)
    assert e.value.code == ss.SS_ERR_WORKSPACE
