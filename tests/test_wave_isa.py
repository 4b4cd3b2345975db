"""Static checks on the generated code of the kernels that read LDS from hand-written assembly.

The small-share kernels at head size 128 issue their fragment reads (`ds_read_b128`,
`ds_read_b64_tr_b16`) in one assembly statement and wait for them in a later one, so that loads
that are under way into other LDS tiles are not waited for.  Between the two statements the
destination registers hold no data yet and the compiler does not know it: nothing may read, copy
or overwrite them there.  The same files rely on being compiled without any accumulation
register.  Both properties are checked here on the ISA the build's own flags produce (no GPU needed).
"""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2301_08984_amd import build as B

FILES = ["fast_wave_fwd128.hip", "fast_wave_bwd128.hip", "fast_fwd128.hip", "fast_dq128.hip", "fast_kv128.hip"]


def _regs(tok):
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", tok)
    return {int(m.group(1))} if m else set()


def pending_read_violations(lines):
    """Instructions that touch a register between the assembly-issued LDS read that targets it and
    the next `s_waitcnt lgkmcnt(0)`."""
    bad, pending, in_app = [], {}, False
    for ln, line in enumerate(lines, 1):
        if "#APP" in line:
            in_app = True
        if "#NO_APP" in line:
            in_app = False
        t = line.split(";")[0].strip()
        if not t or t.startswith(".") or t.endswith(":"):
            if t.endswith(":") and not t.startswith(".LBB"):
                pending = {}  # next function
            continue
        parts = t.replace(",", " ").split()
        op, toks = parts[0], parts[1:]
        if op == "s_waitcnt":
            if "lgkmcnt(0)" in t:
                pending = {}
            continue
        used = set()
        for tk in toks:
            used |= _regs(tk)
        if op.startswith("ds_read") and in_app:
            dst = _regs(toks[0])
            if (used - dst) & set(pending) or dst & set(pending):
                bad.append((ln, t))
            for r in dst:
                pending[r] = ln
            continue
        if used & set(pending):
            bad.append((ln, t))
    return bad


def test_checker_flags_a_planted_use():
    good = ["f:", "\t;#APP", "\tds_read_b128 v[4:7], v1", "\t;#NO_APP", "\tv_add_f32 v9, v8, v8",
            "\ts_waitcnt lgkmcnt(0)", "\tv_add_f32 v9, v4, v8"]
    assert pending_read_violations(good) == []
    bad = list(good)
    bad[4] = "\tv_mov_b32 v9, v5"  # reads v5 before the wait
    assert [ln for ln, _ in pending_read_violations(bad)] == [5]


@pytest.mark.parametrize("src", FILES)
def test_no_register_is_touched_between_an_assembly_read_and_its_wait(src):
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        cmd = ["hipcc", *B.FLAGS, *B.EXTRA_FLAGS.get(src, []), "--cuda-device-only", "-S",
               os.path.join(B.CSRC, src), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        lines = open(out).read().splitlines()
    assert any("ds_read_b64_tr_b16" in l for l in lines)
    assert pending_read_violations(lines) == []
    # compiled without accumulation registers: all 256 registers of a wavefront are vector registers
    assert not any("v_accvgpr" in l for l in lines), "accumulation registers in use"
    agpr = [l for l in lines if ".agpr_count" in l]
    assert agpr and all(l.split()[-1] == "0" for l in agpr), agpr
