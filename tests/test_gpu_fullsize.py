"""Parity at the full workload sizes, in the launch configurations bench.py times: the same
shapes and EVERY co-shard factor a workload names.  Where the fp64 oracle finishes in under a
minute it checks every output; for the triangle shapes it checks sampled rows (rows are
independent) and the bias gradient on sampled query lines; for the long sequence one whole head.
The oracle's values do not depend on k, so they are computed once per workload.  Every k after the
first is also compared bit for bit with the first (the co-shard invariant of Section 3.1 at full
size; needs no oracle).  Both error metrics of parity.py apply; error scales always come from the
oracle's values."""
import numpy as np
import pytest

from oracle import attention as orc
from paper_2301_08984_amd import binding as ss
from paper_2301_08984_amd.runner import DeviceCase
from paper_2301_08984_amd.workloads import WORKLOADS, make_inputs

from parity import AXIS, TOL, assert_close, oracle_problem

pytestmark = pytest.mark.gpu

_INPUTS, _ORACLE, _FIRST = {}, {}, {}
OUTS = ("Y", "lse", "dQ", "dK", "dV", "dG", "dBias")


def _inputs(name):
    if name not in _INPUTS:
        _INPUTS.clear()   # one workload's host tensors at a time
        _INPUTS[name] = make_inputs(**WORKLOADS[name])
    return _INPUTS[name]


def _run(name, k):
    import torch
    w = dict(WORKLOADS[name])
    inp = _inputs(name)
    dc = DeviceCase(inp, dtype=w["dtype"], bias=w["bias"], mask=w["mask"], gated=w["gated"], win=w.get("win"),
                    layout=w.get("layout", "bshd"))
    ext = w["H"] if w["axis"] == "head" else w["B"]
    d = dc.desc(w["axis"], 0, ext, k)
    assert ss.ss_attn_kernel_family(d) != "plain_fp32"
    dc.fwd(d)
    dc.bwd(d, poison=True)
    torch.cuda.synchronize()
    return w, inp, dc


def _bitwise_vs_first(name, k, dc):
    """Device-side comparison with the first k of this workload run in this process."""
    import torch
    outs = {n: getattr(dc, n) for n in OUTS if getattr(dc, n) is not None}
    if name not in _FIRST:
        _FIRST.clear()
        _FIRST[name] = (k, {n: t.clone() for n, t in outs.items()})
        return
    k0, first = _FIRST[name]
    for n, t in outs.items():
        assert torch.equal(t, first[n]), (name, n, f"k={k} differs from k={k0}")
        assert bool(t.isfinite().all()), (name, n)


def _cases(names):
    return [(n, k) for n in names for k in WORKLOADS[n]["k"]]


@pytest.mark.parametrize("name,k", _cases(["gpt3_shard", "af2_msa_row", "swin_window", "af2_msa_col"]))
def test_full_workload_every_output(name, k):
    print(f"full-size {name} k={k}", flush=True)
    w, inp, dc = _run(name, k)
    if name not in _ORACLE:
        _ORACLE.clear()
        p = oracle_problem(inp, w)
        Y, LSE = orc.attn_forward(p, AXIS[w["axis"]])
        g = orc.attn_backward(p, inp["dY"].astype(np.float64), AXIS[w["axis"]])
        _ORACLE[name] = (Y, LSE, g)
    Y, LSE, g = _ORACLE[name]
    tol = TOL[w["dtype"]]
    errs = {"Y": assert_close("Y", dc.host("Y"), Y, tol), "lse": float(np.max(np.abs(dc.host("lse") - LSE)))}
    for n in ("dQ", "dK", "dV") + (("dG",) if w["gated"] else ()) + (("dBias",) if w["bias"] else ()):
        errs[n] = assert_close(n, dc.host(n), g[n], tol)
    print(name, k, {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
    assert errs["lse"] <= 1e-3
    _bitwise_vs_first(name, k, dc)


@pytest.mark.parametrize("k", WORKLOADS["gpt3_long"]["k"])
def test_long_sequence_one_head_against_oracle(k):
    """S = 12288 (the long-document setting): the kernels chosen for a chip-filling share.  The oracle
    computes one whole head (heads are independent): head 6, the first of a chunk for k = 2 and k = 4."""
    name, h = "gpt3_long", 6
    print(f"full-size {name} k={k}, head {h} against the oracle", flush=True)
    w, inp, dc = _run(name, k)
    if name not in _ORACLE:
        _ORACLE.clear()
        one = {n: np.ascontiguousarray(inp[n][:, :, h:h + 1]) for n in ("Q", "K", "V", "dY")}
        p = oracle_problem(one, w)
        Y, LSE = orc.attn_forward(p, orc.AXIS_HEAD)
        g = orc.attn_backward(p, one["dY"].astype(np.float64), orc.AXIS_HEAD)
        _ORACLE[name] = (Y, LSE, g)
    Y, LSE, g = _ORACLE[name]
    tol = TOL["bf16"]
    errs = {"Y": assert_close("Y", dc.host("Y")[:, :, h:h + 1], Y, tol),
            "lse": float(np.max(np.abs(dc.host("lse")[:, h:h + 1] - LSE)))}
    for n in ("dQ", "dK", "dV"):
        errs[n] = assert_close(n, dc.host(n)[:, :, h:h + 1], g[n], tol)
    print(name, k, {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
    assert errs["lse"] <= 1e-3
    _bitwise_vs_first(name, k, dc)


def test_longest_sequence_one_head_against_oracle():
    """S = 16384, the upper end of the long-document range, at k = 2: head 6 (the first of the second
    chunk) against the oracle, every output finite."""
    name, k, h = "gpt3_long_16k", 2, 6
    print(f"full-size {name} k={k}, head {h} against the oracle", flush=True)
    w, inp, dc = _run(name, k)
    _ORACLE.clear()
    one = {n: np.ascontiguousarray(inp[n][:, :, h:h + 1]) for n in ("Q", "K", "V", "dY")}
    p = oracle_problem(one, w)
    Y, LSE = orc.attn_forward(p, orc.AXIS_HEAD)
    g = orc.attn_backward(p, one["dY"].astype(np.float64), orc.AXIS_HEAD)
    tol = TOL["bf16"]
    errs = {"Y": assert_close("Y", dc.host("Y")[:, :, h:h + 1], Y, tol),
            "lse": float(np.max(np.abs(dc.host("lse")[:, h:h + 1] - LSE)))}
    for n in ("dQ", "dK", "dV"):
        errs[n] = assert_close(n, dc.host(n)[:, :, h:h + 1], g[n], tol)
    print(name, k, {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
    assert errs["lse"] <= 1e-3
    for n in ("Y", "dQ", "dK", "dV"):
        assert bool(getattr(dc, n).isfinite().all()), n


TRI_LINES = ((0, [0, 517]), (3, [1023, 64]))


@pytest.mark.parametrize("name,k", _cases(["af2_triangle", "af2_triangle_end"]))
def test_triangle_full_size_sampled(name, k):
    print(f"full-size {name} k={k} (sampled rows)", flush=True)
    w, inp, dc = _run(name, k)
    tol = TOL["bf16"]
    if name not in _ORACLE:
        _ORACLE.clear()
        p = oracle_problem(inp, w)
        dY = inp["dY"].astype(np.float64)
        rng = np.random.default_rng(0)
        # random rows plus both sides of chunk boundaries of k = 4, 16, 64
        rows = sorted(set(rng.integers(0, w["B"], size=4).tolist()) | {0, 15, 16, 255, 256, w["B"] - 1})
        per_row = {}
        for b in rows:
            Y, LSE = orc.attn_forward(p, orc.AXIS_ROW, b, b + 1)
            g = orc.attn_backward(p, dY, orc.AXIS_ROW, b, b + 1)
            per_row[b] = (Y[b], LSE[b], {n: g[n][b] for n in ("dQ", "dK", "dV", "dG")})
        lines = {h: orc.bias_grad_rows(p, dY, h, qs) for h, qs in TRI_LINES}   # sums over ALL rows
        _ORACLE[name] = (per_row, lines)
    per_row, lines = _ORACLE[name]
    for b, (Y, LSE, g) in per_row.items():
        got = {n: getattr(dc, n)[b].float().cpu().numpy().astype(np.float64) for n in ("Y", "dQ", "dK", "dV", "dG")}
        assert_close(f"Y[{b}]", got["Y"], Y, tol)
        for n in ("dQ", "dK", "dV", "dG"):
            assert_close(f"{n}[{b}]", got[n], g[n], tol)
        assert np.max(np.abs(dc.lse[b].cpu().numpy() - LSE)) <= 1e-3
    for h, qs in TRI_LINES:
        assert_close(f"dBias[{h}][{qs}]", dc.dBias[h][qs].cpu().numpy().astype(np.float64), lines[h], tol)
    _bitwise_vs_first(name, k, dc)
