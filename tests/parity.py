"""Shared helpers of the GPU parity tests: run one case through the C ABI and
through the fp64 oracle on the same seeded inputs, compare every output.

Error metric per output tensor: max|x - ref| / max|ref| over the entries of the
share (relative to the tensor's largest magnitude; elementwise relative error is
unbounded next to zeros).  Bars: 1e-4 for fp32 tensors, 2e-2 for bf16 tensors
with fp32 accumulation, against the fp64 oracle."""
import math

import numpy as np

from oracle import attention as orc
from paper_2301_08984_amd import binding as ss
from paper_2301_08984_amd.runner import DeviceCase
from paper_2301_08984_amd.workloads import make_inputs

TOL = {"f32": 1e-4, "bf16": 2e-2}
AXIS = {"head": orc.AXIS_HEAD, "row": orc.AXIS_ROW}


def oracle_problem(inp, cfg, scale=None):
    bias = None
    if cfg.get("bias") == "dense":
        bias = ("dense", inp["bias"].astype(np.float64))
    elif cfg.get("bias") == "relpos":
        bias = ("relpos", inp["bias"].astype(np.float64), cfg["win"][0], cfg["win"][1])
    mask = None
    if cfg.get("mask") == "causal":
        mask = ("causal",)
    elif cfg.get("mask") == "region":
        mask = ("region", inp["region_ids"])
    D = inp["Q"].shape[-1]
    # the scale is rounded to fp32 exactly as the descriptor carries it
    sc = float(np.float32((1.0 / math.sqrt(D)) if scale is None else scale))
    return orc.AttnProblem(inp["Q"], inp["K"], inp["V"], sc, bias, mask, inp.get("G"))


def rel_err(x, ref):
    den = np.max(np.abs(ref))
    if den == 0:
        return float(np.max(np.abs(x)))
    return float(np.max(np.abs(x - ref)) / den)


def share_slices(axis, lo, hi):
    act = (slice(None), slice(None), slice(lo, hi)) if axis == "head" else (slice(lo, hi),)
    lse = (slice(None), slice(lo, hi)) if axis == "head" else (slice(lo, hi),)
    return act, lse


def run_case(cfg, lo=None, hi=None, k=1, flags=0, use_lse=False, inputs=None, scale=None):
    """Returns (DeviceCase after fwd+bwd, inputs)."""
    inp = make_inputs(**cfg) if inputs is None else inputs
    dc = DeviceCase(inp, dtype=cfg["dtype"], bias=cfg.get("bias"), mask=cfg.get("mask"),
                    gated=cfg.get("gated", False), win=cfg.get("win"), scale=scale,
                    layout=cfg.get("layout", "bshd"))
    ext = dc.H if cfg["axis"] == "head" else dc.B
    lo = 0 if lo is None else lo
    hi = ext if hi is None else hi
    d = dc.desc(cfg["axis"], lo, hi, k, flags)
    dc.fwd(d)
    dc.bwd(d, use_lse=use_lse)
    import torch
    torch.cuda.synchronize()
    return dc, inp


def check_against_oracle(cfg, lo=None, hi=None, k=1, flags=0, use_lse=False, scale=None, tol=None, inputs=None):
    dc, inp = run_case(cfg, lo, hi, k, flags, use_lse, inputs=inputs, scale=scale)
    ext = dc.H if cfg["axis"] == "head" else dc.B
    lo = 0 if lo is None else lo
    hi = ext if hi is None else hi
    p = oracle_problem(inp, cfg, scale)
    ax = AXIS[cfg["axis"]]
    Y, LSE = orc.attn_forward(p, ax, lo, hi)
    g = orc.attn_backward(p, inp["dY"].astype(np.float64), ax, lo, hi)
    tol = TOL[cfg["dtype"]] if tol is None else tol
    act, lses = share_slices(cfg["axis"], lo, hi)
    errs = {}
    errs["Y"] = rel_err(dc.host("Y")[act], Y[act])
    errs["lse"] = float(np.max(np.abs(dc.host("lse")[lses] - LSE[lses])))
    for n in ("dQ", "dK", "dV") + (("dG",) if cfg.get("gated") else ()):
        errs[n] = rel_err(dc.host(n)[act], g[n][act])
    if cfg.get("bias"):
        got, ref = dc.host("dBias"), g["dBias"]
        if cfg["axis"] == "head":
            got, ref = got[lo:hi], ref[lo:hi]
        errs["dBias"] = rel_err(got, ref)
    for n, e in errs.items():
        bar = tol if n != "lse" else max(tol, 1e-4) * 4
        assert np.isfinite(e) and e <= bar, (n, e, bar, errs)
    # nothing outside the share may be written (buffers start as NaN)
    for n in ("Y", "dQ", "dK", "dV") + (("dG",) if cfg.get("gated") else ()):
        full = dc.host(n)
        inside = np.zeros(full.shape, dtype=bool)
        inside[act] = True
        assert np.all(np.isnan(full[~inside])), n
        assert not np.any(np.isnan(full[inside])), n
    return dc, errs
