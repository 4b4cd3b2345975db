"""Shared helpers of the GPU parity tests: run one case through the C ABI and
through the fp64 oracle on the same seeded inputs, compare every output.

Two error metrics per output tensor, over the entries of the share:
  * max|x - ref| / max|ref| (relative to the tensor's largest magnitude; element-wise
    relative error is unbounded next to zeros).  Bars: 1e-4 for fp32 tensors, 2e-2 for
    bf16 tensors with fp32 accumulation, against the fp64 oracle;
  * element by element, |x - ref| <= tol * (|ref| + rms(ref)) with the same tol: an error
    confined to small entries passes the first metric and fails this one.  At least
    99.99 % of the entries must pass (`elem_fail` returns the fraction that does not): the
    rounding error of an output row scales with that row's own magnitude, and a few near-zero
    entries of the rows that are several times larger than the tensor's rms (the first
    queries of a causal sequence, which see few keys) exceed a bar taken from the whole
    tensor's rms; one wrong 32 x 32 tile in 3 M entries is 3e-4 and fails.
Every backward call runs on a workspace filled with 0xFF bytes (NaN in every float
format), so scratch that a kernel reads before writing it in the same call shows."""
import math

import numpy as np

from oracle import attention as orc
from paper_2301_08984_amd import binding as ss
from paper_2301_08984_amd.runner import DeviceCase
from paper_2301_08984_amd.workloads import make_inputs

TOL = {"f32": 1e-4, "bf16": 2e-2}
ELEM_FAIL_MAX = 1e-4   # fraction of entries that may miss the element-wise bar
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


def elem_fail(x, ref, tol):
    """Fraction of entries with |x - ref| > tol * (|ref| + rms(ref))."""
    x, ref = np.asarray(x, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:   # an identically zero reference (a one-token sequence has dQ = dK = 0): absolute bar, as rel_err
        rms = 1.0
    bad = ~(np.abs(x - ref) <= tol * (np.abs(ref) + rms))   # NaN counts as a failure
    return float(np.count_nonzero(bad)) / ref.size


def assert_close(name, x, ref, tol):
    """Both metrics for one tensor; returns the max-norm relative error."""
    e = rel_err(x, ref)
    assert np.isfinite(e) and e <= tol, (name, e, tol)
    f = elem_fail(x, ref, tol)
    assert f <= ELEM_FAIL_MAX, (name, "element-wise failures", f)
    return e


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
    dc.bwd(d, use_lse=use_lse, poison=True)
    import torch
    torch.cuda.synchronize()
    return dc, inp


def check_against_oracle(cfg, lo=None, hi=None, k=1, flags=0, use_lse=False, scale=None, tol=None, inputs=None,
                         elem_fail_max=ELEM_FAIL_MAX):
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
    errs, fails = {}, {}
    pairs = [("Y", dc.host("Y")[act], Y[act])]
    errs["lse"] = float(np.max(np.abs(dc.host("lse")[lses] - LSE[lses])))
    for n in ("dQ", "dK", "dV") + (("dG",) if cfg.get("gated") else ()):
        pairs.append((n, dc.host(n)[act], g[n][act]))
    if cfg.get("bias"):
        got, ref = dc.host("dBias"), g["dBias"]
        if cfg["axis"] == "head":
            got, ref = got[lo:hi], ref[lo:hi]
        pairs.append(("dBias", got, ref))
    for n, got, ref in pairs:
        errs[n] = rel_err(got, ref)
        fails[n] = elem_fail(got, ref, tol)
    for n, e in errs.items():
        bar = tol if n != "lse" else max(tol, 1e-4) * 4
        assert np.isfinite(e) and e <= bar, (n, e, bar, errs)
    assert all(f <= elem_fail_max for f in fails.values()), ("element-wise failures", fails, errs)
    # nothing outside the share may be written (buffers start as NaN)
    for n in ("Y", "dQ", "dK", "dV") + (("dG",) if cfg.get("gated") else ()):
        full = dc.host(n)
        inside = np.zeros(full.shape, dtype=bool)
        inside[act] = True
        assert np.all(np.isnan(full[~inside])), n
        assert not np.any(np.isnan(full[inside])), n
    return dc, errs
