"""Host-side arithmetic model of the one-walk recompute + dQ kernel (head size 32, large shares),
checked against the fp64 oracle.

The kernel cannot form dS = P (dP - Delta) while it walks the keys, because Delta is known only
after the last key.  It accumulates A1 = sum_j bf16(p~ dP) K_j and A2 = sum_j bf16(p~) K_j over the
unnormalised probabilities p~ and combines them at the end: dQ = scale / l' (A1 - Delta' A2).  The
two terms cancel on peaked rows, so which mean is subtracted matters: the kernel takes
Delta' = sum_j bf16(p~ dP) / sum_j bf16(p~), the mean of the operands the products saw.  This file
models that arithmetic in numpy (bf16 rounding of the operands, everything else in fp64) and pins
  * that the formula reproduces the oracle's dQ to the accuracy of forming dS directly, and
  * that the mean of the unrounded values (Delta itself) would be several times worse on peaked rows,
so that a change of the kernel's reading of Delta' has a failing test on the CPU.
No GPU, no HIP library: the oracle and the seeded input generator only."""
import math

import numpy as np
import pytest

from oracle import attention as orc
from paper_2301_08984_amd.workloads import make_inputs, round_to_bf16


def _bf(x):
    return round_to_bf16(np.asarray(x, dtype=np.float32)).astype(np.float64)


def _model(Q, K, V, dO, bias, causal, scale):
    """dQ of one (row, head) three ways: dS rounded directly; the two-product formula with the mean of
    the rounded operands; the same with the exact Delta."""
    S = Q.shape[0]
    x = scale * Q @ K.T + (bias if bias is not None else 0.0)
    if causal:
        x = np.where(np.tril(np.ones((S, S), bool)), x, -np.inf)
    p = np.exp(x - x.max(1, keepdims=True))    # unnormalised, largest entry 1
    l = p.sum(1, keepdims=True)
    P = p / l
    dP = dO @ V.T
    delta = (P * dP).sum(1, keepdims=True)
    direct = scale * _bf(P * (dP - delta)) @ K
    pb, wb = _bf(p), _bf(p * dP)
    a1, a2 = wb @ K, pb @ K
    lp = pb.sum(1, keepdims=True)
    fused = scale * (a1 - (wb.sum(1, keepdims=True) / lp) * a2) / lp
    exact_mean = scale * (a1 - delta * a2) / l
    return direct, fused, exact_mean


def _case(S, D, bias, causal, peak, seed):
    inp = make_inputs(B=1, H=1, S=S, D=D, dtype="bf16", bias="dense" if bias else None,
                      mask="causal" if causal else None, seed=seed)
    inp["Q"] = _bf(inp["Q"] * peak).astype(np.float32)   # larger queries: peaked softmax rows
    sc = float(np.float32(1.0 / math.sqrt(D)))
    prob = orc.AttnProblem(inp["Q"], inp["K"], inp["V"], sc,
                           ("dense", inp["bias"].astype(np.float64)) if bias else None,
                           ("causal",) if causal else None, None)
    ref = orc.attn_backward(prob, inp["dY"].astype(np.float64))["dQ"][0, :, 0, :]
    f64 = lambda a: a[0, :, 0, :].astype(np.float64)
    got = _model(f64(inp["Q"]), f64(inp["K"]), f64(inp["V"]), f64(inp["dY"]),
                 inp["bias"][0].astype(np.float64) if bias else None, causal, sc)
    den = np.max(np.abs(ref))
    return [float(np.max(np.abs(g - ref)) / den) for g in got]


@pytest.mark.parametrize("S,D,bias,causal,peak", [(384, 32, True, False, 1.0), (384, 32, True, False, 4.0),
                                                    (200, 32, True, True, 4.0), (130, 32, False, False, 2.0)])
def test_two_product_formula_matches_the_oracle(S, D, bias, causal, peak):
    direct, fused, _ = _case(S, D, bias, causal, peak, seed=11)
    assert direct <= 6e-3 and fused <= 6e-3, (direct, fused)
    assert fused <= 2.0 * direct + 1e-3, (direct, fused)   # as accurate as dS formed directly


def test_mean_of_the_unrounded_values_is_worse_on_peaked_rows():
    ratios = []
    for seed in (11, 12, 13):
        _, fused, exact_mean = _case(384, 32, True, False, 4.0, seed=seed)
        ratios.append(exact_mean / fused)
    assert min(ratios) >= 1.5 and sum(ratios) / len(ratios) >= 2.0, ratios


def test_one_hot_row_cancels_exactly():
    """One key carries all the weight: dS = 0, and the two products cancel to the last bit because the
    mean is the very operand that entered A1."""
    rng = np.random.default_rng(5)
    D, S = 32, 64
    K = _bf(rng.standard_normal((S, D)))
    V = _bf(rng.standard_normal((S, D)))
    dO = _bf(rng.standard_normal((1, D)))
    p = np.zeros((1, S))
    p[0, 17] = 1.0
    dP = dO @ V.T
    pb, wb = _bf(p), _bf(p * dP)
    a1, a2 = wb @ K, pb @ K
    dmean = wb.sum(1, keepdims=True) / pb.sum(1, keepdims=True)
    assert np.array_equal(a1 - dmean * a2, np.zeros((1, D)))
    # ... and does not with the exact mean, which is not a bf16 number
    assert np.max(np.abs(a1 - dP[:, 17:18] * a2)) > 0
