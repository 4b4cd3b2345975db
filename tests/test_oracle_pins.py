"""Pins for the fp64 oracle: every check here compares oracle/attention.py with
something that is not itself -- a brute-force formulation written differently
(explicit loops, softmax without max shift, explicit softmax Jacobian), central
finite differences, closed forms, a library attention routine with library
autograd, and the co-shard invariant (Section 3.1: op-trans yields functionally
equivalent sub-operators; Section 5: gradients of shared inputs are value-split).
The paper prints no worked numeric example of attention, so there is no
paper-printed golden value for this path."""
import itertools
import math

import numpy as np
import pytest

from oracle import attention as orc


def _problem(rng, B=2, H=2, S=6, D=3, bias=None, mask=None, gated=False, win=None, scale=None):
    Q, K, V, dY = (rng.standard_normal((B, S, H, D)) for _ in range(4))
    G = rng.standard_normal((B, S, H, D)) if gated else None
    b = None
    if bias == "dense":
        b = ("dense", rng.standard_normal((H, S, S)))
    elif bias == "relpos":
        wh, ww = win
        b = ("relpos", rng.standard_normal((H, (2 * wh - 1) * (2 * ww - 1))), wh, ww)
    m = None
    if mask == "causal":
        m = ("causal",)
    elif mask == "region":
        ids = rng.integers(0, 2, size=(3, S))
        m = ("region", ids)
    p = orc.AttnProblem(Q, K, V, (1.0 / math.sqrt(D)) if scale is None else scale, b, m, G)
    return p, dY


CASES = [
    dict(),
    dict(mask="causal"),
    dict(bias="dense", gated=True),
    dict(bias="relpos", win=(2, 3), mask="region"),
    dict(bias="dense", mask="causal", gated=True, scale=0.37),
]


# ---------------------------------------------------------------- brute force
def _brute(p, dY, b, h):
    """One (row, head) pair, scalar loops, no max shift, explicit Jacobian."""
    S, D = p.S, p.D
    s = [[0.0] * S for _ in range(S)]
    for i in range(S):
        yi = xi = None
        for j in range(S):
            acc = 0.0
            for d in range(D):
                acc += p.Q[b, i, h, d] * p.K[b, j, h, d]
            acc *= p.scale
            if p.bias is not None:
                if p.bias[0] == "dense":
                    acc += p.bias[1][h][i][j]
                else:
                    wh, ww = p.bias[2], p.bias[3]
                    dy = i // ww - j // ww
                    dx = i % ww - j % ww
                    acc += p.bias[1][h][(dy + wh - 1) * (2 * ww - 1) + dx + ww - 1]
            s[i][j] = acc
    keep = [[True] * S for _ in range(S)]
    if p.mask is not None:
        for i in range(S):
            for j in range(S):
                if p.mask[0] == "causal":
                    keep[i][j] = j <= i
                else:
                    ids = p.mask[1]
                    keep[i][j] = ids[b % len(ids)][i] == ids[b % len(ids)][j]
    P = np.zeros((S, S))
    lse = np.zeros(S)
    for i in range(S):
        z = sum(math.exp(s[i][j]) for j in range(S) if keep[i][j])
        lse[i] = math.log(z)
        for j in range(S):
            P[i, j] = math.exp(s[i][j]) / z if keep[i][j] else 0.0
    V = p.V[b, :, h, :]
    O = np.zeros((S, D))
    for i in range(S):
        for j in range(S):
            O[i] += P[i, j] * V[j]
    g = np.ones((S, D)) if p.G is None else 1.0 / (1.0 + np.exp(-p.G[b, :, h, :]))
    Y = g * O
    dYm = dY[b, :, h, :]
    dG = dYm * O * g * (1 - g)
    dO = dYm * g
    dS = np.zeros((S, S))
    for i in range(S):
        J = np.diag(P[i]) - np.outer(P[i], P[i])  # d softmax / d logits of row i
        dPi = np.array([sum(dO[i, d] * V[j, d] for d in range(D)) for j in range(S)])
        dS[i] = J @ dPi
    dQ = np.zeros((S, D)); dK = np.zeros((S, D)); dV = np.zeros((S, D))
    for i in range(S):
        for j in range(S):
            dQ[i] += p.scale * dS[i, j] * p.K[b, j, h, :]
            dK[j] += p.scale * dS[i, j] * p.Q[b, i, h, :]
            dV[j] += P[i, j] * dO[i]
    return Y, lse, dQ, dK, dV, dG, dS, P


@pytest.mark.parametrize("case", CASES)
def test_brute_force_tiny(case):
    rng = np.random.default_rng(11)
    p, dY = _problem(rng, **case)
    Y, LSE = orc.attn_forward(p)
    g = orc.attn_backward(p, dY)
    dB = None if p.bias is None else np.zeros_like(np.asarray(p.bias[1]))
    for b, h in itertools.product(range(p.B), range(p.H)):
        bY, blse, bdQ, bdK, bdV, bdG, bdS, bP = _brute(p, dY, b, h)
        np.testing.assert_allclose(Y[b, :, h, :], bY, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(LSE[b, h], blse, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(g["dQ"][b, :, h, :], bdQ, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(g["dK"][b, :, h, :], bdK, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(g["dV"][b, :, h, :], bdV, rtol=1e-10, atol=1e-12)
        if p.G is not None:
            np.testing.assert_allclose(g["dG"][b, :, h, :], bdG, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(bP.sum(axis=1), 1.0, rtol=1e-12)
        if dB is not None:
            if p.bias[0] == "dense":
                dB[h] += bdS
            else:
                wh, ww = p.bias[2], p.bias[3]
                for i in range(p.S):
                    for j in range(p.S):
                        r = (i // ww - j // ww + wh - 1) * (2 * ww - 1) + (i % ww - j % ww + ww - 1)
                        dB[h, r] += bdS[i, j]
    if dB is not None:
        np.testing.assert_allclose(g["dBias"], dB, rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------- finite differences
def _loss(p, dY):
    Y, _ = orc.attn_forward(p)
    return float(np.sum(Y * dY))


@pytest.mark.parametrize("case", CASES)
def test_central_finite_differences(case):
    rng = np.random.default_rng(5)
    p, dY = _problem(rng, B=2, H=2, S=6, D=3, **case)
    g = orc.attn_backward(p, dY)
    eps = 1e-5
    targets = [("Q", p.Q, g["dQ"]), ("K", p.K, g["dK"]), ("V", p.V, g["dV"])]
    if p.G is not None:
        targets.append(("G", p.G, g["dG"]))
    if p.bias is not None:
        targets.append(("bias", p.bias[1], g["dBias"]))
    for name, arr, grad in targets:
        flat = arr.reshape(-1)
        gflat = grad.reshape(-1)
        pick = rng.choice(flat.size, size=min(flat.size, 40), replace=False)
        for t in pick:
            old = flat[t]
            flat[t] = old + eps
            up = _loss(p, dY)
            flat[t] = old - eps
            dn = _loss(p, dY)
            flat[t] = old
            fd = (up - dn) / (2 * eps)
            assert abs(fd - gflat[t]) <= 2e-7 * max(1.0, abs(fd)), (name, t, fd, gflat[t])


# ------------------------------------------------------------ library routine
@pytest.mark.parametrize("case", CASES)
def test_library_attention_and_autograd(case):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(23)
    p, dY = _problem(rng, B=2, H=3, S=8 if case.get("bias") != "relpos" else 6, D=4, **case)
    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    Q, K, V = t(p.Q), t(p.K), t(p.V)
    leaves = [Q, K, V]
    add = torch.zeros(p.B, p.H, p.S, p.S, dtype=torch.float64)
    bias_leaf = None
    if p.bias is not None:
        bias_leaf = t(np.asarray(p.bias[1]))
        leaves.append(bias_leaf)
        if p.bias[0] == "dense":
            add = add + bias_leaf[None]
        else:
            idx = torch.tensor(orc.relpos_index(p.bias[2], p.bias[3]))
            add = add + bias_leaf[:, idx][None]
    for b in range(p.B):
        M = p.masked(b)
        if M is not None:
            add[b] = add[b] + torch.tensor(np.where(M, -np.inf, 0.0))[None]
    O = torch.nn.functional.scaled_dot_product_attention(
        Q.permute(0, 2, 1, 3), K.permute(0, 2, 1, 3), V.permute(0, 2, 1, 3), attn_mask=add, scale=p.scale)
    Y = O.permute(0, 2, 1, 3)
    if p.G is not None:
        G = t(p.G)
        leaves.append(G)
        Y = torch.sigmoid(G) * Y
    Y.backward(torch.tensor(dY))
    Yo, _ = orc.attn_forward(p)
    g = orc.attn_backward(p, dY)
    np.testing.assert_allclose(Yo, Y.detach().numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dQ"], Q.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(g["dK"], K.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(g["dV"], V.grad.numpy(), rtol=1e-9, atol=1e-11)
    if p.G is not None:
        np.testing.assert_allclose(g["dG"], leaves[-1].grad.numpy(), rtol=1e-9, atol=1e-11)
    if bias_leaf is not None:
        np.testing.assert_allclose(g["dBias"], bias_leaf.grad.numpy(), rtol=1e-9, atol=1e-11)


# ---------------------------------------------------------------- closed forms
def test_lse_is_log_partition():
    rng = np.random.default_rng(2)
    p, _ = _problem(rng, bias="dense", mask="causal")
    _, LSE = orc.attn_forward(p)
    for b, h in itertools.product(range(p.B), range(p.H)):
        s = p.scale * p.Q[b, :, h] @ p.K[b, :, h].T + p.bias[1][h]
        for i in range(p.S):
            assert math.isclose(LSE[b, h, i], math.log(sum(math.exp(s[i, j]) for j in range(i + 1))), rel_tol=1e-12)


def test_zero_queries_give_mean_of_visible_values():
    rng = np.random.default_rng(3)
    p, _ = _problem(rng, mask="causal")
    p.Q[:] = 0.0
    Y, LSE = orc.attn_forward(p)
    for i in range(p.S):
        np.testing.assert_allclose(Y[:, i], p.V[:, : i + 1].mean(axis=1), rtol=1e-12)
        np.testing.assert_allclose(LSE[:, :, i], math.log(i + 1), rtol=1e-12, atol=1e-14)


def test_causal_first_row_copies_first_value_and_single_token():
    rng = np.random.default_rng(4)
    p, dY = _problem(rng, mask="causal")
    Y, _ = orc.attn_forward(p)
    np.testing.assert_allclose(Y[:, 0], p.V[:, 0], rtol=1e-13)
    p1, dY1 = _problem(rng, S=1)
    Y1, _ = orc.attn_forward(p1)
    g1 = orc.attn_backward(p1, dY1)
    np.testing.assert_allclose(Y1, p1.V)
    np.testing.assert_allclose(g1["dV"], dY1)
    assert np.all(g1["dQ"] == 0) and np.all(g1["dK"] == 0)


def test_constant_values_give_zero_query_key_gradients():
    rng = np.random.default_rng(6)
    p, dY = _problem(rng, bias="dense")
    p.V[:] = rng.standard_normal((p.B, 1, p.H, p.D))
    Y, _ = orc.attn_forward(p)
    np.testing.assert_allclose(Y, np.broadcast_to(p.V[:, :1], Y.shape), rtol=1e-12)
    g = orc.attn_backward(p, dY)
    assert np.max(np.abs(g["dQ"])) < 1e-14 and np.max(np.abs(g["dK"])) < 1e-14
    assert np.max(np.abs(g["dBias"])) < 1e-14


def test_row_constant_in_bias_changes_nothing_and_dbias_rows_sum_to_zero():
    rng = np.random.default_rng(7)
    p, dY = _problem(rng, bias="dense", gated=True)
    Y0, _ = orc.attn_forward(p)
    g0 = orc.attn_backward(p, dY)
    p.bias[1][:] += rng.standard_normal((p.H, p.S, 1))
    Y1, _ = orc.attn_forward(p)
    g1 = orc.attn_backward(p, dY)
    np.testing.assert_allclose(Y1, Y0, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(g1["dQ"], g0["dQ"], rtol=1e-9, atol=1e-12)
    assert np.max(np.abs(g0["dBias"].sum(axis=2))) < 1e-13
    pr, dYr = _problem(rng, bias="relpos", win=(3, 2), mask="region")
    gr = orc.attn_backward(pr, dYr)
    assert np.max(np.abs(gr["dBias"].sum(axis=1))) < 1e-13


def test_key_permutation_permutes_dk_dv_only():
    rng = np.random.default_rng(8)
    p, dY = _problem(rng)
    perm = rng.permutation(p.S)
    q = orc.AttnProblem(p.Q, p.K[:, perm], p.V[:, perm], p.scale)
    Y0, _ = orc.attn_forward(p)
    Y1, _ = orc.attn_forward(q)
    np.testing.assert_allclose(Y1, Y0, rtol=1e-11, atol=1e-13)
    g0, g1 = orc.attn_backward(p, dY), orc.attn_backward(q, dY)
    np.testing.assert_allclose(g1["dQ"], g0["dQ"], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(g1["dK"], g0["dK"][:, perm], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(g1["dV"], g0["dV"][:, perm], rtol=1e-10, atol=1e-13)


def test_region_mask_equals_attention_within_each_region():
    rng = np.random.default_rng(9)
    p, dY = _problem(rng, B=3, S=8, mask="region")
    Y, _ = orc.attn_forward(p)
    g = orc.attn_backward(p, dY)
    ids = p.mask[1]
    for b in range(p.B):
        for r in np.unique(ids[b % len(ids)]):
            sel = np.nonzero(ids[b % len(ids)] == r)[0]
            sub = orc.AttnProblem(p.Q[b:b + 1, sel], p.K[b:b + 1, sel], p.V[b:b + 1, sel], p.scale)
            Ys, _ = orc.attn_forward(sub)
            gs = orc.attn_backward(sub, dY[b:b + 1, sel])
            np.testing.assert_allclose(Y[b, sel], Ys[0], rtol=1e-11, atol=1e-13)
            np.testing.assert_allclose(g["dK"][b, sel], gs["dK"][0], rtol=1e-10, atol=1e-13)


def test_relpos_table_equals_gathered_dense_bias():
    rng = np.random.default_rng(10)
    p, dY = _problem(rng, S=6, bias="relpos", win=(2, 3))
    wh, ww = 2, 3
    dense = np.zeros((p.H, p.S, p.S))
    for i in range(p.S):
        for j in range(p.S):
            r = (i // ww - j // ww + wh - 1) * (2 * ww - 1) + (i % ww - j % ww + ww - 1)
            dense[:, i, j] = p.bias[1][:, r]
    q = orc.AttnProblem(p.Q, p.K, p.V, p.scale, ("dense", dense))
    np.testing.assert_allclose(orc.attn_forward(p)[0], orc.attn_forward(q)[0], rtol=1e-12)
    gp, gq = orc.attn_backward(p, dY), orc.attn_backward(q, dY)
    scat = np.zeros_like(p.bias[1])
    for i in range(p.S):
        for j in range(p.S):
            r = (i // ww - j // ww + wh - 1) * (2 * ww - 1) + (i % ww - j % ww + ww - 1)
            scat[:, r] += gq["dBias"][:, i, j]
    np.testing.assert_allclose(gp["dBias"], scat, rtol=1e-11, atol=1e-13)
    # 7x7 window: 169 entries, centre entry is the zero displacement
    idx = orc.relpos_index(7, 7)
    assert idx.min() == 0 and idx.max() == 168 and np.all(np.diag(idx) == 84)
    assert idx[0, 48] == 0 and idx[48, 0] == 168 and idx[0, 1] == 83 and idx[0, 7] == 84 - 13


# ------------------------------------------------------------- chunk invariant
def test_chunk_ranges():
    assert orc.chunk_ranges(0, 12, 4) == [(0, 3), (3, 6), (6, 9), (9, 12)]
    assert orc.chunk_ranges(2, 9, 3) == [(2, 4), (4, 6), (6, 9)]
    assert orc.chunk_ranges(5, 8, 3) == [(5, 6), (6, 7), (7, 8)]
    for lo, hi, k in [(0, 7, 2), (3, 20, 5), (0, 5, 5)]:
        r = orc.chunk_ranges(lo, hi, k)
        assert r[0][0] == lo and r[-1][1] == hi
        assert all(a[1] == b[0] for a, b in zip(r, r[1:]))
        sizes = [b - a for a, b in r]
        assert min(sizes) >= 1 and max(sizes) - min(sizes) <= 1
    with pytest.raises(ValueError):
        orc.chunk_ranges(0, 3, 4)
    with pytest.raises(ValueError):
        orc.chunk_ranges(0, 3, 0)


@pytest.mark.parametrize("axis,extent", [(orc.AXIS_HEAD, "H"), (orc.AXIS_ROW, "B")])
@pytest.mark.parametrize("case", [CASES[2], CASES[3]])
def test_coshard_equals_unsplit(axis, extent, case):
    rng = np.random.default_rng(12)
    p, dY = _problem(rng, B=5, H=5, S=6, D=3, **case)
    n = getattr(p, extent)
    for lo, hi in [(0, n), (1, n)]:
        Y0, L0 = orc.attn_forward(p, axis, lo, hi)
        g0 = orc.attn_backward(p, dY, axis, lo, hi)
        for k in (1, 2, 3, hi - lo):
            Y1, L1 = orc.coshard_forward(p, axis, lo, hi, k)
            g1 = orc.coshard_backward(p, dY, axis, lo, hi, k)
            assert np.array_equal(Y0, Y1) and np.array_equal(L0, L1)
            for name in g0:
                if name == "dBias":
                    np.testing.assert_allclose(g1[name], g0[name], rtol=1e-12, atol=1e-14)
                else:
                    assert np.array_equal(g0[name], g1[name]), name
    # outside the range nothing is produced
    Y, _ = orc.attn_forward(p, axis, 1, n)
    assert np.all((Y[:, :, 0] if axis == orc.AXIS_HEAD else Y[0]) == 0)


def test_planted_mistakes_are_caught():
    """The brute-force pin must fail for plausible slips; plant them in a copy."""
    rng = np.random.default_rng(13)
    p, dY = _problem(rng, bias="dense", mask="causal", gated=True)
    g = orc.attn_backward(p, dY)
    _, _, bdQ, bdK, bdV, bdG, bdS, _ = _brute(p, dY, 0, 0)
    wrong_transposed = p.scale * (bdS.T @ p.K[0, :, 0])     # dQ with dS transposed
    wrong_noscale = bdS @ p.K[0, :, 0]                      # dropped scale
    assert not np.allclose(g["dQ"][0, :, 0], wrong_transposed, rtol=1e-6)
    assert not np.allclose(g["dQ"][0, :, 0], wrong_noscale, rtol=1e-6)
    np.testing.assert_allclose(g["dQ"][0, :, 0], bdQ, rtol=1e-10, atol=1e-12)


def test_bias_grad_rows_equals_rows_of_full_gradient():
    rng = np.random.default_rng(14)
    for case in (dict(bias="dense", gated=True), dict(bias="dense", mask="causal")):
        p, dY = _problem(rng, B=4, H=2, S=7, D=3, **case)
        full = orc.attn_backward(p, dY, orc.AXIS_ROW, 1, 4)["dBias"]
        for h in range(p.H):
            got = orc.bias_grad_rows(p, dY, h, [0, 3, 6], 1, 4)
            np.testing.assert_allclose(got, full[h][[0, 3, 6]], rtol=1e-11, atol=1e-13)
