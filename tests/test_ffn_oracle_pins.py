"""Pins of the feed-forward oracle (CPU): brute force, finite differences, a library
implementation with library autograd, closed forms, the chunk invariant, planted mistakes."""
import numpy as np
import pytest

from oracle import ffn as orc


def _problem(seed=0, T=5, dm=6, dh=40, kind=orc.ACT_GELU_TANH, b2=True):
    g = np.random.default_rng(seed)
    return orc.FfnProblem(g.standard_normal((T, dm)), g.standard_normal((dm, dh)) * 0.5, g.standard_normal(dh) * 0.3,
                          g.standard_normal((dh, dm)) * 0.5, g.standard_normal(dm) if b2 else None, kind), \
        g.standard_normal((T, dm))


def _brute_forward(p, lo, hi):
    import math
    Y = np.zeros((p.T, p.dm))
    for t in range(p.T):
        for j in range(lo, hi):
            z = p.b1[j]
            for i in range(p.dm):
                z += p.X[t, i] * p.W1[i, j]
            if p.kind == orc.ACT_RELU:
                h = z if z > 0 else 0.0
            else:
                h = 0.5 * z * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z * z * z)))
            for o in range(p.dm):
                Y[t, o] += h * p.W2[j, o]
    if p.b2 is not None:
        Y += p.b2
    return Y


@pytest.mark.parametrize("kind", [orc.ACT_RELU, orc.ACT_GELU_TANH])
def test_forward_matches_scalar_loops(kind):
    p, _ = _problem(1, kind=kind)
    assert np.allclose(orc.ffn_forward(p, 8, 33), _brute_forward(p, 8, 33), rtol=1e-12, atol=1e-12)
    assert np.allclose(orc.ffn_forward(p), _brute_forward(p, 0, p.dh), rtol=1e-12, atol=1e-12)


def test_gelu_matches_library_and_its_derivative_matches_differences():
    import torch
    z = np.linspace(-6, 6, 1201)
    ref = torch.nn.functional.gelu(torch.from_numpy(z), approximate="tanh").numpy()
    assert np.allclose(orc.act(z, orc.ACT_GELU_TANH), ref, rtol=1e-13, atol=1e-15)
    e = 1e-6
    num = (orc.act(z + e, orc.ACT_GELU_TANH) - orc.act(z - e, orc.ACT_GELU_TANH)) / (2 * e)
    assert np.allclose(orc.act_grad(z, orc.ACT_GELU_TANH), num, rtol=1e-7, atol=1e-8)
    assert abs(orc.act(np.array([1.0]), orc.ACT_GELU_TANH)[0] - 0.8411919906082768) < 1e-12  # textbook value


@pytest.mark.parametrize("kind", [orc.ACT_RELU, orc.ACT_GELU_TANH])
def test_backward_matches_finite_differences(kind):
    p, dY = _problem(2, kind=kind)
    lo, hi = 8, 32
    g = orc.ffn_backward(p, dY, lo, hi)
    loss = lambda q: float(np.sum(orc.ffn_forward(q, lo, hi) * dY))
    e = 1e-6
    rng = np.random.default_rng(5)
    for name, arr in (("dX", "X"), ("dW1", "W1"), ("db1", "b1"), ("dW2", "W2"), ("db2", "b2")):
        a = getattr(p, arr)
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in a.shape)
            if kind == orc.ACT_RELU:  # stay away from the kink
                Z = p.X @ p.W1 + p.b1
                if np.min(np.abs(Z)) < 1e-3:
                    continue
            old = a[idx]
            a[idx] = old + e; up = loss(p)
            a[idx] = old - e; dn = loss(p)
            a[idx] = old
            assert abs((up - dn) / (2 * e) - g[name][idx]) < 1e-6, (name, idx)
    # outside the share the weight gradients are exactly zero
    assert not g["dW1"][:, :lo].any() and not g["dW1"][:, hi:].any() and not g["dW2"][:lo].any()


def test_matches_library_autograd():
    import torch
    p, dY = _problem(3, T=7, dm=8, dh=48)
    t = {n: torch.tensor(getattr(p, n), requires_grad=True) for n in ("X", "W1", "b1", "W2", "b2")}
    Y = torch.nn.functional.gelu(t["X"] @ t["W1"] + t["b1"], approximate="tanh") @ t["W2"] + t["b2"]
    Y.backward(torch.tensor(dY))
    assert np.allclose(orc.ffn_forward(p), Y.detach().numpy(), rtol=1e-12, atol=1e-12)
    g = orc.ffn_backward(p, dY)
    for n, a in (("dX", "X"), ("dW1", "W1"), ("db1", "b1"), ("dW2", "W2"), ("db2", "b2")):
        assert np.allclose(g[n], t[a].grad.numpy(), rtol=1e-11, atol=1e-12), n


def test_closed_forms():
    # ReLU with all pre-activations positive is one affine map; with all negative the output is b2
    g = np.random.default_rng(4)
    X = np.abs(g.standard_normal((4, 5))); W1 = np.abs(g.standard_normal((5, 32))); b1 = np.ones(32)
    W2 = g.standard_normal((32, 5)); b2 = g.standard_normal(5)
    p = orc.FfnProblem(X, W1, b1, W2, b2, orc.ACT_RELU)
    assert np.allclose(orc.ffn_forward(p), (X @ W1 + b1) @ W2 + b2)
    q = orc.FfnProblem(X, -W1, -b1, W2, b2, orc.ACT_RELU)
    assert np.allclose(orc.ffn_forward(q), np.broadcast_to(b2, (4, 5)))
    gq = orc.ffn_backward(q, np.ones((4, 5)))
    assert not gq["dX"].any() and not gq["dW1"].any() and not gq["dW2"].any() and np.allclose(gq["db2"], 4.0)


def test_chunk_ranges_and_invariant():
    # literal values: the plain balanced split, and the same split in whole units of 16 columns
    assert orc.chunk_ranges(0, 10, 3) == [(0, 3), (3, 6), (6, 10)]
    assert orc.chunk_ranges(5, 9, 4) == [(5, 6), (6, 7), (7, 8), (8, 9)]
    assert orc.chunk_ranges(0, 40, 3, unit=16) == [(0, 16), (16, 32), (32, 40)]
    assert orc.chunk_ranges(16, 200, 3, unit=16) == [(16, 80), (80, 144), (144, 200)]
    for unit in (1, 16):
        for lo, hi, k in ((0, 64, 4), (16, 200, 3), (0, 40, 7), (32, 48, 2), (0, 16, 3)):
            r = orc.chunk_ranges(lo, hi, k, unit)
            assert len(r) == k and r[0][0] == lo and r[-1][1] == hi
            assert all(a <= b for a, b in r) and all(r[i][1] == r[i + 1][0] for i in range(k - 1))
            assert all((a - lo) % unit == 0 for a, _ in r)
            sizes = [b - a for a, b in r]
            assert max(sizes) - min(sizes) <= unit + (unit - (hi - lo) % unit) % unit
    p, dY = _problem(6, T=6, dm=8, dh=112)
    for lo, hi in ((0, 112), (16, 100)):
        Y1 = orc.coshard_forward(p, lo, hi, 1)
        assert np.allclose(Y1, orc.ffn_forward(p, lo, hi))
        g1 = orc.coshard_backward(p, dY, lo, hi, 1)
        for k, unit in ((2, 1), (3, 1), (5, 1), (3, 16), (5, 16)):
            assert np.allclose(orc.coshard_forward(p, lo, hi, k, unit), Y1, rtol=1e-12, atol=1e-12)
            gk = orc.coshard_backward(p, dY, lo, hi, k, unit)
            for n in g1:
                assert np.allclose(gk[n], g1[n], rtol=1e-12, atol=1e-12), (n, k)


def test_planted_mistakes_are_caught():
    """Each plausible slip changes a result that one of the pins above fixes."""
    p, dY = _problem(7)
    g = orc.ffn_backward(p, dY)
    Z = p.X @ p.W1 + p.b1
    H = orc.act(Z, p.kind)
    dH = dY @ p.W2.T
    wrong = {
        "dW2 from the pre-activations instead of the activations": not np.allclose(Z.T @ dY, g["dW2"]),
        "dZ without the activation derivative": not np.allclose(dH @ p.W1.T, g["dX"]),
        "derivative of the erf form instead of the tanh form": not np.allclose(
            (dH * (0.5 * (1 + np.vectorize(__import__("math").erf)(Z / np.sqrt(2)))
                   + Z * np.exp(-Z * Z / 2) / np.sqrt(2 * np.pi))) @ p.W1.T, g["dX"], rtol=1e-6),
        "db1 summed over the wrong axis": dH.sum(axis=1).shape != g["db1"].shape,
        "bias b1 dropped": not np.allclose(orc.act(p.X @ p.W1, p.kind) @ p.W2 + p.b2, orc.ffn_forward(p)),
    }
    assert all(wrong.values()), wrong
