"""fp64 CPU oracle for the co-sharded feed-forward operator, forward and backward.

TEST INFRASTRUCTURE ONLY.  Plain reference the HIP path is judged against: it shares
no code with the HIP path, imports nothing from the product package and must never be
called from a product code path.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may use it.

What it follows
---------------
The paper applies the co-shard plan to the feed-forward operator as well as to attention
(Section 6.1 "parallelization plans": attention heads and feed-forward hidden dimensions are
partitioned; Section 6.3: co-shard is applied to the attention and feed-forward operators, with
recompute).  Following Section 2 and Section 3.1 the operator is split along its hidden
dimension into k functionally equivalent sub-operators that run one after another on one GPU.
Unlike the head split of attention, every sub-operator contributes to the *whole* output: the
outputs are value-split partial sums that have to be added (Section 4, RVD: a V-split tensor;
Section 5 for the gradient of the shared input).  The operator itself is the one the paper
cites (position-wise feed-forward of the original Transformer), which it does not print:

    Z = X W1 + b1            X [T, dm], W1 [dm, dh], b1 [dh]
    H = act(Z)               act = ReLU (the cited definition) or GELU in its tanh form
    Y = H W2 (+ b2)          W2 [dh, dm]

    dH = dY W2^T ; dZ = dH * act'(Z)
    dW2 = H^T dY ; db2 = sum_t dY ; dW1 = X^T dZ ; db1 = sum_t dZ ; dX = dZ W1^T

A GPU's share is a hidden range [lo, hi) (tensor parallelism over the hidden dimension): it
produces the partial sum of Y and dX over that range, and the slices [lo, hi) of dW1, db1, dW2.
Co-shard cuts [lo, hi) into k chunks; partial sums over the chunks are added, slices are
concatenated.  b2 belongs to the full operator, not to a hidden range: it is added when given.

Everything is evaluated in float64 on inputs already rounded to the run dtype.

Pins: tests/test_ffn_oracle_pins.py (scalar-loop brute force, central finite differences on every
input, a library implementation with library autograd, closed forms, the chunk invariant, a
planted-mistake check).  The paper prints no worked numeric example for this operator.
"""
from __future__ import annotations

import numpy as np

ACT_RELU = 0
ACT_GELU_TANH = 1

_C0 = 0.7978845608028654  # sqrt(2/pi)
_C1 = 0.044715


def chunk_ranges(lo: int, hi: int, k: int, unit: int = 1):
    """Split the hidden range [lo,hi) into k consecutive chunks, as even as possible (Section 4
    assumes even partitions; the balanced floor split extends that to k not dividing the range).
    `unit` is an interface parameter, not part of the method: an implementation may promise chunk
    boundaries at multiples of `unit` columns counted from lo, and the split is then balanced in
    whole units.  The default is the plain split.  Chunks may be empty only if k exceeds the
    number of units."""
    n = hi - lo
    units = -(-n // unit)
    out = []
    for c in range(k):
        a = lo + min(n, unit * (c * units // k))
        b = lo + min(n, unit * ((c + 1) * units // k))
        out.append((a, b))
    return out


def act(z, kind):
    if kind == ACT_RELU:
        return np.maximum(z, 0.0)
    u = _C0 * (z + _C1 * z ** 3)
    return 0.5 * z * (1.0 + np.tanh(u))


def act_grad(z, kind):
    if kind == ACT_RELU:
        return (z > 0).astype(np.float64)
    u = _C0 * (z + _C1 * z ** 3)
    t = np.tanh(u)
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * _C0 * (1.0 + 3.0 * _C1 * z * z)


class FfnProblem:
    def __init__(self, X, W1, b1, W2, b2=None, kind=ACT_GELU_TANH):
        f = lambda a: None if a is None else np.asarray(a, dtype=np.float64)
        self.X, self.W1, self.b1, self.W2, self.b2, self.kind = f(X), f(W1), f(b1), f(W2), f(b2), kind
        self.T, self.dm = self.X.shape
        self.dh = self.W1.shape[1]
        assert self.W1.shape == (self.dm, self.dh) and self.W2.shape == (self.dh, self.dm)
        assert self.b1.shape == (self.dh,)


def ffn_forward(p: FfnProblem, lo=0, hi=None, add_b2=True):
    """Partial output over the hidden range [lo,hi): Y [T, dm]."""
    hi = p.dh if hi is None else hi
    Z = np.matmul(p.X, p.W1[:, lo:hi]) + p.b1[lo:hi]
    Y = np.matmul(act(Z, p.kind), p.W2[lo:hi])
    if add_b2 and p.b2 is not None:
        Y = Y + p.b2
    return Y


def ffn_backward(p: FfnProblem, dY, lo=0, hi=None):
    """Gradients of the share [lo,hi): dX is the partial sum over the range; dW1, db1, dW2 are
    returned at full size with zeros outside [lo,hi); db2 is the full gradient of b2."""
    hi = p.dh if hi is None else hi
    dY = np.asarray(dY, dtype=np.float64)
    Z = np.matmul(p.X, p.W1[:, lo:hi]) + p.b1[lo:hi]   # recomputed: nothing kept from the forward
    H = act(Z, p.kind)
    dH = np.matmul(dY, p.W2[lo:hi].T)
    dZ = dH * act_grad(Z, p.kind)
    out = {"dX": np.matmul(dZ, p.W1[:, lo:hi].T), "dW1": np.zeros_like(p.W1), "db1": np.zeros_like(p.b1),
           "dW2": np.zeros_like(p.W2), "db2": dY.sum(axis=0)}
    out["dW1"][:, lo:hi] = np.matmul(p.X.T, dZ)
    out["db1"][lo:hi] = dZ.sum(axis=0)
    out["dW2"][lo:hi] = np.matmul(H.T, dY)
    return out


def coshard_forward(p: FfnProblem, lo, hi, k, unit=1):
    """The k sub-operators one after another; their outputs are partial sums and are added."""
    Y = np.zeros((p.T, p.dm))
    for a, b in chunk_ranges(lo, hi, k, unit):
        if b > a:
            Y += ffn_forward(p, a, b, add_b2=False)
    if p.b2 is not None:
        Y += p.b2
    return Y


def coshard_backward(p: FfnProblem, dY, lo, hi, k, unit=1):
    tot = None
    for a, b in chunk_ranges(lo, hi, k, unit):
        if b <= a:
            continue
        g = ffn_backward(p, dY, a, b)
        if tot is None:
            tot = g
        else:
            for n in ("dX", "dW1", "db1", "dW2"):   # dX: value-split sum; the others: disjoint slices
                tot[n] = tot[n] + g[n]
    return tot
