"""fp64 CPU oracle for co-sharded multi-head attention, forward and backward.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP
path is judged against.  It shares no code with the HIP path, imports nothing
from the product package, and must never be called from a product code path.
Only tests, the smoke check and the benchmark's cpu_baseline leg may use it.

What it follows
---------------
The paper (SuperScaler, Section 2 "co-shard"; Section 3.1 "op-trans";
Section 3.2 "op-assign"/"op-order"; Section 3.3 dependency materialisation;
Section 4 "RVD representation"; Section 5 "Autograd for forward operator
transformation") defines the *plan*: an operator is split along one axis into
k functionally equivalent sub-operators, all placed on the same GPU and run
one after another; outputs whose axis was split are concatenated, gradients of
a tensor that every sub-operator consumes are value-partitioned and must be
summed.  The paper does not print the attention operator itself (it names it
and cites the original), so the operator below is the textbook definition of
scaled-dot-product attention with an additive bias, a 0/-inf mask and an
optional sigmoid output gate, and its analytic gradient:

    S[i,j]  = scale * sum_d Q[i,d] K[j,d] + Bias[h,i,j]
    P[i,:]  = softmax over unmasked j of S[i,:]         (masked => P = 0 exactly)
    O       = P V ;  Y = sigmoid(G) * O  if gated else O
    LSE[i]  = log sum_{j unmasked} exp(S[i,j])

    g = sigmoid(G); dO = dY*g (gated) ; dG = dY * O * g * (1-g)
    dV = P^T dO ; dP = dO V^T ; Delta_i = sum_j P[i,j] dP[i,j]
    dS = P * (dP - Delta_i) ; dQ = scale * dS K ; dK = scale * dS^T Q
    dBias[h,i,j] = sum_b dS[b,h,i,j]
    dTable[h,r]  = sum_b sum_{(i,j): idx(i,j)=r} dS[b,h,i,j]

Everything is evaluated in float64 on inputs that are already rounded to the
run dtype (the caller upcasts exactly).  Tensors are laid out [B, S, H, D]
("B" is the batch-like row axis: batch, window, MSA row or triangle row).

Pins: tests/test_oracle_pins.py checks every function here against brute force
on tiny inputs (a differently written formulation with an explicit softmax
Jacobian), central finite differences, closed forms, a library attention
routine with library autograd, and the chunk invariant.  The paper prints no
worked numeric example for attention, so no pin comes from the paper's text.
"""
from __future__ import annotations

import numpy as np

AXIS_HEAD = 0
AXIS_ROW = 1


# ----------------------------------------------------------------------------
# Plan arithmetic (Section 4, RVD: uniform partition of one axis into k parts)
# ----------------------------------------------------------------------------
def chunk_ranges(lo: int, hi: int, k: int):
    """Split [lo,hi) into k consecutive, balanced, non-empty sub-ranges.

    The paper assumes even partitions (Section 4, "most parallelization plans
    partition operators evenly"); for a k that does not divide n = hi-lo the
    reading taken is the balanced floor split: chunk c = [lo + floor(c*n/k),
    lo + floor((c+1)*n/k)).
    """
    n = hi - lo
    if not (1 <= k <= n):
        raise ValueError("need 1 <= k <= hi-lo")
    return [(lo + (c * n) // k, lo + ((c + 1) * n) // k) for c in range(k)]


def relpos_index(win_h: int, win_w: int) -> np.ndarray:
    """idx[i,j] into a relative-position table of (2*win_h-1)*(2*win_w-1) entries.

    Token i sits at (y,x) = (i // win_w, i % win_w); the entry is selected by
    the displacement (yi-yj, xi-xj), row-major over displacements shifted to be
    non-negative.
    """
    S = win_h * win_w
    idx = np.empty((S, S), dtype=np.int64)
    for i in range(S):
        yi, xi = divmod(i, win_w)
        for j in range(S):
            yj, xj = divmod(j, win_w)
            idx[i, j] = (yi - yj + win_h - 1) * (2 * win_w - 1) + (xi - xj + win_w - 1)
    return idx


class AttnProblem:
    """All inputs of one attention operator (whole tensors, before any split).

    Q, K, V, (G), (dY): float64 [B,S,H,D].
    bias: None | ("dense", [H,S,S]) | ("relpos", [H,R], win_h, win_w)
    mask: None | ("causal",) | ("region", int ids [period,S])
    """

    def __init__(self, Q, K, V, scale, bias=None, mask=None, G=None):
        self.Q = np.asarray(Q, dtype=np.float64)
        self.K = np.asarray(K, dtype=np.float64)
        self.V = np.asarray(V, dtype=np.float64)
        self.G = None if G is None else np.asarray(G, dtype=np.float64)
        self.scale = float(scale)
        self.bias = bias
        self.mask = mask
        self.B, self.S, self.H, self.D = self.Q.shape
        if bias is not None and bias[0] == "relpos":
            self._idx = relpos_index(bias[2], bias[3])
            assert self._idx.shape == (self.S, self.S)

    # additive bias of head h as an [S,S] matrix
    def bias_matrix(self, h):
        if self.bias is None:
            return None
        if self.bias[0] == "dense":
            return np.asarray(self.bias[1], dtype=np.float64)[h]
        if self.bias[0] == "relpos":
            return np.asarray(self.bias[1], dtype=np.float64)[h][self._idx]
        raise ValueError(self.bias[0])

    # boolean [S,S], True where the pair (i,j) is masked out, for row b
    def masked(self, b):
        if self.mask is None:
            return None
        if self.mask[0] == "causal":
            i = np.arange(self.S)
            return i[None, :] > i[:, None]
        if self.mask[0] == "region":
            ids = np.asarray(self.mask[1])
            r = ids[b % ids.shape[0]]
            return r[:, None] != r[None, :]
        raise ValueError(self.mask[0])


def _probabilities(p: AttnProblem, b: int, h: int):
    """P [S,S] and LSE [S] of one (row, head) pair, from the definition."""
    S = p.scale * (p.Q[b, :, h, :] @ p.K[b, :, h, :].T)
    Bm = p.bias_matrix(h)
    if Bm is not None:
        S = S + Bm
    M = p.masked(b)
    if M is not None:
        if np.any(np.all(M, axis=1)):
            raise ValueError("a query row has every key masked (precondition violated)")
        S = np.where(M, -np.inf, S)
    m = np.max(S, axis=1, keepdims=True)
    E = np.exp(S - m)  # exp(-inf) = 0 exactly on masked pairs
    l = np.sum(E, axis=1, keepdims=True)
    return E / l, (m + np.log(l))[:, 0]


def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def _range(p: AttnProblem, axis, lo, hi):
    if axis == AXIS_HEAD:
        if not (0 <= lo < hi <= p.H):
            raise ValueError("bad head range")
        return range(p.B), range(lo, hi)
    if axis == AXIS_ROW:
        if not (0 <= lo < hi <= p.B):
            raise ValueError("bad row range")
        return range(lo, hi), range(p.H)
    raise ValueError("axis")


# ----------------------------------------------------------------------------
# The unsplit operator on a sub-range [lo,hi) of one axis
# ----------------------------------------------------------------------------
def attn_forward(p: AttnProblem, axis=AXIS_HEAD, lo=0, hi=None):
    """Y [B,S,H,D] and LSE [B,H,S]; entries outside the range are left 0."""
    if hi is None:
        hi = p.H if axis == AXIS_HEAD else p.B
    rows, heads = _range(p, axis, lo, hi)
    Y = np.zeros_like(p.Q)
    LSE = np.zeros((p.B, p.H, p.S))
    for b in rows:
        for h in heads:
            P, lse = _probabilities(p, b, h)
            O = P @ p.V[b, :, h, :]
            if p.G is not None:
                O = _sigmoid(p.G[b, :, h, :]) * O
            Y[b, :, h, :] = O
            LSE[b, h, :] = lse
    return Y, LSE


def attn_backward(p: AttnProblem, dY, axis=AXIS_HEAD, lo=0, hi=None):
    """Gradients of L = sum(dY * Y) restricted to the range.

    Returns dict with dQ, dK, dV [B,S,H,D] (0 outside the range), dG (if
    gated), and dBias: dense -> [H,S,S]; relpos -> [H,R]; summed over the rows
    of the range (for a head range only heads inside it are non-zero).
    """
    if hi is None:
        hi = p.H if axis == AXIS_HEAD else p.B
    rows, heads = _range(p, axis, lo, hi)
    dY = np.asarray(dY, dtype=np.float64)
    out = {k: np.zeros_like(p.Q) for k in ("dQ", "dK", "dV")}
    if p.G is not None:
        out["dG"] = np.zeros_like(p.Q)
    dBias = None
    if p.bias is not None:
        dBias = np.zeros(np.asarray(p.bias[1]).shape)
    for b in rows:
        for h in heads:
            Qm, Km, Vm = p.Q[b, :, h, :], p.K[b, :, h, :], p.V[b, :, h, :]
            P, _ = _probabilities(p, b, h)
            dO = dY[b, :, h, :]
            if p.G is not None:
                g = _sigmoid(p.G[b, :, h, :])
                O = P @ Vm
                out["dG"][b, :, h, :] = dO * O * g * (1.0 - g)
                dO = dO * g
            dP = dO @ Vm.T
            Delta = np.sum(P * dP, axis=1, keepdims=True)
            dS = P * (dP - Delta)
            out["dV"][b, :, h, :] = P.T @ dO
            out["dQ"][b, :, h, :] = p.scale * (dS @ Km)
            out["dK"][b, :, h, :] = p.scale * (dS.T @ Qm)
            if dBias is not None:
                if p.bias[0] == "dense":
                    dBias[h] += dS
                else:
                    np.add.at(dBias[h], p._idx.ravel(), dS.ravel())
    if dBias is not None:
        out["dBias"] = dBias
    return out


def bias_grad_rows(p: AttnProblem, dY, h: int, queries, lo=0, hi=None):
    """Dense bias gradient restricted to chosen query rows: dBias[h, i, :] for i in
    `queries`, summed over rows b in [lo,hi).  Row i of the softmax and of dS depends on
    row i of Q, dY and G only, so it is evaluated from the definition without forming the
    other rows; used to check full-size runs on sampled rows.  Returns [len(queries), S]."""
    if p.bias is None or p.bias[0] != "dense":
        raise ValueError("dense bias only")
    hi = p.B if hi is None else hi
    dY = np.asarray(dY, dtype=np.float64)
    out = np.zeros((len(queries), p.S))
    for b in range(lo, hi):
        Km, Vm = p.K[b, :, h, :], p.V[b, :, h, :]
        M = p.masked(b)
        for n, i in enumerate(queries):
            s = p.scale * (Km @ p.Q[b, i, h, :]) + np.asarray(p.bias[1], dtype=np.float64)[h, i]
            if M is not None:
                s = np.where(M[i], -np.inf, s)
            e = np.exp(s - np.max(s))
            pr = e / np.sum(e)
            dO = dY[b, i, h, :]
            if p.G is not None:
                dO = dO * _sigmoid(p.G[b, i, h, :])
            dP = Vm @ dO
            out[n] += pr * (dP - np.sum(pr * dP))
    return out


# ----------------------------------------------------------------------------
# The co-shard form (Section 2): k sub-operators run one after another on the
# same device; split-axis outputs are concatenated, gradients of tensors that
# every sub-operator reads (the bias) are summed (Section 5, value partition).
# ----------------------------------------------------------------------------
def coshard_forward(p: AttnProblem, axis, lo, hi, k):
    Y = np.zeros_like(p.Q)
    LSE = np.zeros((p.B, p.H, p.S))
    for (a, b) in chunk_ranges(lo, hi, k):
        Yc, Lc = attn_forward(p, axis, a, b)
        if axis == AXIS_HEAD:
            Y[:, :, a:b, :] = Yc[:, :, a:b, :]
            LSE[:, a:b, :] = Lc[:, a:b, :]
        else:
            Y[a:b] = Yc[a:b]
            LSE[a:b] = Lc[a:b]
    return Y, LSE


def coshard_backward(p: AttnProblem, dY, axis, lo, hi, k):
    total = None
    for (a, b) in chunk_ranges(lo, hi, k):
        part = attn_backward(p, dY, axis, a, b)
        if total is None:
            total = {name: np.zeros_like(v) for name, v in part.items()}
        for name, v in part.items():
            if name == "dBias":
                total[name] += v  # value-split: reduce
            elif axis == AXIS_HEAD:
                total[name][:, :, a:b, :] = v[:, :, a:b, :]  # axis-split: concatenate
            else:
                total[name][a:b] = v[a:b]
    return total
