"""Seeded synthetic inputs shaped like the workloads the co-shard plan is run on.

This module holds no attention arithmetic.  It draws random tensors, rounds
them once to the run dtype, and describes each workload (shapes, which bias and
mask it carries, the split axis and the co-shard factors).  Both the test
oracle and the HIP path are fed from here so that they see the same bits.

Recipe (all draws from numpy Generator(PCG64(seed)), float32, in the fixed
order Q, K, V, dY, bias-or-table, G):
  * activations ~ N(0,1), layout [B, S, H, D] contiguous;
  * dense bias ~ N(0,1) [H,S,S]; relative-position table ~ N(0, 0.02^2) [H,R];
  * gate logits ~ N(0,1);
  * bf16 runs: every tensor is rounded to bfloat16 (round to nearest even) once
    here; the oracle upcasts those bits exactly to float64.
The shifted-window region ids imitate a 112x112-token feature map cut into
7x7 windows after a cyclic shift of 3: a token's id is 3*r(y)+c(x), with r and
c in {0,1,2} telling whether the coordinate lies before the last window, in
the last window before the shifted seam, or after it.
"""
from __future__ import annotations

import numpy as np


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array -> float32 array holding bfloat16-representable values (RNE)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array of bf16-representable values -> uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bits_to_f32(u16: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 values."""
    return (np.ascontiguousarray(u16).astype(np.uint32) << 16).view(np.float32).reshape(u16.shape)


def shifted_window_region_ids(map_hw: int = 112, win: int = 7, shift: int = 3) -> np.ndarray:
    """int32 [num_windows, win*win] region id of every token of every window."""
    def band(c):
        return 0 if c < map_hw - win else (1 if c < map_hw - shift else 2)
    img = np.empty((map_hw, map_hw), dtype=np.int32)
    for y in range(map_hw):
        for x in range(map_hw):
            img[y, x] = 3 * band(y) + band(x)
    n = map_hw // win
    ids = img.reshape(n, win, n, win).transpose(0, 2, 1, 3).reshape(n * n, win * win)
    return np.ascontiguousarray(ids)


# name -> description.  "k" lists the co-shard factors the workload is run with.
WORKLOADS = {
    "tiny_mha": dict(seed=1001, B=1, H=4, S=128, D=32, dtype="f32", bias=None, mask=None,
                     gated=False, axis="head", k=(1, 2)),
    "gpt3_shard": dict(seed=2002, B=1, H=12, S=2048, D=128, dtype="bf16", bias=None, mask="causal",
                       gated=False, axis="head", k=(1, 2, 4)),
    "swin_window": dict(seed=3003, B=4096, H=16, S=49, D=32, dtype="bf16", bias="relpos", win=(7, 7),
                        mask="region", gated=False, axis="row", k=(4,)),
    "af2_msa_row": dict(seed=4004, B=512, H=8, S=384, D=32, dtype="bf16", bias="dense", mask=None,
                        gated=True, axis="row", k=(1, 4, 16)),
    "af2_triangle": dict(seed=5005, B=1024, H=4, S=1024, D=32, dtype="bf16", bias="dense", mask=None,
                         gated=True, axis="row", k=(4, 16, 64)),
    # beyond the five headline configurations: the long-document setting of Section 6.3 (sequence
    # lengths of 10k-16k tokens, where co-shard's memory argument is made) on the same GPT share
    # the transposed AlphaFold2 operators: same kernels, the two leading axes swapped in storage
    # (`layout="sbhd"`: stride_b < stride_s, every row of a tile a separate 64-byte segment):
    # MSA column attention (per residue column, across the 512 sequences; gated, no pair bias) and
    # triangle attention around the ending node
    "af2_msa_col": dict(seed=7007, B=384, H=8, S=512, D=32, dtype="bf16", bias=None, mask=None,
                        gated=True, axis="row", k=(1, 4, 16), layout="sbhd"),
    "af2_triangle_end": dict(seed=8008, B=1024, H=4, S=1024, D=32, dtype="bf16", bias="dense", mask=None,
                             gated=True, axis="row", k=(4, 16, 64), layout="sbhd"),
    "gpt3_long": dict(seed=6006, B=1, H=12, S=12288, D=128, dtype="bf16", bias=None, mask="causal",
                      gated=False, axis="head", k=(1, 2, 4)),
    # the upper end of that range
    "gpt3_long_16k": dict(seed=6016, B=1, H=12, S=16384, D=128, dtype="bf16", bias=None, mask="causal",
                          gated=False, axis="head", k=(1, 2, 4)),
}


def make_inputs(B, H, S, D, dtype="bf16", bias=None, mask=None, gated=False, seed=0, win=None,
                rows=None, **_unused):
    """Draw one workload's tensors.  Returns a dict of float32 numpy arrays
    (already rounded to `dtype`) plus 'region_ids' (int32) when mask == "region".

    `rows`: optional (lo, hi): only rows [lo,hi) of the activations are drawn
    (shape [hi-lo,S,H,D]) from a generator keyed by (seed, tensor, row), so a
    slice of a large workload is the same bits as the same rows of a larger slice.
    """
    rnd = (lambda a: round_to_bf16(a)) if dtype == "bf16" else (lambda a: np.ascontiguousarray(a, np.float32))
    out = {}
    if rows is None:
        g = np.random.Generator(np.random.PCG64(seed))
        for name in ("Q", "K", "V", "dY"):
            out[name] = rnd(g.standard_normal((B, S, H, D), dtype=np.float32))
    else:
        lo, hi = rows
        for t, name in enumerate(("Q", "K", "V", "dY")):
            buf = np.empty((hi - lo, S, H, D), dtype=np.float32)
            for b in range(lo, hi):
                gb = np.random.Generator(np.random.PCG64([seed, t, b]))
                buf[b - lo] = gb.standard_normal((S, H, D), dtype=np.float32)
            out[name] = rnd(buf)
        g = np.random.Generator(np.random.PCG64([seed, 99]))
    if bias == "dense":
        out["bias"] = rnd(g.standard_normal((H, S, S), dtype=np.float32))
    elif bias == "relpos":
        wh, ww = win
        assert wh * ww == S
        out["bias"] = rnd(0.02 * g.standard_normal((H, (2 * wh - 1) * (2 * ww - 1)), dtype=np.float32))
    if gated:
        if rows is None:
            out["G"] = rnd(g.standard_normal((B, S, H, D), dtype=np.float32))
        else:
            lo, hi = rows
            buf = np.empty((hi - lo, S, H, D), dtype=np.float32)
            for b in range(lo, hi):
                gb = np.random.Generator(np.random.PCG64([seed, 7, b]))
                buf[b - lo] = gb.standard_normal((S, H, D), dtype=np.float32)
            out["G"] = rnd(buf)
    if mask == "region":
        w = 7 if win is None else win[0]
        assert win is None or win[0] == win[1], "region-id recipe is for square windows"
        # 16 windows per side, cyclic shift of half a window (7 -> 112x112 map, shift 3)
        out["region_ids"] = shifted_window_region_ids(16 * w, w, w // 2)
    return out


# ---------------------------------------------------------------------------
# Feed-forward operator (the other operator the co-shard plan is applied to, Sections 6.1 and 6.3)
# ---------------------------------------------------------------------------
FFN_WORKLOADS = {
    "tiny_ffn": dict(seed=9001, T=100, dm=64, dh=256, lo=0, hi=256, act="gelu", k=(1, 2, 4)),
    # one GPU's tensor-parallel share of a GPT-3 175B feed-forward block: d_model 12288, hidden 49152
    # split 8 ways, 2048 tokens (the sequence of the attention share)
    "gpt3_ffn": dict(seed=9002, T=2048, dm=12288, dh=6144, lo=0, hi=6144, act="gelu", k=(1, 2, 4)),
    # the same share with a micro-batch of four sequences: enough tiles in every product to fill the chip
    "gpt3_ffn_mb4": dict(seed=9003, T=8192, dm=12288, dh=6144, lo=0, hi=6144, act="gelu", k=(1, 2, 4)),
}


def make_ffn_inputs(T, dm, dh, seed=0, **_unused):
    """Seeded float32 arrays already rounded to bf16: X, dY ~ N(0,1); W1 ~ N(0, 1/dm), W2 ~ N(0, 1/dh) (so
    that pre-activations and outputs are O(1)); biases ~ N(0, 0.02^2)."""
    g = np.random.Generator(np.random.PCG64(seed))
    rnd = round_to_bf16
    out = {"X": rnd(g.standard_normal((T, dm), dtype=np.float32)),
           "dY": rnd(g.standard_normal((T, dm), dtype=np.float32)),
           "W1": rnd(g.standard_normal((dm, dh), dtype=np.float32) * np.float32(dm ** -0.5)),
           "W2": rnd(g.standard_normal((dh, dm), dtype=np.float32) * np.float32(dh ** -0.5)),
           "b1": rnd(g.standard_normal(dh, dtype=np.float32) * np.float32(0.02)),
           "b2": rnd(g.standard_normal(dm, dtype=np.float32) * np.float32(0.02))}
    return out
