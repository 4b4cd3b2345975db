"""Device-side harness: puts one workload's tensors in HBM (torch is used for
allocation and streams only) and calls the C ABI through `binding`.  No
attention arithmetic happens here."""
from __future__ import annotations

import math

import numpy as np
import torch

from . import binding as ss

_AXIS = {"head": ss.SS_AXIS_HEAD, "row": ss.SS_AXIS_ROW}
_MASK = {None: ss.SS_MASK_NONE, "causal": ss.SS_MASK_CAUSAL, "region": ss.SS_MASK_REGION}
_BIAS = {None: ss.SS_BIAS_NONE, "dense": ss.SS_BIAS_DENSE, "relpos": ss.SS_BIAS_RELPOS}


class DeviceCase:
    """One attention operator resident on the GPU plus its output buffers."""

    def __init__(self, inputs: dict, *, dtype: str, bias=None, mask=None, gated=False, win=None,
                 scale=None, device="cuda:0", fill=float("nan"), layout="bshd"):
        """`layout`: how the [B,S,H,D] activations sit in memory.  "bshd": packed as indexed.  "sbhd":
        the two leading axes swapped in storage (the operator walks the *second* storage axis as its
        sequence): the transposed variants of a row-wise operator, e.g. attention along MSA columns,
        reached through stride_b / stride_s alone."""
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the HIP path has no CPU fallback")
        self.dev = torch.device(device)
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.dtype = ss.SS_BF16 if dtype == "bf16" else ss.SS_F32
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(self.dev).to(self.tdtype).contiguous()
        self.layout = layout
        if layout == "sbhd":
            # stored [S,B,H,D]; every activation is kept as its logical [B,S,H,D] view of that storage
            act = lambda a: up(a).permute(1, 0, 2, 3).contiguous().permute(1, 0, 2, 3)
        elif layout == "bshd":
            act = up
        else:
            raise ValueError(layout)
        self.Q, self.K, self.V, self.dY = (act(inputs[n]) for n in ("Q", "K", "V", "dY"))
        self.B, self.S, self.H, self.D = self.Q.shape
        self.scale = (1.0 / math.sqrt(self.D)) if scale is None else scale
        self.bias_kind, self.mask_kind, self.gated, self.win = _BIAS[bias], _MASK[mask], gated, win or (0, 0)
        self.bias = up(inputs["bias"]) if bias else None
        self.G = act(inputs["G"]) if gated else None
        self.region = None
        self.mask_period = 0
        if mask == "region":
            self.region = torch.from_numpy(np.ascontiguousarray(inputs["region_ids"], dtype=np.int32)).to(self.dev)
            self.mask_period = self.region.shape[0]
        mk = lambda: torch.full_like(self.Q, fill, memory_format=torch.preserve_format)
        self.Y, self.dQ, self.dK, self.dV = mk(), mk(), mk(), mk()
        self.dG = mk() if gated else None
        self.lse = torch.full((self.B, self.H, self.S), fill, dtype=torch.float32, device=self.dev)
        self.dBias = (torch.full(self.bias.shape, fill, dtype=torch.float32, device=self.dev)
                      if bias else None)
        self.ws = None

    def desc(self, axis, lo, hi, k, flags=0):
        sb, ss_, sh, sd = self.Q.stride()
        assert sd == 1
        return ss.make_desc(self.B, self.H, self.S, self.D, self.dtype, self.scale, _AXIS[axis], lo, hi, k,
                            stride_b=sb, stride_s=ss_, stride_h=sh, bias_kind=self.bias_kind, win=self.win, mask_kind=self.mask_kind,
                            mask_period=self.mask_period, gated=self.gated, flags=flags)

    def workspace(self, desc):
        _, need = ss.ss_attn_workspace_bytes(desc)
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.dev)
        return need

    def fwd(self, desc, want_lse=True, stream=None):
        st = torch.cuda.current_stream(self.dev).cuda_stream if stream is None else stream
        ss.ss_attn_fwd(desc, self.Q, self.K, self.V, self.bias, self.region, self.G, self.Y,
                       self.lse if want_lse else None, None, 0, st)

    def bwd(self, desc, use_lse=False, stream=None, poison=False):
        """`poison`: fill the workspace with 0xFF bytes (NaN in every float format) first, so that a
        kernel that reads scratch it has not written in this call shows up in the results."""
        need = self.workspace(desc)
        if poison:
            self.ws.fill_(0xFF)
        st = torch.cuda.current_stream(self.dev).cuda_stream if stream is None else stream
        ss.ss_attn_bwd(desc, self.Q, self.K, self.V, self.bias, self.region, self.G, self.dY,
                       self.lse if use_lse else None, self.dQ, self.dK, self.dV, self.dBias, self.dG,
                       self.ws, self.ws.numel(), st)
        return need

    def caller_bytes(self):
        """Bytes of every tensor the caller holds for forward+backward (without the workspace)."""
        ts = [self.Q, self.K, self.V, self.dY, self.Y, self.dQ, self.dK, self.dV, self.G, self.dG,
              self.bias, self.dBias, self.region, self.lse]
        return sum(t.numel() * t.element_size() for t in ts if t is not None)

    def host(self, name):
        t = getattr(self, name)
        return None if t is None else t.detach().float().cpu().numpy().astype(np.float64)


class FfnCase:
    """One feed-forward operator resident on the GPU plus its output buffers (bf16)."""

    def __init__(self, inputs: dict, *, act="gelu", device="cuda:0", fill=float("nan"), pad=(0, 0, 0)):
        """pad = extra elements (multiples of 8) in the leading dimension of the [T, dm] matrices, of
        W1 / dW1 and of W2 / dW2; the padding holds NaN, so any read of it shows in the results."""
        from . import ffn_binding as fb
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the HIP path has no CPU fallback")
        self.fb = fb
        self.dev = torch.device(device)
        self.pad = tuple(pad)

        def matrix(rows, cols, extra, values=None):
            buf = torch.full((rows, cols + extra), float("nan") if values is not None else fill, dtype=torch.bfloat16,
                             device=self.dev)
            view = buf[:, :cols]
            if values is not None:
                view.copy_(torch.from_numpy(np.ascontiguousarray(values)).to(self.dev).to(torch.bfloat16))
            elif extra:
                buf[:, cols:] = float("nan")
            return view

        vec = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(self.dev).to(torch.bfloat16)
        self.T, self.dm = inputs["X"].shape
        self.dh = inputs["W1"].shape[1]
        px, pw1, pw2 = self.pad
        self.X = matrix(self.T, self.dm, px, inputs["X"])
        self.dY = matrix(self.T, self.dm, px, inputs["dY"])
        self.W1 = matrix(self.dm, self.dh, pw1, inputs["W1"])
        self.W2 = matrix(self.dh, self.dm, pw2, inputs["W2"])
        self.b1, self.b2 = vec(inputs.get("b1")), vec(inputs.get("b2"))
        self.act = fb.SS_ACT_GELU_TANH if act == "gelu" else fb.SS_ACT_RELU
        self.Y, self.dX = matrix(self.T, self.dm, px), matrix(self.T, self.dm, px)
        self.dW1, self.dW2 = matrix(self.dm, self.dh, pw1), matrix(self.dh, self.dm, pw2)
        self.db1, self.db2 = torch.full_like(self.b1, fill), torch.full((self.dm,), fill, dtype=torch.bfloat16, device=self.dev)
        self.ws = None

    def desc(self, lo, hi, k, flags=0):
        return self.fb.make_desc(self.T, self.dm, self.dh, lo, hi, k, act=self.act, ld_x=self.dm + self.pad[0],
                                 ld_w1=self.dh + self.pad[1], ld_w2=self.dm + self.pad[2], flags=flags)

    def workspace(self, desc):
        f, b = self.fb.ss_ffn_workspace_bytes(desc)
        need = max(f, b, 256)
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
        return f, b

    def fwd(self, desc, poison=False, stream=None):
        self.workspace(desc)
        if poison:
            self.ws.fill_(0xFF)
        st = torch.cuda.current_stream(self.dev).cuda_stream if stream is None else stream
        self.fb.ss_ffn_fwd(desc, self.X, self.W1, self.b1, self.W2, self.b2, self.Y, self.ws, self.ws.numel(), st)

    def bwd(self, desc, poison=False, stream=None):
        self.workspace(desc)
        if poison:
            self.ws.fill_(0xFF)
        st = torch.cuda.current_stream(self.dev).cuda_stream if stream is None else stream
        self.fb.ss_ffn_bwd(desc, self.X, self.W1, self.b1, self.W2, self.dY, self.dX, self.dW1, self.db1, self.dW2,
                           self.db2, self.ws, self.ws.numel(), st)

    def caller_bytes(self):
        ts = [self.X, self.W1, self.b1, self.W2, self.b2, self.dY, self.Y, self.dX, self.dW1, self.db1, self.dW2,
              self.db2]
        return sum(t.numel() * t.element_size() for t in ts if t is not None)

    def host(self, name):
        t = getattr(self, name)
        return None if t is None else t.detach().float().cpu().numpy().astype(np.float64)
