"""The backward entry point that allocates nothing (ss_attn_bwd_static: scratch built into the
library instead of a caller workspace) against ss_attn_bwd on the same inputs: every output bit for
bit, on two calls in a row of which the second is smaller (the built-in buffer then still holds the
first call's contents), for a biased gated row-split case and a causal head-split one."""
import pytest

from paper_2301_08984_amd import binding as ss

pytestmark = pytest.mark.gpu

PAIRS = {
    "af2_like": (dict(seed=71, B=6, H=2, S=200, D=32, dtype="bf16", bias="dense", gated=True, axis="row"), 3,
                 dict(seed=72, B=3, H=2, S=100, D=32, dtype="bf16", bias="dense", gated=True, axis="row"), 2),
    "gpt_like": (dict(seed=73, B=1, H=4, S=600, D=128, dtype="bf16", mask="causal", axis="head"), 2,
                 dict(seed=74, B=1, H=2, S=300, D=128, dtype="bf16", mask="causal", axis="head"), 1),
    "swin_like": (dict(seed=75, B=40, H=4, S=49, D=32, dtype="bf16", bias="relpos", win=(7, 7), mask="region",
                       axis="row"), 4,
                  dict(seed=76, B=9, H=4, S=49, D=32, dtype="bf16", bias="relpos", win=(7, 7), mask="region",
                       axis="row"), 2),
}
OUTS = ("dQ", "dK", "dV", "dG", "dBias")


def _both(cfg, k):
    import torch
    from paper_2301_08984_amd.runner import DeviceCase
    from paper_2301_08984_amd.workloads import make_inputs
    inp = make_inputs(**cfg)
    mk = lambda: DeviceCase(inp, dtype=cfg["dtype"], bias=cfg.get("bias"), mask=cfg.get("mask"),
                            gated=cfg.get("gated", False), win=cfg.get("win"))
    ref, dc = mk(), mk()
    ext = ref.H if cfg["axis"] == "head" else ref.B
    d = ref.desc(cfg["axis"], 0, ext, k)
    ref.bwd(d, poison=True)
    st = torch.cuda.current_stream(dc.dev).cuda_stream
    before = torch.cuda.memory_allocated(dc.dev)
    ss.ss_attn_bwd_static(d, dc.Q, dc.K, dc.V, dc.bias, dc.region, dc.G, dc.dY, None, dc.dQ, dc.dK, dc.dV, dc.dBias,
                          dc.dG, st)
    assert torch.cuda.memory_allocated(dc.dev) == before
    torch.cuda.synchronize()
    for n in OUTS:
        a, b = getattr(dc, n), getattr(ref, n)
        if a is not None:
            assert torch.equal(torch.nan_to_num(a, nan=12345.0), torch.nan_to_num(b, nan=12345.0)), n
            assert bool(a.isfinite().all()), n


@pytest.mark.parametrize("name", list(PAIRS))
def test_static_scratch_backward_matches_workspace_backward(name):
    big, kb, small, ks = PAIRS[name]
    print(f"no-alloc backward {name}: first call", flush=True)
    _both(big, kb)
    print(f"no-alloc backward {name}: second, smaller call", flush=True)
    _both(small, ks)
