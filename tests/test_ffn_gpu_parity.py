"""GPU parity of the co-sharded feed-forward operator: the HIP path through the C ABI against the
fp64 oracle on the same seeded inputs, for every k, in both accumulation modes (partial sums of Y
and dX in the bf16 output itself: the default, whose workspace shrinks as 1/k; or in fp32 in the
workspace with SS_FFN_FLAG_EXACT_SUM); and the co-shard invariant across k: bit for bit for every
output in the fp32 mode and for the weight and bias gradients in both, within rounding for Y and dX
in the default mode."""
import numpy as np
import pytest

from oracle import ffn as orc
from paper_2301_08984_amd.workloads import FFN_WORKLOADS, make_ffn_inputs

from parity import ELEM_FAIL_MAX, elem_fail, rel_err

pytestmark = pytest.mark.gpu

TOL = 2e-2  # bf16 operands, fp32 accumulation: max|x - ref| / max|ref| per tensor

SMALL = {
    "tiny_ffn": FFN_WORKLOADS["tiny_ffn"],
    "ragged": dict(seed=61, T=333, dm=200, dh=424, lo=0, hi=424, act="gelu"),
    "sub_range_relu": dict(seed=62, T=130, dm=136, dh=512, lo=48, hi=400, act="relu"),
    "several_tiles": dict(seed=63, T=600, dm=320, dh=704, lo=0, hi=704, act="gelu"),
    "one_token": dict(seed=64, T=1, dm=64, dh=128, lo=0, hi=128, act="gelu"),
}


EXACT = 1  # SS_FFN_FLAG_EXACT_SUM


def _run(cfg, k, flags=0):
    import torch
    from paper_2301_08984_amd.runner import FfnCase
    inp = make_ffn_inputs(**cfg)
    fc = FfnCase(inp, act=cfg["act"])
    d = fc.desc(cfg["lo"], cfg["hi"], k, flags)
    fc.fwd(d, poison=True)
    fc.bwd(d, poison=True)
    torch.cuda.synchronize()
    return fc, inp


def _oracle(cfg, inp):
    kind = orc.ACT_GELU_TANH if cfg["act"] == "gelu" else orc.ACT_RELU
    p = orc.FfnProblem(inp["X"], inp["W1"], inp["b1"], inp["W2"], inp["b2"], kind)
    return orc.ffn_forward(p, cfg["lo"], cfg["hi"]), orc.ffn_backward(p, inp["dY"].astype(np.float64), cfg["lo"], cfg["hi"])


def _ks(cfg):
    units = -(-(cfg["hi"] - cfg["lo"]) // 16)
    return sorted({1, 2, 3, min(units, 7)})


@pytest.mark.parametrize("flags", [0, EXACT], ids=["sum_in_output", "sum_in_fp32"])
@pytest.mark.parametrize("name", list(SMALL))
def test_matches_oracle_for_every_k(name, flags):
    cfg = SMALL[name]
    lo, hi = cfg["lo"], cfg["hi"]
    for k in _ks(cfg):
        print(f"ffn case {name} k={k} flags={flags}", flush=True)
        fc, inp = _run(cfg, k, flags)
        Y, g = _oracle(cfg, inp)
        errs = {"Y": rel_err(fc.host("Y"), Y), "dX": rel_err(fc.host("dX"), g["dX"]),
                "dW1": rel_err(fc.host("dW1")[:, lo:hi], g["dW1"][:, lo:hi]),
                "db1": rel_err(fc.host("db1")[lo:hi], g["db1"][lo:hi]),
                "dW2": rel_err(fc.host("dW2")[lo:hi], g["dW2"][lo:hi]), "db2": rel_err(fc.host("db2"), g["db2"])}
        print(name, k, {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
        for n, e in errs.items():
            assert np.isfinite(e) and e <= TOL, (n, k, e)
        fails = {"Y": elem_fail(fc.host("Y"), Y, TOL), "dX": elem_fail(fc.host("dX"), g["dX"], TOL),
                 "dW1": elem_fail(fc.host("dW1")[:, lo:hi], g["dW1"][:, lo:hi], TOL),
                 "db1": elem_fail(fc.host("db1")[lo:hi], g["db1"][lo:hi], TOL),
                 "dW2": elem_fail(fc.host("dW2")[lo:hi], g["dW2"][lo:hi], TOL),
                 "db2": elem_fail(fc.host("db2"), g["db2"], TOL)}
        assert all(f <= ELEM_FAIL_MAX for f in fails.values()), ("element-wise failures", k, fails)
        # outside the share the weight gradients are left untouched (NaN fill)
        if lo > 0:
            assert np.all(np.isnan(fc.host("dW1")[:, :lo])) and np.all(np.isnan(fc.host("dW2")[:lo]))
        if hi < cfg["dh"]:
            assert np.all(np.isnan(fc.host("dW1")[:, hi:])) and np.all(np.isnan(fc.host("db1")[hi:]))


@pytest.mark.parametrize("flags", [0, EXACT], ids=["sum_in_output", "sum_in_fp32"])
@pytest.mark.parametrize("name", ["tiny_ffn", "ragged", "sub_range_relu", "several_tiles"])
def test_results_identical_across_k(name, flags):
    """The weight and bias gradients never depend on k; Y and dX are the same bits for every k when the
    partial sums are kept in fp32, and agree to a few bf16 roundings (one per chunk) when they live in
    the output."""
    cfg = SMALL[name]
    ref = None
    for k in _ks(cfg):
        print(f"ffn case {name} across k: k={k} flags={flags}", flush=True)
        fc, _ = _run(cfg, k, flags)
        outs = {n: fc.host(n) for n in ("Y", "dX", "dW1", "db1", "dW2", "db2")}
        if ref is None:
            ref = outs
        else:
            for n in outs:
                if flags == EXACT or n not in ("Y", "dX"):
                    assert np.array_equal(outs[n], ref[n], equal_nan=True), (name, k, n)
                else:
                    assert rel_err(outs[n], ref[n]) <= k * 2.0 ** -8, (name, k, n, rel_err(outs[n], ref[n]))


_FULL = {}


def _full_size_oracle():
    """Oracle values of the sampled rows / columns of the benchmark configuration (they do not depend
    on k): computed once."""
    if not _FULL:
        cfg = dict(FFN_WORKLOADS["gpt3_ffn"])
        inp = make_ffn_inputs(**cfg)
        kind = orc.ACT_GELU_TANH
        dY = inp["dY"].astype(np.float64)
        rows = [0, 1, 777, 2047]
        p = orc.FfnProblem(inp["X"][rows], inp["W1"], inp["b1"], inp["W2"], inp["b2"], kind)
        cols = [0, 15, 16, 1535, 1536, 3071, 3072, 4607, 4608, 6143]   # both sides of every boundary of k = 2, 4
        q = orc.FfnProblem(inp["X"], inp["W1"][:, cols], inp["b1"][cols], inp["W2"][cols], None, kind)
        _FULL.update(cfg=cfg, inp=inp, rows=rows, cols=cols, Y=orc.ffn_forward(p), g=orc.ffn_backward(p, dY[rows]),
                     gq=orc.ffn_backward(q, dY))
    return _FULL


@pytest.mark.parametrize("k", FFN_WORKLOADS["gpt3_ffn"]["k"])
def test_full_size_gpt3_share_sampled(k):
    """The benchmark configuration, every k it names.  The oracle checks Y and dX on sampled tokens
    (rows are independent), dW1 / dW2 / db1 on sampled hidden columns (each needs all tokens but only
    its own column of the hidden layer), db2 in full.  Error scales come from the oracle's values."""
    import torch
    from paper_2301_08984_amd.runner import FfnCase
    o = _full_size_oracle()
    print(f"ffn full size gpt3_ffn k={k} (sampled)", flush=True)
    fc = FfnCase(o["inp"], act=o["cfg"]["act"])
    d = fc.desc(o["cfg"]["lo"], o["cfg"]["hi"], k)
    fc.fwd(d, poison=True)
    fc.bwd(d, poison=True)
    torch.cuda.synchronize()
    rows, cols, Y, g, gq = o["rows"], o["cols"], o["Y"], o["g"], o["gq"]
    for n, got, ref in (("Y", fc.host("Y")[rows], Y), ("dX", fc.host("dX")[rows], g["dX"]),
                        ("dW1", fc.host("dW1")[:, cols], gq["dW1"]), ("dW2", fc.host("dW2")[cols], gq["dW2"]),
                        ("db1", fc.host("db1")[cols], gq["db1"]), ("db2", fc.host("db2"), gq["db2"])):
        assert rel_err(got, ref) <= TOL, (n, k, rel_err(got, ref))
        assert elem_fail(got, ref, TOL) <= ELEM_FAIL_MAX, (n, k, elem_fail(got, ref, TOL))
    for n in ("Y", "dX", "dW1", "db1", "dW2", "db2"):
        assert bool(getattr(fc, n).isfinite().all()), n
    # across k at full size, against the first k run in this process: the weight and bias gradients bit for
    # bit; Y and dX (partial sums in the bf16 output, one rounding per chunk) within those roundings
    outs = {n: getattr(fc, n).clone() for n in ("Y", "dX", "dW1", "db1", "dW2", "db2")}
    first = o.setdefault("first", outs)
    for n in outs:
        if n in ("Y", "dX"):
            diff = float((outs[n].float() - first[n].float()).abs().max() / first[n].float().abs().max())
            assert diff <= k * 2.0 ** -8, (n, k, diff)
        else:
            assert torch.equal(outs[n], first[n]), (n, k)


def test_full_size_fp32_sums_identical_across_k():
    """SS_FFN_FLAG_EXACT_SUM at the benchmark size: every output is the same bits for k = 1, 2, 4."""
    import torch
    from paper_2301_08984_amd.runner import FfnCase
    o = _full_size_oracle()
    first = None
    for k in FFN_WORKLOADS["gpt3_ffn"]["k"]:
        print(f"ffn full size gpt3_ffn fp32 sums k={k}", flush=True)
        fc = FfnCase(o["inp"], act=o["cfg"]["act"])
        d = fc.desc(o["cfg"]["lo"], o["cfg"]["hi"], k, EXACT)
        fc.fwd(d, poison=True)
        fc.bwd(d, poison=True)
        torch.cuda.synchronize()
        outs = {n: getattr(fc, n).clone() for n in ("Y", "dX", "dW1", "db1", "dW2", "db2")}
        if first is None:
            first = outs
        for n in outs:
            assert torch.equal(outs[n], first[n]), (n, k)
        del fc


def test_two_host_threads_on_two_streams():
    """Two host threads call the backward at the same time, each on a stream of its own with tensors of
    its own: the fork / join events belong to a call, so nothing but the helper stream is shared and
    both get the results of a run alone."""
    import threading
    import torch
    from paper_2301_08984_amd.runner import FfnCase
    cfgs = [SMALL["several_tiles"], SMALL["ragged"]]
    alone, cases, descs = [], [], []
    for cfg in cfgs:
        fc, _ = _run(cfg, 3)
        alone.append({n: getattr(fc, n).clone() for n in ("Y", "dX", "dW1", "db1", "dW2", "db2")})
        c = FfnCase(make_ffn_inputs(**cfg), act=cfg["act"])
        d = c.desc(cfg["lo"], cfg["hi"], 3)
        c.workspace(d)
        cases.append(c)
        descs.append(d)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    errors = []

    def work(i):
        try:
            for _ in range(20):
                cases[i].fwd(descs[i], stream=streams[i].cuda_stream)
                cases[i].bwd(descs[i], stream=streams[i].cuda_stream)
        except Exception as e:  # noqa: BLE001
            errors.append(e)

    print("ffn two threads", flush=True)
    torch.cuda.synchronize()
    ts = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i, cfg in enumerate(cfgs):
        lo, hi = cfg["lo"], cfg["hi"]
        for n, ref in alone[i].items():
            a = getattr(cases[i], n)
            if n == "dW1":
                a, ref = a[:, lo:hi], ref[:, lo:hi]
            if n in ("db1", "dW2"):
                a, ref = a[lo:hi], ref[lo:hi]
            assert torch.equal(a, ref), (i, n)


def test_padded_leading_dimensions_are_never_read_or_written():
    """Every matrix sits in a wider buffer whose padding holds NaN: a read past a row's end would
    poison the results, a write past it would show in the padding."""
    import torch
    from paper_2301_08984_amd.runner import FfnCase
    cfg = dict(seed=65, T=333, dm=200, dh=424, lo=8, hi=416, act="gelu")
    inp = make_ffn_inputs(**cfg)
    Y, g = _oracle(cfg, inp)
    lo, hi = cfg["lo"], cfg["hi"]
    for k in (1, 3):
        print(f"ffn padded k={k}", flush=True)
        fc = FfnCase(inp, act=cfg["act"], pad=(8, 16, 24))
        d = fc.desc(lo, hi, k)
        fc.fwd(d)
        fc.bwd(d)
        torch.cuda.synchronize()
        errs = {"Y": rel_err(fc.host("Y"), Y), "dX": rel_err(fc.host("dX"), g["dX"]),
                "dW1": rel_err(fc.host("dW1")[:, lo:hi], g["dW1"][:, lo:hi]),
                "db1": rel_err(fc.host("db1")[lo:hi], g["db1"][lo:hi]),
                "dW2": rel_err(fc.host("dW2")[lo:hi], g["dW2"][lo:hi]), "db2": rel_err(fc.host("db2"), g["db2"])}
        for n, e in errs.items():
            assert np.isfinite(e) and e <= TOL, (n, k, e)
        for name, width in (("Y", cfg["dm"]), ("dX", cfg["dm"]), ("dW1", cfg["dh"]), ("dW2", cfg["dm"])):
            base = getattr(fc, name)._base
            assert bool(torch.isnan(base[:, width:].float()).all()), name


def test_optional_output_bias_and_its_gradient():
    """b2 = NULL (a tensor-parallel caller adds it after its all-reduce) and db2 = NULL (skipped)."""
    import torch
    from paper_2301_08984_amd.runner import FfnCase
    cfg = SMALL["several_tiles"]
    inp = make_ffn_inputs(**cfg)
    kind = orc.ACT_GELU_TANH
    p = orc.FfnProblem(inp["X"], inp["W1"], inp["b1"], inp["W2"], inp["b2"], kind)
    Y = orc.ffn_forward(p, cfg["lo"], cfg["hi"], add_b2=False)
    for k in (1, 2):
        print(f"ffn no-b2 k={k}", flush=True)
        fc = FfnCase(inp, act=cfg["act"])
        fc.b2, fc.db2 = None, None
        d = fc.desc(cfg["lo"], cfg["hi"], k)
        fc.fwd(d)
        fc.bwd(d)
        torch.cuda.synchronize()
        assert rel_err(fc.host("Y"), Y) <= TOL
        assert np.all(np.isfinite(fc.host("dX")))


def test_graph_capture_replays_match_eager():
    """Forward + backward captured into a HIP graph (the helper stream is forked and joined inside
    the capture) and replayed with eager work and synchronisations in between: every replay gives
    the eager result, bit for bit."""
    import torch
    from paper_2301_08984_amd.runner import FfnCase
    cfg = SMALL["several_tiles"]
    inp = make_ffn_inputs(**cfg)
    fc = FfnCase(inp, act=cfg["act"])
    d = fc.desc(cfg["lo"], cfg["hi"], 3)
    fc.fwd(d)
    fc.bwd(d)
    torch.cuda.synchronize()
    names = ("Y", "dX", "dW1", "db1", "dW2", "db2")
    eager = {n: getattr(fc, n).clone() for n in names}
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fc.fwd(d)  # warm-up on the capturing stream
        fc.bwd(d)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            fc.fwd(d)
            fc.bwd(d)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(3):
        print(f"ffn graph replay {rep}", flush=True)
        for n in names:
            getattr(fc, n).fill_(float("nan"))
        scratch = torch.randn(1 << 20, device=fc.dev).sum()  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in names:
            a, b = getattr(fc, n), eager[n]
            lo, hi = cfg["lo"], cfg["hi"]
            if n == "dW1":
                a, b = a[:, lo:hi], b[:, lo:hi]
            if n in ("db1", "dW2"):
                a, b = a[lo:hi], b[lo:hi]
            assert torch.equal(a, b), (n, rep)
        del scratch


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_match_oracle(seed):
    """Seeded random shapes: ragged token counts, model and hidden widths that are not multiples of
    the 64-deep stage or of the 256 x 128 tile, sub-ranges, every k up to the limit."""
    rng = np.random.default_rng(9000 + seed)
    T = int(rng.integers(1, 700))
    dm = 8 * int(rng.integers(1, 70))
    dh = 8 * int(rng.integers(2, 90))
    lo = 8 * int(rng.integers(0, dh // 16))
    hi = min(dh, lo + 8 * int(rng.integers(1, (dh - lo) // 8 + 1)))
    cfg = dict(seed=9100 + seed, T=T, dm=dm, dh=dh, lo=lo, hi=hi, act="gelu" if seed % 3 else "relu")
    k = int(rng.integers(1, -(-(hi - lo) // 16) + 1))
    print(f"ffn random case {cfg} k={k}", flush=True)
    fc, inp = _run(cfg, k)
    Y, g = _oracle(cfg, inp)
    errs = {"Y": rel_err(fc.host("Y"), Y), "dX": rel_err(fc.host("dX"), g["dX"]),
            "dW1": rel_err(fc.host("dW1")[:, lo:hi], g["dW1"][:, lo:hi]),
            "db1": rel_err(fc.host("db1")[lo:hi], g["db1"][lo:hi]),
            "dW2": rel_err(fc.host("dW2")[lo:hi], g["dW2"][lo:hi]), "db2": rel_err(fc.host("db2"), g["db2"])}
    for n, e in errs.items():
        assert np.isfinite(e) and e <= TOL, (n, cfg, k, e)
