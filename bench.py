#!/usr/bin/env python3
"""Benchmark of the co-sharded attention hot path on one MI355X.

One step = ss_attn_fwd + ss_attn_bwd over the whole share of one workload at one
co-shard factor k (all k chunks, one stream).  Inputs are seeded synthetic
tensors already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gpt3_shard] [--k 2]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_BF16 = 2.5e15  # dense bf16 FLOP/s, MI355X
PEAK_HBM = 8.0e12        # B/s
# Vector-ALU peak in lane-operations per second: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz (one
# fp32 instruction of a 64-wide wavefront occupies its SIMD for 4 cycles).  This is half of the 78.6
# TFLOP/s fp32 vector figure (which counts an fma as two flops) and a quarter of 157.3 (packed fp32,
# which this build does not emit); transcendental instructions (exp2, rcp) run at a quarter of it.
PEAK_VALU_LANEOPS = 256 * 64 * 2.4e9
# which roofline bounds the dominant kernel of each workload: the D = 128 shapes are matrix-core
# work; at D = 32 a score element costs 2-3 matrix steps but the same softmax arithmetic, so the vector
# ALUs (exp2 above all) bind and the HBM fraction is reported beside it; the window shape moves its
# activations in 64-byte pieces and is nearest to the HBM roof
BOUND = {"gpt3_shard": "mfma", "gpt3_long": "mfma", "gpt3_long_16k": "mfma", "swin_window": "hbm", "af2_msa_row": "alu", "af2_triangle": "alu",
         "af2_msa_col": "alu", "af2_triangle_end": "alu", "tiny_mha": "hbm"}
# Contractions (each 2*D flop per visible score element) of the METHOD that a kernel stands for: the
# forward has 2 (scores, value product), the backward 5 (scores, dP, dV, dK, dQ); where the backward
# is two kernels the scores and dP are counted once, half with each; the recompute pass and the score
# recompute of the bias-gradient kernel are not part of the method's count.
CONTRACTIONS = {"fwd": 2, "recompute": 0, "dq": 2, "dkdv": 3, "dbias": 0, "table_reduce": 0, "dq_dkdv": 5,
                "dbias_fold": 0, "recompute_dq": 2}
# contractions a kernel actually executes on the matrix cores (scores and dP are formed again by
# every kernel that needs them)
EXECUTED = {"fwd": 2, "recompute": 2, "dq": 3, "dkdv": 4, "dbias": 2, "table_reduce": 0, "dq_dkdv": 8,
            "dbias_fold": 0, "recompute_dq": 5}
# ("dq_dkdv": the one-gradient-per-work-group launch forms the scores three times and dP twice: 3 + 2 + 3;
# "recompute_dq": scores, dP, the value product and the two products that combine into dQ)


def executed_table(w):
    """EXECUTED for this workload: at head size 128 without a bias the separate dK/dV launch of the
    large shares is one gradient per work-group too and forms the scores twice (3 + 2)."""
    t = dict(EXECUTED)
    if w["D"] == 128 and w["bias"] is None:
        t["dkdv"] = 5
    return t

# Vector-ALU lane-operations per visible score element that the method needs at least, quarter-rate
# instructions counted as 4: forward = scale/bias fma 1 + running max 1 + exp2 4 + row sum 1 + bf16
# conversion 1 = 8; backward = score fma 1 + exp2 4 + (dP - Delta) 1 + times P 1 + two conversions 2
# = 9, + 1 for the bias-gradient addition.  Recomputation is not counted.
VALU_SLOTS = {"fwd": 8, "recompute": 0, "dq": 4.5, "dkdv": 4.5, "dbias": 1, "table_reduce": 0, "dq_dkdv": 9,
              "dbias_fold": 0, "recompute_dq": 4.5}


def choose_steps(a, step):
    """Default step counts: the clocks of an idle GPU take some 20 ms of load to settle (the GPT share reads
    0.164 ms per step after 10 warm-up steps and 0.147 ms after 100), so the default warm-up and the
    default timed region are each about 0.15 s of steps, between 20 and 500 of them."""
    import torch
    if a.steps is not None and a.warmup is not None:
        return
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        step()
    torch.cuda.synchronize()
    n = int(0.15 / max((time.perf_counter() - t0) / 3, 1e-6))
    n = min(500, max(20, n))
    if a.steps is None:
        a.steps = n
    if a.warmup is None:
        a.warmup = n


def visible_fraction(w):
    return 0.5 if w["mask"] == "causal" else 1.0


def job_flops(w):
    """fwd+bwd algorithmic flop of the whole share: 14*E*D, half under a causal mask."""
    E = w["B"] * w["H"] * w["S"] ** 2
    return 14.0 * E * w["D"] * visible_fraction(w)


def kernel_flops(w, name, units, axis_extent, table=CONTRACTIONS):
    E = w["B"] * w["H"] * w["S"] ** 2 * (units / axis_extent)
    return 2.0 * table[name] * E * w["D"] * visible_fraction(w)


def kernel_laneops(w, name, units, axis_extent):
    E = w["B"] * w["H"] * w["S"] ** 2 * (units / axis_extent) * visible_fraction(w)
    return VALU_SLOTS[name] * E


def kernel_bytes(w, name, units, axis_extent):
    """Bytes a kernel must move once per launch: its activation tensors plus bias."""
    es = 2 if w["dtype"] == "bf16" else 4
    T = w["B"] * w["H"] * w["S"] * w["D"] * es * (units / axis_extent)
    g = 1 if w["gated"] else 0
    nb = 0
    if w["bias"] == "dense":
        nb = w["H"] * w["S"] ** 2 * es
    elif w["bias"] == "relpos":
        nb = w["H"] * 169 * es
    stat = w["B"] * w["H"] * w["S"] * 4 * (units / axis_extent)
    table = {
        "fwd": (4 + g) * T + nb + stat,
        "recompute": (4 + g) * T + 2 * g * T + nb + 2 * stat,
        "dq": 5 * T + nb + 2 * stat,
        "dkdv": 6 * T + nb + 2 * stat,
        "dq_dkdv": 7 * T + nb + 2 * stat,
        "recompute_dq": (5 + g) * T + 2 * g * T + nb + 2 * stat,
        "dbias": 4 * T + nb + 2 * stat + (w["H"] * w["S"] ** 2 * 4 if w["bias"] else 0),
        "table_reduce": w["H"] * w["S"] ** 2 * 4,
        "dbias_fold": 3 * w["H"] * w["S"] ** 2 * 4,
    }
    return table[name]


def cpu_baseline(w, budget_s=15.0):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload."""
    from oracle import attention as orc
    from paper_2301_08984_amd.workloads import make_inputs
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from parity import oracle_problem
    axis = orc.AXIS_HEAD if w["axis"] == "head" else orc.AXIS_ROW
    ext = w["H"] if w["axis"] == "head" else w["B"]
    rows = None if w["axis"] == "head" else (0, min(ext, 64))
    small = dict(w)
    if rows is not None:
        small["B"] = rows[1]
    inp = make_inputs(**small, rows=rows)
    p = oracle_problem(inp, small)
    dY = inp["dY"].astype(np.float64)
    avail = small["H"] if w["axis"] == "head" else small["B"]

    def run(n):
        t0 = time.perf_counter()
        orc.coshard_forward(p, axis, 0, n, 1)
        orc.coshard_backward(p, dY, axis, 0, n, 1)
        return time.perf_counter() - t0

    t1 = run(1)
    n = int(max(1, min(avail, budget_s / max(t1, 1e-4))))
    t = run(n) if n > 1 else t1
    flops = job_flops(w) * n / ext
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        threads = 1
    threads = min(threads, len(os.sched_getaffinity(0)))
    unit = "heads" if w["axis"] == "head" else "rows"
    return {"value": flops / t / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} of {ext} {unit} of {w['name']} (fwd+bwd, fp64 numpy), {t:.2f} s",
            "seconds": t}


def ffn_cpu_baseline(w, budget_s=15.0):
    """The fp64 feed-forward oracle on a bounded sample of the workload's tokens."""
    from oracle import ffn as orc
    from paper_2301_08984_amd.workloads import make_ffn_inputs
    inp = make_ffn_inputs(**w)
    kind = orc.ACT_GELU_TANH if w["act"] == "gelu" else orc.ACT_RELU

    def run(nt):
        p = orc.FfnProblem(inp["X"][:nt], inp["W1"], inp["b1"], inp["W2"], inp["b2"], kind)
        t0 = time.perf_counter()
        orc.coshard_forward(p, w["lo"], w["hi"], 1)
        orc.coshard_backward(p, inp["dY"][:nt].astype(np.float64), w["lo"], w["hi"], 1)
        return time.perf_counter() - t0

    t1 = run(16)
    nt = int(max(16, min(w["T"], 16 * budget_s / max(t1, 1e-4))))
    t = run(nt)
    flops = 12.0 * nt * w["dm"] * (w["hi"] - w["lo"])
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        threads = 1
    threads = min(threads, len(os.sched_getaffinity(0)))
    return {"value": flops / t / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"{nt} of {w['T']} tokens of {w['name']} (fwd+bwd, fp64 numpy), {t:.2f} s", "seconds": t}


def ffn_main(a):
    """Co-sharded feed-forward: one step = ss_ffn_fwd + ss_ffn_bwd over the whole hidden share."""
    import torch
    from paper_2301_08984_amd import ffn_binding as fb
    from paper_2301_08984_amd.runner import FfnCase
    from paper_2301_08984_amd.workloads import FFN_WORKLOADS, make_ffn_inputs

    w = dict(FFN_WORKLOADS[a.workload], name=a.workload)
    ks = list(w["k"])
    k_main = a.k if a.k is not None else (ks[1] if len(ks) > 1 else ks[0])
    fb.lib()
    fc = FfnCase(make_ffn_inputs(**w), act=w["act"], fill=0.0)
    nh = w["hi"] - w["lo"]
    flops = 12.0 * w["T"] * w["dm"] * nh   # six products of 2*T*dm*nh (two forward, four backward; recompute not counted)
    desc = fc.desc(w["lo"], w["hi"], k_main)

    def step(d):
        fc.fwd(d)
        fc.bwd(d)

    if a.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=fc.dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    choose_steps(a, lambda: step(desc))
    for _ in range(a.warmup):
        step(desc)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(desc)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / a.steps * 1e3
    value = flops / (ms * 1e-3) / 1e12
    # second pass with an event after every step, for the spread (see the attention path)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(a.steps + 1)]
    marks[0].record()
    for i in range(a.steps):
        step(desc)
        marks[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(a.steps))
    out = {"metric": "feed-forward fwd+bwd TFLOP/s (1 GPU) + % MFMA peak; peak HBM bytes vs co-shard k",
           "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": a.workload, "T": w["T"], "d_model": w["dm"], "hidden_share": nh, "act": w["act"],
                      "k": k_main},
           "pct_mfma_peak": 100.0 * value * 1e12 / PEAK_MFMA_BF16,
           "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0]}
    if not a.no_extras:
        fb.ss_ffn_profile_enable(True)
        for _ in range(a.steps):
            step(desc)
        torch.cuda.synchronize()
        fb.ss_ffn_profile_enable(False)
        per_kernel = {}
        for kid, name in enumerate(fb.KERNEL_NAMES):
            tot, n = fb.ss_ffn_profile_read(kid)
            if n:
                per_kernel[name] = {"avg_us": tot / n * 1e3, "launches_per_step": n / a.steps, "ms_per_step": tot / a.steps}
        dom = max(per_kernel, key=lambda n: per_kernel[n]["ms_per_step"])
        # every product of a chunk is 2*T*dm*(nh/k) flop; `up` runs twice per step (forward and recompute)
        ach = 2.0 * w["T"] * w["dm"] * (nh / k_main) / (per_kernel[dom]["avg_us"] * 1e-6) / 1e12
        out["roofline"] = {"bound": "mfma", "achieved": ach, "peak": PEAK_MFMA_BF16 / 1e12, "unit": "TFLOP/s",
                           "frac": ach * 1e12 / PEAK_MFMA_BF16, "traffic": None, "kernel": dom,
                           "avg_launch_us": per_kernel[dom]["avg_us"]}
        try:
            with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as fh:
                out["roofline"]["traffic"] = json.load(fh).get(a.workload, {}).get(dom)
        except OSError:
            pass
        out["kernels"] = per_kernel
        table = []
        caller = fc.caller_bytes()
        for k in ([] if a.no_per_k else sorted(set(ks) | {k_main})):
            d = fc.desc(w["lo"], w["hi"], k)
            fwd_b, bwd_b = fb.ss_ffn_workspace_bytes(d)
            for _ in range(2):
                step(d)
            torch.cuda.synchronize()
            n = max(3, a.steps // 5)
            t0 = time.perf_counter()
            for _ in range(n):
                step(d)
            torch.cuda.synchronize()
            t = (time.perf_counter() - t0) / n
            table.append({"k": k, "ms_per_step": t * 1e3, "tflops": flops / t / 1e12, "workspace_bytes": max(fwd_b, bwd_b),
                          "peak_hbm_bytes": caller + max(fwd_b, bwd_b),
                          "hidden_activation_bytes_per_chunk": int(2 * w["T"] * -(-nh // k) * 2)})
        out["per_k"] = table
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = ffn_cpu_baseline(w)
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default: about 0.15 s of them, between 20 and 500)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default: as many)")
    ap.add_argument("--workload", default="gpt3_shard")
    ap.add_argument("--k", type=int, default=None, help="co-shard factor of the timed steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the per-k table and the instrumented pass")
    ap.add_argument("--no-per-k", action="store_true", help="skip the table over the workload's other k")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 1 GiB read + 1 GiB write elementwise kernel (known size, to scale rocprofv3 counters by)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding across GPUs); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2301_08984_amd import binding as ss
    from paper_2301_08984_amd.runner import DeviceCase
    from paper_2301_08984_amd.workloads import FFN_WORKLOADS, WORKLOADS, make_inputs

    if a.workload in FFN_WORKLOADS:
        return ffn_main(a)
    w = dict(WORKLOADS[a.workload], name=a.workload)
    ext = w["H"] if w["axis"] == "head" else w["B"]
    ks = list(w["k"])
    k_main = a.k if a.k is not None else (ks[1] if len(ks) > 1 else ks[0])
    ss.lib()  # fail loudly if the HIP library is missing
    host_inputs = make_inputs(**w)
    torch.zeros(1, device="cuda:0")   # context and allocator set up before the first memory reading
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    dc = DeviceCase(host_inputs, dtype=w["dtype"], bias=w["bias"], mask=w["mask"], gated=w["gated"],
                    win=w.get("win"), fill=0.0, layout=w.get("layout", "bshd"))
    del host_inputs
    torch.cuda.synchronize()
    torch.cuda.empty_cache()   # staging copies of the upload go back to the driver
    caller_measured = free0 - torch.cuda.mem_get_info()[0]
    desc = dc.desc(w["axis"], 0, ext, k_main)
    family = ss.ss_attn_kernel_family(desc)
    dc.workspace(desc)

    def step(d):
        dc.fwd(d, want_lse=False)
        dc.bwd(d)

    if a.calibration_copy:
        # a plain streaming kernel of known size: reads 1 GiB, writes 1 GiB
        src = torch.ones(1 << 28, dtype=torch.float32, device=dc.dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    choose_steps(a, lambda: step(desc))
    for _ in range(a.warmup):
        step(desc)
    torch.cuda.synchronize()
    # the timed region: exactly K steps between two synchronisations, nothing else on the stream
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(desc)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt / a.steps * 1e3
    value = job_flops(w) / (ms * 1e-3) / 1e12
    # a second pass over K steps with an event after every step, for the spread (the library enqueues on
    # torch's current stream, so events recorded there bracket each step)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(a.steps + 1)]
    marks[0].record()
    for i in range(a.steps):
        step(desc)
        marks[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(a.steps))

    out = {
        "metric": "attn fwd+bwd TFLOP/s (1 GPU) + % MFMA peak; peak HBM bytes vs co-shard k",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w["dtype"], "data": "synthetic",
        "config": {"workload": a.workload, "B": w["B"], "H": w["H"], "S": w["S"], "D": w["D"],
                   "layout": w.get("layout", "bshd"),
                   "bias": w["bias"], "mask": w["mask"], "gated": w["gated"], "shard_axis": w["axis"],
                   "k": k_main, "kernels": family},
        "pct_mfma_peak": 100.0 * value * 1e12 / PEAK_MFMA_BF16,
        # per-step durations between events on the launch stream, from the second pass (the value above is
        # wall clock over the K steps of the timed region)
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
    }

    if not a.no_extras:
        # instrumented pass over the same K steps: HIP events around every kernel launch
        ss.ss_attn_profile_enable(True)
        for _ in range(a.steps):
            step(desc)
        torch.cuda.synchronize()
        ss.ss_attn_profile_enable(False)
        per_kernel = {}
        for kid, name in enumerate(ss.KERNEL_NAMES):
            tot, n = ss.ss_attn_profile_read(kid)
            if n:
                per_kernel[name] = {"avg_us": tot / n * 1e3, "launches_per_step": n / a.steps,
                                    "ms_per_step": tot / a.steps}
        dom = max(per_kernel, key=lambda n: per_kernel[n]["ms_per_step"])
        units = ext / k_main
        dur = per_kernel[dom]["avg_us"] * 1e-6
        gbs = kernel_bytes(w, dom, units, ext) / dur / 1e9
        tfs = kernel_flops(w, dom, units, ext) / dur / 1e12
        if BOUND[a.workload] == "mfma":
            roof = {"bound": "mfma", "achieved": tfs, "peak": PEAK_MFMA_BF16 / 1e12, "unit": "TFLOP/s",
                    "frac": tfs * 1e12 / PEAK_MFMA_BF16, "traffic": None}
        elif BOUND[a.workload] == "alu":
            ach = kernel_laneops(w, dom, units, ext) / dur / 1e12
            roof = {"bound": "alu", "achieved": ach, "peak": PEAK_VALU_LANEOPS / 1e12, "unit": "Tlane-op/s",
                    "frac": ach * 1e12 / PEAK_VALU_LANEOPS, "traffic": None}
        else:
            roof = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                    "frac": gbs * 1e9 / PEAK_HBM, "traffic": None}
        # the other two fractions of the same kernel, for context: algorithmic bytes against HBM, the
        # method's contractions against the matrix cores, and the contractions the kernel executes
        roof["hbm_frac"] = gbs * 1e9 / PEAK_HBM
        roof["mfma_frac"] = tfs * 1e12 / PEAK_MFMA_BF16
        roof["mfma_issue_frac"] = kernel_flops(w, dom, units, ext, executed_table(w)) / dur / PEAK_MFMA_BF16
        # HBM bytes per launch of that kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
        # same command (calibrated by a known-size copy), recorded under profiles/
        try:
            with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as fh:
                roof["traffic"] = json.load(fh).get(a.workload, {}).get(dom)
        except OSError:
            pass
        roof["kernel"] = dom
        roof["avg_launch_us"] = per_kernel[dom]["avg_us"]
        out["roofline"] = roof
        out["kernels"] = per_kernel

        # throughput, workspace and peak HBM bytes for every co-shard factor of the workload
        # "measured" = what hipMemGetInfo (through torch) says the device lost: the caller tensors once, the
        # workspace per k (allocated alone after the allocator's cache was emptied; the allocator
        # rounds blocks up, 2 MiB granularity for large ones, so the reading sits a little above the exact figure)
        table = []
        caller = dc.caller_bytes()
        for k in ([] if a.no_per_k else sorted(set(ks) | {k_main})):
            d = dc.desc(w["axis"], 0, ext, k)
            _, wsb = ss.ss_attn_workspace_bytes(d)
            dc.ws = None
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
            f0 = torch.cuda.mem_get_info()[0]
            dc.workspace(d)
            for _ in range(3):
                step(d)
            torch.cuda.synchronize()
            ws_measured = f0 - torch.cuda.mem_get_info()[0]
            n = max(5, a.steps // 5)
            t0 = time.perf_counter()
            for _ in range(n):
                step(d)
            torch.cuda.synchronize()
            t = (time.perf_counter() - t0) / n
            chunk_units = -(-ext // k)
            sxs = chunk_units * (w["B"] * w["H"] / ext) * w["S"] ** 2 * 2
            table.append({"k": k, "ms_per_step": t * 1e3, "tflops": job_flops(w) / t / 1e12,
                          "workspace_bytes": wsb, "peak_hbm_bytes": caller + wsb,
                          "measured_peak_hbm_bytes": caller_measured + ws_measured,
                          "unfused_scores_bytes_per_chunk": int(sxs)})
        out["per_k"] = table

    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
