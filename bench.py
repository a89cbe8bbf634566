#!/usr/bin/env python3
"""Benchmark of the MoE layer hot path on one MI355X.

A step is one pass of the whole path -- moe_plan + moe_forward + moe_backward -- over one batch
of synthetic input that is already resident in HBM.  Protocol as in the paper's Section 5.1:
warm-up rounds that are not counted, then the timed runs (16 by default), mean time.

Prints ONE JSON line: whole-step throughput in tokens/s (`value`), the roofline of the dominant
kernel (the grouped matrix product, timed per launch with HIP events on the launch stream in a
second pass of the same number of steps) and the CPU oracle timed on a bounded token sample.
"""
import argparse
import json
import sys
import time

import numpy as np

METRIC = "MoE layer fwd+bwd tokens/sec and grouped-GEMM % of bf16 MFMA peak, 1 GPU"
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3      # vector fp32 (the fp32 workload does not use the matrix cores)
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="C1", help="C0..C4 (C1 is the configuration the metric is quoted on)")
    ap.add_argument("--custom", default=None, metavar="N,d,h,E,k[,zipf_s]",
                    help="a bf16 layer of another shape (sweeps of experts / rows per expert); overrides --workload")
    ap.add_argument("--cpu-sample-tokens", type=int, default=-1, help="tokens of the oracle sample (0: skip)")
    ap.add_argument("--sweep-experts", default=None, metavar="E1,E2,...",
                    help="the paper's single-GPU experiment (Section 5.2, computation time against the number of "
                         "experts at n_b=4096, d_m=1024, d_h=4096, k=2): one JSON line per expert count with the "
                         "forward and backward times; replaces the default output")
    ap.add_argument("--sweep-rows", default=None, metavar="N1,N2,...",
                    help="throughput of the grouped matrix products against the batch an expert sees (the paper's "
                         "Section 4 figure of GeMM throughput against problem size): token counts at d_m=1024, "
                         "d_h=4096, 16 experts, k=2, i.e. N/8 rows per expert; one JSON line per count")
    ap.add_argument("--calibrate-hbm-counters", type=int, default=0, metavar="MiB",
                    help="no benchmark: a plain device copy of this many MiB, five times, for scaling rocprofv3's FETCH_SIZE / "
                         "WRITE_SIZE (run under `rocprofv3 --pmc FETCH_SIZE`, then WRITE_SIZE: the copy kernel moves exactly that "
                         "many MiB in and out per launch, so counter / (MiB * 1024) is the factor by which the counter over- or "
                         "under-reports KiB on this machine; use a size above the 256 MB Infinity Cache, e.g. 1024)")
    ap.add_argument("--library-gemm", action="store_true",
                    help="context only: the rate of the vendor library's dense bf16 product (torch.matmul) on the six "
                         "product shapes of the workload with equal experts, i.e. what a tuned plain GEMM reaches on "
                         "this machine where the grouped kernel reaches roofline.achieved; one JSON line per shape")
    return ap.parse_args()


def cpu_baseline(w, inputs, n_tokens):
    """The fp64 oracle, as it stands, on a seeded token sample of the same workload."""
    import oracle as orc
    from oracle.build import build_oracle

    build_oracle(force=False)
    bg = inputs["bg"].astype(np.float64)
    p = orc.OracleProblem(inputs["X"], inputs["Wg"], inputs["W1"], inputs["W2"], w.k, bg=bg, dY=inputs["dY"])
    toks = np.sort(np.random.default_rng(w.seed).choice(w.N, size=min(n_tokens, w.N), replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    orc.layer(p, tokens=toks)
    dt = time.perf_counter() - t0
    return {"value": toks.size / dt, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{toks.size} of {w.N} tokens of {w.name} (seeded subset), full forward+backward incl. all "
                      f"weight gradients, {dt:.1f} s"}


def measured_hbm_bytes_per_gemm_launch(workload):
    """HBM bytes per grouped-GEMM launch (mean over the launches of a step), from the tracked summary of two
    rocprofv3 --pmc runs of this file (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter reads for a
    plain 1 GiB copy: profiles/<workload>_hbm_traffic_pmc.md holds the commands, the per-kernel figures and the line
    `grouped_gemm_hbm_bytes_per_launch = <bytes>` that is read here.  Counters cannot be read from inside a run, so
    this is the stored measurement, not a live one; None if there is no summary for the workload."""
    import os
    import re

    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"{workload}_hbm_traffic_pmc.md")
    try:
        m = re.search(r"^grouped_gemm_hbm_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(path).read(), re.M)
    except OSError:
        return None
    return float(m.group(1)) if m else None


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (all experts local, no collectives); --gpus {a.gpus} is not "
              "supported", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2103_13262_amd import binding as B
    from paper_2103_13262_amd.synth import WORKLOADS, make_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if a.calibrate_hbm_counters:
        src = torch.empty(a.calibrate_hbm_counters << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration_copy_mib": a.calibrate_hbm_counters, "launches": 5}))
        return
    B.lib()   # raises if the HIP library has not been built: there is no fallback
    if a.sweep_experts:
        for E in (int(v) for v in a.sweep_experts.split(",")):
            a.custom, a.cpu_sample_tokens = f"4096,1024,4096,{E},2", 0
            out = run(a, torch, B, WORKLOADS, make_inputs)
            kt = {n: v["avg_us"] * v["launches_per_step"] for n, v in out["kernels"].items()}
            fwd = sum(kt.get(n, 0.0) for n in ("ggemm_fc1_gelu", "ggemm_fc2", "combine"))
            plan = sum(kt.get(n, 0.0) for n in ("gate_topk", "plan"))
            print(json.dumps({"sweep": "experts", "n_b": 4096, "d_m": 1024, "d_h": 4096, "k": 2, "n_e": E,
                              "ms_per_step": out["ms_per_step"], "gate_and_plan_ms": plan / 1e3, "forward_ms": fwd / 1e3,
                              "backward_ms": (sum(kt.values()) - fwd - plan) / 1e3, "tokens_per_s": out["value"],
                              "grouped_gemm_tflops": out["roofline"]["achieved"]}), flush=True)
            torch.cuda.empty_cache()
        return
    if a.sweep_rows:
        for N in (int(v) for v in a.sweep_rows.split(",")):
            a.custom, a.cpu_sample_tokens = f"{N},1024,4096,16,2", 0
            out = run(a, torch, B, WORKLOADS, make_inputs)
            print(json.dumps({"sweep": "rows", "d_m": 1024, "d_h": 4096, "n_e": 16, "k": 2, "n_b": N,
                              "rows_per_expert": N * 2 / 16, "ms_per_step": out["ms_per_step"],
                              "tokens_per_s": out["value"], "grouped_gemm_tflops": out["roofline"]["achieved"],
                              "grouped_gemm_avg_launch_us": out["roofline"]["avg_launch_us"]}), flush=True)
            torch.cuda.empty_cache()
        return
    if a.library_gemm:
        w = WORKLOADS[a.workload]
        M = w.N * w.k
        # (rows, columns, reduction) of FC1 / dH, FC2 / dXs and of the two weight gradients taken over all rows at once
        for name, (m, n, kk) in (("fc1", (M, w.h, w.d)), ("fc2", (M, w.d, w.h)), ("dw1_all_rows", (w.d, w.h, M)),
                                 ("dw2_all_rows", (w.h, w.d, M))):
            x = torch.randn(m, kk, device="cuda:0", dtype=torch.bfloat16)
            y = torch.randn(kk, n, device="cuda:0", dtype=torch.bfloat16)
            for _ in range(a.warmup):
                x @ y
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(a.steps):
                x @ y
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / a.steps * 1e3
            print(json.dumps({"library_gemm": name, "workload": w.name, "m": m, "n": n, "k": kk, "us": us,
                              "tflops": 2.0 * m * n * kk / us / 1e6}), flush=True)
        return
    print(json.dumps(run(a, torch, B, WORKLOADS, make_inputs)))


def run(a, torch, B, WORKLOADS, make_inputs):
    w = WORKLOADS[a.workload]
    if a.custom:
        from paper_2103_13262_amd.synth import Workload
        f = a.custom.split(",")
        w = Workload("custom", int(f[0]), int(f[1]), int(f[2]), int(f[3]), int(f[4]), "bf16",
                     float(f[5]) if len(f) > 5 else 0.0, 20210313 * 10 + 9)
    inputs = make_inputs(w)
    dev = torch.device("cuda:0")
    bf = w.dtype == "bf16"
    dt = B.MOE_BF16 if bf else B.MOE_F32

    def up(x):
        if bf:
            return torch.from_numpy(x.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(x).to(dev)

    X, Wg, W1, W2, dY = (up(inputs[n]) for n in ("X", "Wg", "W1", "W2", "dY"))
    bg = torch.from_numpy(inputs["bg"]).to(dev)
    desc = B.make_desc(w.N, w.d, w.h, w.E, w.k, dt, dt, 0)
    buf = B.MoeLayerBuffers(desc, dev)
    act = torch.bfloat16 if bf else torch.float32
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    dWg, dW1, dW2 = torch.empty_like(Wg), torch.empty_like(W1), torch.empty_like(W2)
    dbg = torch.empty(max(w.E, 4), dtype=torch.float32, device=dev)
    stream = buf.stream()

    def step():
        B.moe_plan(desc, X, Wg, bg, buf.plan, buf.workspace, buf.ws_bytes, stream)
        B.moe_forward(desc, buf.plan, X, W1, W2, None, None, Y, buf.workspace, buf.ws_bytes, stream)
        B.moe_backward(desc, buf.plan, X, Wg, W1, W2, dY, dX, dWg, dbg, dW1, dW2, buf.workspace, buf.ws_bytes, stream)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / a.steps

    # second pass of the same steps with per-kernel HIP events (recorded on the launch stream)
    B.moe_profile_enable(True)
    for _ in range(a.steps):
        step()
    prof = B.moe_profile_read()
    B.moe_profile_enable(False)

    flops_product = 2.0 * w.M * w.d * w.h                    # one grouped product: 2 M d h
    kern = {n: {"launches_per_step": c / a.steps, "avg_us": 1e3 * t / c} for n, (c, t) in prof.items()}
    gemm = {n: v for n, v in prof.items() if n.startswith("ggemm_")}
    products = {n: 2 if "+" in n else 1 for n in gemm}       # the bf16 backward runs two products per launch
    g_launches = sum(c for c, _ in gemm.values())
    g_ms = sum(t for _, t in gemm.values())
    avg_launch_ms = g_ms / g_launches
    flops_launch = flops_product * sum(products[n] * c for n, (c, _) in gemm.items()) / g_launches   # mean per launch
    achieved = flops_launch / (avg_launch_ms * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if bf else PEAK_FP32_TFLOPS
    for n, (c, t) in gemm.items():
        kern[n]["tflops"] = products[n] * flops_product / (t / c * 1e-3) / 1e12
    # the data-movement kernels against the HBM roofline: algorithmic bytes per launch / mean duration
    eb = 2 if bf else 4
    Md, Nd = w.M * w.d * eb, w.N * w.d * eb
    # (the combine backward also writes the scattered inputs Xs: it reads X, dY and Ys and writes Xs and dYs)
    moved = {"gate_topk": Nd, "combine": Md + Nd, "dcombine": 2 * Nd + (0 if w.k == 1 else Md) + 2 * Md, "gate_bwd": 2 * Md + 2 * Nd}
    for n, nbytes in moved.items():
        if n in prof and prof[n][0]:
            c, t = prof[n]
            kern[n]["algorithmic_bytes"] = nbytes
            kern[n]["gbps"] = nbytes / (t / c * 1e-3) / 1e9
            kern[n]["frac_of_hbm_peak"] = kern[n]["gbps"] / PEAK_HBM_GBS
    clock_mhz = None
    if bf:   # the shader clock the last grouped product ran at (the chip does not hold its 2.4 GHz under matrix-core load)
        off, n = B.moe_workspace_region(desc, "clock")
        cyc, ticks = (int(v) for v in buf.workspace[off:off + n].view(torch.int64).cpu())
        clock_mhz = 100.0 * cyc / ticks if ticks > 0 else None
    roofline = {"bound": "mfma" if bf else "alu",
                # (the bf16 backward puts dZ with dW2 and dXs with dW1 into one launch each where that pays)
                "kernel": ("ggemm_cls_kernel / ggemm_pair_kernel / ggemm_sk_kernel" if bf else "ggemm_f32_kernel")
                + " (%d launches of 6 products per step)" % round(g_launches / a.steps),
                "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                "traffic": measured_hbm_bytes_per_gemm_launch(w.name) if not a.custom else None,
                "flops_per_launch": flops_launch, "avg_launch_us": avg_launch_ms * 1e3,
                # context: the same fraction against 256 CUs x 4096 flop/clk at the clock measured during the launch
                "shader_clock_mhz": clock_mhz,
                "frac_of_peak_at_measured_clock": (achieved / (256 * 4096 * clock_mhz * 1e6 / 1e12)) if clock_mhz else None}

    out = {
        "metric": METRIC, "value": w.N / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: N={w.N} d_m={w.d} d_h={w.h} E={w.E} top-{w.k} {w.dtype}, "
                               f"{'Zipf s=%g gate bias' % w.zipf_s if w.zipf_s else 'near-uniform gate'}; "
                               "step = moe_plan + moe_forward + moe_backward"},
        "expert_gemm_tflops_whole_step": w.expert_flops() / (ms_step * 1e-3) / 1e12,
        "grouped_gemm_pct_of_bf16_mfma_peak": 100.0 * achieved / PEAK_BF16_TFLOPS if bf else None,
        "roofline": roofline,
        "kernels": kern,
    }
    n_cpu = a.cpu_sample_tokens
    if n_cpu < 0:   # about 10-30 s of CPU work: the oracle costs ~24 M d h flop-pairs per assignment
        n_cpu = int(max(8, min(w.N, 2.5e11 / (12.0 * w.k * w.d * w.h))))
    if n_cpu > 0:
        out["cpu_baseline"] = cpu_baseline(w, inputs, n_cpu)
    return out


if __name__ == "__main__":
    main()
