#!/usr/bin/env python3
"""Benchmark of the INT8 training-convolution hot path on one MI355X.

A "step" is one pass of the whole path over one layer's synthetic tensors, all resident in HBM
before the timed region starts:
    quantize(a) + quantize(W) + DSGC clip search(g_z) + quantize(g_z; stochastic, d_c)
    + conv forward + conv backward-data + conv backward-weight.
The workload is the ResNet-18-style 3x3 layer (N=64, C=K=64, 56x56, stride 1, pad 1).
Metric: INT8 conv TOPS = 3 * 2 * N*K*P*Q*C*R*S / step time  (the three convolutions' integer
operations over the time of the whole step, quantizers and clip search included).

Prints ONE JSON line.  `roofline` is for the kernel that dominates the step; `cpu_baseline` times
the CPU oracle on a bounded slice of the same workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
INT8_MFMA_PEAK_TOPS = 5000.0
# plain (unpacked) vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, one operation per lane per issue
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12

CALLS = ["quantize_x", "quantize_w", "dsgc", "quantize_dy", "fwd", "bwd_data", "bwd_weight"]


def algorithmic(L, n_cand):
    """Algorithmic HBM bytes and arithmetic per call (what the method must move / compute)."""
    n_x = L.N * L.C * L.H * L.W
    n_w = L.K * (L.C // L.groups) * L.R * L.S
    n_y = L.N * L.K * L.P * L.Q
    macs = L.macs
    return {
        "quantize_x": dict(bytes=4 * n_x + 4 * n_x + n_x, ops=0),          # absmax read + read + code write
        "quantize_w": dict(bytes=9 * n_w, ops=0),
        # absmax pass (4 B/elem) + one sweep (4 B/elem).  Vector-ALU work of the sweep: 4.5 operations per
        # element and candidate (fused multiply-add, convert, 0.75 byte gather, 1.75 uint8 dot-product
        # accumulates) + 25 per element and 16-candidate chunk (draw, fixed point, digit planes)
        "dsgc": dict(bytes=8 * n_y, ops=(4.5 * n_cand + 25 * ((n_cand + 15) // 16)) * n_y),
        "quantize_dy": dict(bytes=5 * n_y, ops=0),
        "fwd": dict(bytes=n_x + n_w + 4 * n_y, ops=2 * macs),
        "bwd_data": dict(bytes=n_y + n_w + 4 * n_x, ops=2 * macs),
        "bwd_weight": dict(bytes=n_x + n_y + 4 * n_w, ops=2 * macs),
    }


def cpu_baseline(L, x, w, dy, ratios, n_img):
    """The oracle's full layer step on the first n_img images of the batch."""
    import numpy as np

    import oracle
    xs, dys = np.ascontiguousarray(x[:n_img]), np.ascontiguousarray(dy[:n_img])
    od = oracle.make_desc(n_img, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, L.groups)
    t0 = time.perf_counter()
    xq, _ = oracle.quantize(xs)
    wq, _ = oracle.quantize(w)
    o = oracle.dsgc(dys.reshape(-1), ratios, mode=oracle.ROUND_STOCHASTIC, seed=0)
    dyq, _ = oracle.quantize(dys, c=o["clip"], mode=oracle.ROUND_STOCHASTIC, seed=0)
    oracle.conv_fwd(od, xq, wq)
    oracle.conv_bwd_data(od, dyq, wq)
    oracle.conv_bwd_weight(od, xq, dyq)
    dt = time.perf_counter() - t0
    macs = n_img * L.K * L.P * L.Q * (L.C // L.groups) * L.R * L.S
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    threads = min(threads, os.cpu_count() or threads)
    return {"value": 6 * macs / dt / 1e12, "unit": "TOPS", "cores": threads, "kind": "oracle",
            "sample": f"first {n_img} of {L.N} images of the same layer, full step "
                      f"(quantize x3 + 32-candidate brute-force clip search + three int64 direct "
                      f"convolutions; convolutions on {threads} OpenMP threads, quantizers on 1), "
                      f"{dt:.2f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="benchmark config index (default 1: ResNet-18 3x3)")
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-images", type=int, default=64)
    ap.add_argument("--all-layers", action="store_true", help="also print a per-layer table for every config (stderr)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path shards over the batch, see DESIGN.md, but no multi-GPU run is part of it).",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1912_12607_amd import inputs
    from paper_1912_12607_amd.step import LayerStep

    assert torch.cuda.is_available(), "bench.py needs the GPU: the HIP library has no CPU fallback"
    n_cand = 32
    ratios = inputs.default_ratios(n_cand)

    def bench_layer(cfg, li, steps, warmup):
        L, x, w, dy = inputs.make_layer_inputs(cfg, li)
        st = LayerStep(L, n_cand=n_cand, keep_acc=False)
        st.upload(x, w, dy, ratios)
        torch.cuda.synchronize()
        for i in range(warmup):
            st.run(seed=i)
        torch.cuda.synchronize()
        # per-call HIP events on the launch stream (torch's current stream is the one the binding uses)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(CALLS) + 1)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            e = ev[i]
            e[0].record()
            st.quantize_x(); e[1].record()
            st.quantize_w(); e[2].record()
            st.dsgc(i); e[3].record()
            st.quantize_dy(i); e[4].record()
            st.fwd(); e[5].record()
            st.bwd_data(); e[6].record()
            st.bwd_weight(); e[7].record()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        per_call = {c: float(np.mean([ev[i][k].elapsed_time(ev[i][k + 1]) for i in range(steps)])) * 1e3
                    for k, c in enumerate(CALLS)}          # microseconds
        return L, (x, w, dy), dt / steps, per_call

    L, host, t_step, per_call = bench_layer(args.config, args.layer, args.steps, args.warmup)
    tops = 6 * L.macs / t_step / 1e12
    alg = algorithmic(L, n_cand)
    dom = max(per_call, key=per_call.get)
    t_dom = per_call[dom] * 1e-6
    a = alg[dom]
    # which roofline bounds the dominant call
    t_hbm = a["bytes"] / (HBM_PEAK_GBS * 1e9)
    if dom == "dsgc":
        t_alu = a["ops"] / (VALU_PEAK_TOPS * 1e12)
        if t_alu > t_hbm:
            roof = dict(bound="alu", achieved=a["ops"] / t_dom / 1e12, peak=VALU_PEAK_TOPS, unit="TOP/s")
        else:
            roof = dict(bound="hbm", achieved=a["bytes"] / t_dom / 1e9, peak=HBM_PEAK_GBS, unit="GB/s")
    elif a["ops"] / (INT8_MFMA_PEAK_TOPS * 1e12) > t_hbm:
        roof = dict(bound="mfma", achieved=a["ops"] / t_dom / 1e12, peak=INT8_MFMA_PEAK_TOPS, unit="TOP/s")
    else:
        roof = dict(bound="hbm", achieved=a["bytes"] / t_dom / 1e9, peak=HBM_PEAK_GBS, unit="GB/s")
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = None
    roof["kernel"] = {"dsgc": "int8t_dsgc_clip = absmax_kernel + dsgc_sweep_kernel + dsgc_finish_kernel",
                      "quantize_x": "int8t_quantize(a) = absmax_kernel + quantize_act_kernel",
                      "quantize_w": "int8t_quantize(W) = absmax_kernel + quantize_wgt_kernel",
                      "quantize_dy": "int8t_quantize(g_z) = quantize_act_kernel + deviation_finish_kernel",
                      "fwd": "int8t_conv_fwd = igemm_kernel", "bwd_data": "int8t_conv_bwd_data = igemm_kernel",
                      "bwd_weight": "int8t_conv_bwd_weight = wgrad_kernel + wgrad_reduce_kernel"}[dom]
    roof["us_per_launch"] = per_call[dom]

    out = {
        "metric": "INT8 conv TOPS (fwd+bwd-data+bwd-weight incl. quantize); % int8 MFMA peak",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config {args.config} layer {args.layer}: {L.name} N={L.N} C={L.C} "
                               f"H=W={L.H}x{L.W} K={L.K} {L.R}x{L.S} stride {L.stride[0]} pad {L.pad} "
                               f"groups {L.groups}; DSGC 32 candidates every step",
                   "pct_int8_mfma_peak": 100.0 * tops / INT8_MFMA_PEAK_TOPS,
                   "us_per_call": per_call,
                   "sum_calls_us": sum(per_call.values())},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(L, *host, ratios, args.cpu_images)

    if args.all_layers:
        for cfg in sorted(inputs.CONFIGS):
            for li in range(len(inputs.CONFIGS[cfg])):
                if (cfg, li) == (args.config, args.layer):
                    Lx, ts, pc = L, t_step, per_call
                else:
                    Lx, _, ts, pc = bench_layer(cfg, li, max(5, args.steps // 2), 3)
                al = algorithmic(Lx, n_cand)
                row = {"layer": f"{cfg}.{li} {Lx.name}", "ms_per_step": round(ts * 1e3, 4),
                       "TOPS": round(6 * Lx.macs / ts / 1e12, 2)}
                for c in CALLS:
                    t = pc[c] * 1e-6
                    row[c] = {"us": round(pc[c], 2), "GB/s": round(al[c]["bytes"] / t / 1e9, 1),
                              "TOP/s": round(al[c]["ops"] / t / 1e12, 2)}
                print(json.dumps(row), file=sys.stderr, flush=True)

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
