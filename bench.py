#!/usr/bin/env python3
"""Benchmark of the INT8 training-convolution hot path on one MI355X.

A "step" is one pass of the whole path over one layer's synthetic tensors, all resident in HBM
before the timed region starts:
    quantize(a) + quantize(W) + DSGC clip search(g_z) + quantize(g_z; stochastic, d_c)
    + conv forward + conv backward-data + conv backward-weight.
The clip search returns d_c (the input of Eq.7); the quantizer's optional second Eq.6 report is off.
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

# HBM bytes per launch from rocprofv3 counter runs (FETCH_SIZE + WRITE_SIZE, each scaled by what the same
# counter reads for a copy kernel of known size); keyed by (config, layer, kernel).  See profiles/.
TRAFFIC = {(1, 0, "dsgc_sweep_kernel"): 50979 * 1024,
           (1, 0, "band_kernel"): 63166 * 1024}        # mean of the forward and the backward-data launch

def algorithmic(L, n_cand):
    """Algorithmic HBM bytes and arithmetic of one step, per kernel name (what the method must move
    and compute, summed over that kernel's launches in the step; scratch traffic is not counted)."""
    n_x = L.N * L.C * L.H * L.W
    n_w = L.K * (L.C // L.groups) * L.R * L.S
    n_y = L.N * L.K * L.P * L.Q
    macs = L.macs
    conv2 = dict(bytes=(n_x + n_w + 4 * n_y) + (n_y + n_w + 4 * n_x), ops=4 * macs)   # forward + backward-data
    wg = dict(bytes=n_x + n_y + 4 * n_w, ops=2 * macs)
    return {
        # the step quantizes a and W in one batched call (one absmax launch, one quantize launch) and g_z on its own
        "absmax_batch_kernel": dict(bytes=4 * (n_x + n_w), ops=0),                # a, W: one read each
        "quantize_batch_kernel": dict(bytes=5 * n_x + 6 * n_w, ops=0),            # fp32 read + code write (two copies of W)
        "absmax_kernel": dict(bytes=4 * n_y, ops=0),                              # g_z: one read
        "quantize_act_kernel": dict(bytes=5 * n_y, ops=0),                        # fp32 read + code write of g_z
        "quantize_planar_kernel": dict(bytes=5 * n_y, ops=0),
        "quantize_wgt_kernel": dict(bytes=6 * n_w, ops=0),
        "deviation_finish_kernel": dict(bytes=0, ops=0),
        # one read of g_z.  Vector-ALU work of the sweep: 2.75 operations per element and candidate (round-down
        # fused multiply-add, convert, 0.75 byte gather) + 30 per element and 32-candidate chunk (draw, fixed
        # point, digit planes, LDS traffic); the products and sums themselves run on the matrix cores
        "dsgc_sweep_kernel": dict(bytes=4 * n_y, ops=(2.75 * n_cand + 30 * ((n_cand + 31) // 32)) * n_y),
        "igemm_kernel": conv2, "band_kernel": conv2, "dw_conv_kernel": conv2,
        "igemm_reduce_kernel": dict(bytes=4 * (n_x + n_y), ops=0),               # final sum of a split reduction
        "wgrad_kernel": wg, "dw_wgrad_kernel": wg,
        "wgrad_reduce_kernel": dict(bytes=4 * n_w, ops=0), "dw_wgrad_reduce_kernel": dict(bytes=4 * n_w, ops=0),
        "s2d_repack_kernel": dict(bytes=2 * n_x, ops=0),                          # codes of a in, rearranged codes out
        "s2d_weights_kernel": dict(bytes=2 * n_w, ops=0),
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
    # a step takes about 0.15 ms: with a few dozen steps the GPU is still ramping its clocks up while it is
    # measured (50 steps after 5: 0.149 ms per step; 500 after 200: 0.140 ms), hence the long defaults
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=1, help="benchmark config index (default 1: ResNet-18 3x3)")
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--dsgc-period", type=int, default=1,
                    help="run the clip search every P-th step only (Periodic Update, Table 2); default 1 = "
                         "every step, the benchmark's setting")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true",
                    help="issue every call on one stream (default: a, W quantization and the forward convolution "
                         "run on a second stream beside the clip search in the steps that search)")
    ap.add_argument("--cpu-images", type=int, default=64)
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="after the steps, run a plain elementwise copy of this many MiB three times "
                         "(reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--all-layers", action="store_true", help="also print a per-layer table for every config (stderr)")
    ap.add_argument("--resnet50", type=int, default=0, metavar="BATCH",
                    help="also time the step of every ResNet-50 convolution and its classifier at this batch "
                         "(Fig.10's workload) and print the per-layer table and the network total (stderr)")
    ap.add_argument("--mobilenetv2", type=int, default=0, metavar="BATCH", help="the same for every convolution of MobileNetV2")
    ap.add_argument("--inceptionv3", type=int, default=0, metavar="BATCH",
                    help="the same for one layer of each kind in InceptionV3 (no network total: not every layer is listed)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path would shard over the batch, but no multi-GPU run is part of it).",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1912_12607_amd import binding as B
    from paper_1912_12607_amd import inputs
    from paper_1912_12607_amd.step import LayerStep, two_stream_default

    assert torch.cuda.is_available(), "bench.py needs the GPU: the HIP library has no CPU fallback"
    n_cand = 32
    period = max(1, args.dsgc_period)
    ratios = inputs.default_ratios(n_cand)

    overlap = False if args.no_overlap else None        # None: LayerStep decides per layer

    def bench_layer(cfg, li, steps, warmup):
        """Returns layer, host tensors, seconds per step, {kernel: (launches per step, us per launch)} of
        an untimed pass with every kernel launch carrying events, and the dominant kernel's
        (name, launches per step, us per launch) measured by events inside the timed region itself."""
        L, x, w, dy = inputs.make_layer_inputs(cfg, li)
        st = LayerStep(L, n_cand=n_cand, keep_acc=False, requantize_deviation=False)
        st.upload(x, w, dy, ratios)
        torch.cuda.synchronize()
        # The GPU ramps its clocks up over the first tens of milliseconds of work (50 steps after 5 read 6 %
        # slower than 1000 after 200): whatever W is, the card has run at least 300 steps before the timed
        # region, so that a short run measures the same steady state as a long one.
        for i in range(max(0, 300 - warmup)):
            st.run(seed=i, overlap=overlap)
        for i in range(warmup):
            st.run(seed=i, overlap=overlap)
        torch.cuda.synchronize()
        # pass 1 (untimed): HIP events around every kernel launch, on the launch stream, inside the library
        nprof = max(3, min(10, steps))
        B.int8t_profile_start(None)
        for i in range(nprof):
            st.run(seed=i, search=(i % period == 0))
        torch.cuda.synchronize()
        prof = B.int8t_profile_stop()
        per_kernel = {k: (n / nprof, ms * 1e3 / n) for k, (n, ms) in prof.items()}
        dom = max(prof, key=lambda k: prof[k][1])
        torch.cuda.synchronize()
        # pass 2 (the timed region): only the dominant kernel carries events, and only every 5th of its
        # launches -- a timed dispatch idles the GPU for about 5 us before and after it (measured with a
        # kernel trace), which would otherwise be charged to every step
        every = 5 if steps * per_kernel[dom][0] >= 5 else 1
        B.int8t_profile_start_sampled(dom, every)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            st.run(seed=i, search=(i % period == 0), overlap=overlap)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        n, ms = B.int8t_profile_stop()[dom]
        return L, (x, w, dy), dt / steps, per_kernel, (dom, per_kernel[dom][0], ms * 1e3 / n)

    L, host, t_step, per_kernel, (dom, dom_launches, dom_us) = bench_layer(args.config, args.layer, args.steps, args.warmup)
    tops = 6 * L.macs / t_step / 1e12
    a = algorithmic(L, n_cand)[dom]
    t_dom = dom_us * 1e-6 * dom_launches           # the kernel's time per step
    # which roofline bounds the dominant kernel
    t_hbm = a["bytes"] / (HBM_PEAK_GBS * 1e9)
    if dom == "dsgc_sweep_kernel" and a["ops"] / (VALU_PEAK_TOPS * 1e12) > t_hbm:
        roof = dict(bound="alu", achieved=a["ops"] / t_dom / 1e12, peak=VALU_PEAK_TOPS, unit="TOP/s")
    elif dom != "dsgc_sweep_kernel" and a["ops"] / (INT8_MFMA_PEAK_TOPS * 1e12) > t_hbm:
        roof = dict(bound="mfma", achieved=a["ops"] / t_dom / 1e12, peak=INT8_MFMA_PEAK_TOPS, unit="TOP/s")
    else:
        roof = dict(bound="hbm", achieved=a["bytes"] / t_dom / 1e9, peak=HBM_PEAK_GBS, unit="GB/s")
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = TRAFFIC.get((args.config, args.layer, dom))
    roof["kernel"] = dom
    roof["launches_per_step"] = dom_launches
    roof["us_per_launch"] = dom_us
    two_streams = overlap is None and period == 1 and two_stream_default(L)
    if two_streams:
        # In the timed region the kernel shares the compute units with the second stream's kernels; what it
        # does with the machine to itself comes from the untimed one-stream pass.
        roof["us_per_launch_one_stream"] = per_kernel[dom][1]
        roof["frac_one_stream"] = roof["frac"] * dom_us / per_kernel[dom][1]

    out = {
        "metric": "INT8 conv TOPS (fwd+bwd-data+bwd-weight incl. quantize); % int8 MFMA peak",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config {args.config} layer {args.layer}: {L.name} N={L.N} C={L.C} "
                               f"H=W={L.H}x{L.W} K={L.K} {L.R}x{L.S} stride {L.stride[0]} pad {L.pad} "
                               f"groups {L.groups}; DSGC 32 candidates " + ("every step" if period == 1 else f"every {period} steps"),
                   "streams": ("2: quantization of a, W and the forward convolution beside the clip search"
                               if two_streams else "1"),
                   "pct_int8_mfma_peak": 100.0 * tops / INT8_MFMA_PEAK_TOPS,
                   "us_per_kernel": {k: {"launches_per_step": v[0], "us_per_launch": round(v[1], 2)}
                                     for k, v in sorted(per_kernel.items(), key=lambda kv: -kv[1][0] * kv[1][1])},
                   "sum_kernels_us": sum(v[0] * v[1] for v in per_kernel.values())},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(L, *host, ratios, args.cpu_images)

    if args.copy_calibration > 0:
        src = torch.ones(args.copy_calibration * (1 << 20) // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)       # one elementwise kernel: reads and writes the stated size once
        torch.cuda.synchronize()

    if args.all_layers:
        for cfg in sorted(inputs.CONFIGS):
            for li in range(len(inputs.CONFIGS[cfg])):
                if (cfg, li) == (args.config, args.layer):
                    Lx, ts, pk = L, t_step, per_kernel
                else:
                    Lx, _, ts, pk, _ = bench_layer(cfg, li, max(5, args.steps // 2), 3)
                al = algorithmic(Lx, n_cand)
                row = {"layer": f"{cfg}.{li} {Lx.name}", "ms_per_step": round(ts * 1e3, 4),
                       "TOPS": round(6 * Lx.macs / ts / 1e12, 2)}
                for k, (n, us) in sorted(pk.items(), key=lambda kv: -kv[1][0] * kv[1][1]):
                    t = n * us * 1e-6
                    row[k] = {"us_per_step": round(n * us, 2), "GB/s": round(al[k]["bytes"] / t / 1e9, 1),
                              "TOP/s": round(al[k]["ops"] / t / 1e12, 2)}
                print(json.dumps(row), file=sys.stderr, flush=True)

    def sweep(title, batch, layers, seed_cfg):
        """One step per distinct layer shape; the network's time is the sum over shapes x multiplicity."""
        total_ms, total_ops = 0.0, 0
        for i, (count, Lx) in enumerate(layers):
            # the first layer's input is the image: no backward-data pass there (4 of the 6 MAC passes counted)
            st = LayerStep(Lx, n_cand=n_cand, keep_acc=False, requantize_deviation=False, input_grad=i > 0)
            passes = 6 if i > 0 else 4
            st.upload(inputs.make_x(Lx, seed_cfg, i), inputs.make_w(Lx, seed_cfg, i), inputs.make_dy(Lx, seed_cfg, i), ratios)
            nst = max(20, args.steps // 10)
            for k in range(80):          # the first few dozen steps on fresh buffers run at up to twice the steady time
                st.run(seed=k, overlap=overlap)
            if overlap is None and period == 1:
                st.tune()                # one or two streams for this layer, by measurement (untimed)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(nst):
                st.run(seed=k, search=(k % period == 0), overlap=overlap)
            torch.cuda.synchronize()
            ts = (time.perf_counter() - t0) / nst
            total_ms += count * ts * 1e3
            total_ops += count * Lx.macs * passes
            print(json.dumps({"layer": Lx.name, "count": count, "C": Lx.C, "HW": Lx.H, "K": Lx.K, "RS": [Lx.R, Lx.S],
                              "stride": Lx.stride[0], "groups": Lx.groups, "ms_per_step": round(ts * 1e3, 4),
                              "TOPS": round(passes * Lx.macs / ts / 1e12, 1)}), file=sys.stderr, flush=True)
            del st
        print(json.dumps({"network": title, "batch": batch, "ms_per_iteration": round(total_ms, 3),
                          "TOPS": round(total_ops / total_ms / 1e9, 1),
                          "images_per_s": round(batch / total_ms * 1e3, 1)}), file=sys.stderr, flush=True)

    if args.resnet50 > 0:
        sweep("ResNet-50 convolutions + classifier", args.resnet50, inputs.resnet50_layers(args.resnet50), 50)
    if args.mobilenetv2 > 0:
        sweep("MobileNetV2 convolutions", args.mobilenetv2, inputs.mobilenetv2_layers(args.mobilenetv2), 51)
    if args.inceptionv3 > 0:
        sweep("InceptionV3, one layer of each kind", args.inceptionv3, inputs.inceptionv3_layers(args.inceptionv3), 52)

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
