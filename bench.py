#!/usr/bin/env python3
"""Benchmark of the INT8 training-convolution hot path on one MI355X.

A "step" is one pass of the whole path over one layer's synthetic tensors, all resident in HBM
before the timed region starts:
    quantize(a) + quantize(W) + DSGC clip search(g_z) + quantize(g_z; stochastic)
    + conv forward + conv backward-data + conv backward-weight.
The clip search returns d_c (the input of Eq.7); the quantizer's optional second Eq.6 report is off.

Workload of the headline line: the largest of the benchmark's layers, the InceptionV3-style 1x7
convolution (config 4 layer 0: N=64, C=K=768, 17x17, pad (0,3); 152.7 G integer operations per
convolution pass) -- the layer on which "per cent of the int8 MFMA peak" means something.  Any other
layer: --config / --layer.
Metric: INT8 conv TOPS = 3 * 2 * N*K*P*Q*C*R*S / step time  (the three convolutions' integer
operations over the time of the whole step, quantizers and clip search included).

Successive steps alternate between --rotate (default 2) complete sets of buffers holding the same
values, so that no step finds its tensors in the 256 MB last-level cache because the previous step
left them there (a layer of a network never does); `single_set_ms_per_step` is the same loop on one
set, for comparison.

Prints ONE JSON line.  `roofline` is for the kernel with the largest share of the step, its
duration measured with HIP events inside the timed region; `config.passes` and `config.layers` give
every pass of the headline layer and every benchmark layer against its own roofline (int8 MFMA peak
for the convolutions, HBM peak for the quantizer passes); `cpu_baseline` times the CPU oracle on a
bounded slice of the same workload on this machine's host cores.
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

# STORED figures, not measured by this run: HBM bytes per launch from rocprofv3 counter runs
# (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a copy kernel of known
# size), keyed by (config, layer, kernel) -> (bytes, the profiles/ file that holds the run).
TRAFFIC = {
    (4, 0, "igemm_dma_kernel"): (int((50.2 + 81.0) * 1e6), "profiles/step_config4_inception_1x7_kernels_and_counters.md"),
    (4, 0, "wgrad_lines_kernel"): (int((101.6 + 49.5) * 1e6), "profiles/step_config4_inception_1x7_kernels_and_counters.md"),
    (2, 1, "igemm_dma_kernel"): (int((12.8 + 33.6) * 1e6), "profiles/step_config2_resnet50_3x3_kernels_and_counters.md"),
    (2, 1, "dsgc_sweep_kernel"): (int((25.9 + 0.6) * 1e6), "profiles/step_config2_resnet50_3x3_kernels_and_counters.md"),
    (2, 0, "igemm_dma_kernel"): (int((20.9 + 72.8) * 1e6), "profiles/step_config2_resnet50_1x1_reduce_kernels_and_counters.md"),
    (2, 0, "dsgc_sweep_kernel"): (int((25.9 + 0.6) * 1e6), "profiles/step_config2_resnet50_1x1_reduce_kernels_and_counters.md"),
    (1, 0, "dsgc_sweep_kernel"): (int((51.6 + 0.6) * 1e6), "profiles/step_config1_resnet18_3x3_kernels_and_counters.md"),
    (1, 0, "band_reg_kernel"): (int((13.3 + 51.4) * 1e6), "profiles/step_config1_resnet18_3x3_kernels_and_counters.md"),
}

MIN_STEPS_BEFORE_TIMING = 300


def sizes(L):
    n_x = L.N * L.C * L.H * L.W
    n_w = L.K * (L.C // L.groups) * L.R * L.S
    n_y = L.N * L.K * L.P * L.Q
    return n_x, n_w, n_y


def pass_algorithmic(L, n_cand):
    """Algorithmic HBM bytes and arithmetic of each pass of the step: what the method must move and
    compute (scratch traffic, second code copies' reads and the like are not counted).
    {pass: (bytes, ops, kind of ops)}"""
    n_x, n_w, n_y = sizes(L)
    macs = L.macs
    return {
        "absmax_xw": (4 * (n_x + n_w), 0, None),                 # one read of a and W
        "quantize_xw": (5 * n_x + 6 * n_w, 0, None),             # fp32 read + code write (W: two layouts)
        "absmax_gz": (4 * n_y, 0, None),                         # max|g_z| and sum g_z^2, one read
        # One read of g_z.  Vector-ALU work of the sweep: 2.5 operations per element and candidate (round-down
        # fused multiply-add, convert-and-pack, a shift and a mask per four) + 31 per element and 32-candidate
        # chunk (draw, fixed point, digit planes, LDS traffic); the products and sums themselves run on the matrix cores.
        "dsgc_search": (4 * n_y, (2.5 * n_cand + 31 * ((n_cand + 31) // 32)) * n_y, "valu"),
        "quantize_gz": (5 * n_y, 0, None),
        "fwd": (n_x + n_w + 4 * n_y, 2 * macs, "mfma"),
        "bwd_data": (n_y + n_w + 4 * n_x, 2 * macs, "mfma"),
        "bwd_weight": (n_x + n_y + 4 * n_w, 2 * macs, "mfma"),
    }


def roofline_of(nbytes, ops, kind, seconds, depthwise=False):
    """The roofline that bounds (bytes, ops) and the fraction of it reached in `seconds`."""
    t_hbm = nbytes / (HBM_PEAK_GBS * 1e9)
    if kind == "mfma" and not depthwise and ops / (INT8_MFMA_PEAK_TOPS * 1e12) > t_hbm:
        r = dict(bound="mfma", achieved=ops / seconds / 1e12, peak=INT8_MFMA_PEAK_TOPS, unit="TOP/s")
    elif kind == "valu" and ops / (VALU_PEAK_TOPS * 1e12) > t_hbm:
        r = dict(bound="alu", achieved=ops / seconds / 1e12, peak=VALU_PEAK_TOPS, unit="TOP/s")
    else:
        r = dict(bound="hbm", achieved=nbytes / seconds / 1e9, peak=HBM_PEAK_GBS, unit="GB/s")
    r["frac"] = r["achieved"] / r["peak"]
    return r


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
    # a step takes 0.1 - 0.4 ms: with a few dozen steps the GPU is still ramping its clocks up while it is
    # measured, hence the long defaults (and MIN_STEPS_BEFORE_TIMING)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--config", type=int, default=4, help="benchmark config index (default 4: InceptionV3-style layers)")
    ap.add_argument("--layer", type=int, default=0, help="layer of the config (default 0: the 1x7 convolution)")
    ap.add_argument("--rotate", type=int, default=2,
                    help="sets of buffers the steps alternate between (default 2: together above the 256 MB "
                         "last-level cache for every benchmark layer; 1 = one set, re-used by every step)")
    ap.add_argument("--dsgc-period", type=int, default=1,
                    help="run the clip search every P-th step only (Periodic Update, Table 2); default 1 = "
                         "every step, the benchmark's setting")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true",
                    help="issue every call on one stream (default: a, W quantization and the forward convolution "
                         "run on a second stream beside the clip search where that pays)")
    ap.add_argument("--no-tune", action="store_true", help="keep the library's own kernel choice (default: each layer's kernels are "
                                                           "chosen by timing the admissible variants before its steps are timed)")
    ap.add_argument("--no-layers", action="store_true", help="leave the per-layer table of all benchmark layers out")
    ap.add_argument("--cpu-images", type=int, default=0, help="images of the batch the oracle is timed on (0: by layer size)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="after the steps, run a plain elementwise copy of this many MiB three times "
                         "(reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--all-layers", action="store_true", help="also print the per-kernel table of every layer (stderr)")
    ap.add_argument("--resnet50", type=int, default=0, metavar="BATCH",
                    help="also time the step of every ResNet-50 convolution and its classifier at this batch "
                         "(Fig.10's workload) and print the per-layer table and the network total (stderr)")
    ap.add_argument("--mobilenetv2", type=int, default=0, metavar="BATCH", help="the same for every convolution of MobileNetV2")
    ap.add_argument("--variant-table", action="store_true",
                    help="in the network sweeps, also time every kernel variant of every layer and pass (stderr; the sweep itself "
                         "keeps the library's own choice)")
    ap.add_argument("--fused-forward", action="store_true",
                    help="also time quantize(a, W) + forward against the fused forward (int8t_conv_fwd_fused) on 1x1 layers (stderr)")
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
    rotate = max(1, args.rotate)
    ratios = inputs.default_ratios(n_cand)
    overlap = False if args.no_overlap else None        # None: LayerStep decides per layer

    def profile_calls(calls, reps):
        """{kernel: (launches per call sequence, us per launch)} of `calls` run `reps` times on one
        stream with every launch carrying HIP events."""
        for _ in range(20):
            for c in calls:
                c()
        torch.cuda.synchronize()
        B.int8t_profile_start(None)
        for _ in range(reps):
            for c in calls:
                c()
        torch.cuda.synchronize()
        prof = B.int8t_profile_stop()
        return {k: (n / reps, ms * 1e3 / n) for k, (n, ms) in prof.items()}

    def pass_table(L, st):
        """Every pass of the step on its own (one stream, launches back to back): its kernels, its time,
        its algorithmic bytes / operations and the fraction of the roofline that bounds it.  Also returns
        {kernel: [algorithmic bytes, ops, kind, launches]} summed over the passes each kernel served."""
        alg = pass_algorithmic(L, n_cand)
        dw = L.groups != 1
        sp = B.stream_pointer(None)
        # (the calls with their arguments marshalled once: launched back to back they keep the GPU busy, which a
        # loop that rebuilds its arguments in Python does not -- an idling GPU drops its clocks)
        calls = [("quantize_xw", lambda: st._k_xw(sp)), ("dsgc", lambda: st._k_clip(0, sp)),
                 ("quantize_gz", lambda: st._k_qdy(0, sp)), ("fwd", lambda: st._k_fwd(sp)),
                 ("bwd_data", lambda: st._k_bwd_data(sp)), ("bwd_weight", lambda: st._k_bwd_weight(sp))]
        rows, per_kernel = [], {}

        def add(name, kernels, key):
            us = sum(n * t for n, t in kernels.values())
            nbytes, ops, kind = alg[key]
            row = {"pass": name, "us": round(us, 2), "kernels": {k: round(n * t, 2) for k, (n, t) in kernels.items()},
                   "algorithmic_bytes": nbytes, "algorithmic_ops": ops}
            row.update({k: (round(v, 4) if isinstance(v, float) else v)
                        for k, v in roofline_of(nbytes, ops, kind, us * 1e-6, dw).items()})
            rows.append(row)
            main_k = max(kernels, key=lambda k: kernels[k][0] * kernels[k][1])
            e = per_kernel.setdefault(main_k, [0, 0, kind, 0])
            e[0] += nbytes
            e[1] += ops
            e[3] += kernels[main_k][0]

        for name, fn in calls:
            pk = profile_calls([fn], 20)
            if name == "quantize_xw":
                add("absmax_xw", {k: v for k, v in pk.items() if k.startswith("absmax")}, "absmax_xw")
                add("quantize_xw", {k: v for k, v in pk.items() if not k.startswith("absmax")}, "quantize_xw")
            elif name == "dsgc":
                add("absmax_gz", {k: v for k, v in pk.items() if k.startswith("absmax")}, "absmax_gz")
                add("dsgc_search", {k: v for k, v in pk.items() if not k.startswith("absmax")}, "dsgc_search")
            else:
                add(name, pk, name)
        return rows, per_kernel

    kernel_choice = {}

    def make_sets(cfg, li, count):
        """`count` sets of buffers of the layer holding the same values; the layer's kernels are chosen by
        measurement first (untimed; the per-layer choice "before training" of the paper's Suppl.)."""
        L, x, w, dy = inputs.make_layer_inputs(cfg, li)
        sets = []
        for _ in range(count):
            st = LayerStep(L, n_cand=n_cand, keep_acc=False, requantize_deviation=False)
            st.upload(x, w, dy, ratios)
            sets.append(st)
        if not args.no_tune:
            for i in range(30):
                sets[0].run(seed=i, overlap=False)
            torch.cuda.synchronize()
            ch = sets[0].tune_kernels()
            kernel_choice[f"{cfg}.{li}"] = {k: v[0] for k, v in ch.items()}
            for st in sets[1:]:
                st.refresh_scratch()
        torch.cuda.synchronize()
        return L, (x, w, dy), sets

    def timed_steps(sets, steps, warm, sampled_kernel=None, every=5):
        """Seconds per step over `steps` steps after `warm` untimed ones, the steps alternating between
        the buffer sets; with sampled_kernel, every `every`-th launch of that kernel carries HIP events
        inside the timed region: returns (seconds per step, us per sampled launch or None)."""
        k = len(sets)
        for i in range(warm):
            sets[i % k].run(seed=i, search=(i % period == 0), overlap=overlap)
        torch.cuda.synchronize()
        if sampled_kernel:
            B.int8t_profile_start_sampled(sampled_kernel, every)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            sets[i % k].run(seed=i, search=(i % period == 0), overlap=overlap)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        us = None
        if sampled_kernel:
            n, ms = B.int8t_profile_stop()[sampled_kernel]
            us = ms * 1e3 / n
        return dt, us

    def step_kernels(st):
        """{kernel: (launches per step, us per launch)} of whole one-stream steps with every launch timed."""
        nprof = 5
        for i in range(3):
            st.run(seed=i, overlap=False)
        torch.cuda.synchronize()
        B.int8t_profile_start(None)
        for i in range(nprof):
            st.run(seed=i, search=(i % period == 0), overlap=False)
        torch.cuda.synchronize()
        prof = B.int8t_profile_stop()
        return {k: (n / nprof, ms * 1e3 / n) for k, (n, ms) in prof.items()}

    # ---- headline layer -------------------------------------------------------------------------
    L, host, sets = make_sets(args.config, args.layer, rotate)
    warm_total = max(args.warmup, MIN_STEPS_BEFORE_TIMING)
    # The GPU ramps its clocks up over the first tens of milliseconds of work: whatever --warmup is, at
    # least MIN_STEPS_BEFORE_TIMING steps run before anything is measured; `warmup` in the output is the
    # number that ran.
    timed_steps(sets, 1, warm_total)
    per_kernel = step_kernels(sets[0])
    dom = max(per_kernel, key=lambda k: per_kernel[k][0] * per_kernel[k][1])
    passes, kernel_alg = pass_table(L, sets[0])
    every = 5 if args.steps * per_kernel[dom][0] >= 5 else 1
    t_step, dom_us = timed_steps(sets, args.steps, 20, dom, every)
    tops = 6 * L.macs / t_step / 1e12

    nbytes, ops, kind, launches = kernel_alg.get(dom, [0, 0, None, per_kernel[dom][0]])
    launches = launches or per_kernel[dom][0]
    # per launch, as the duration is: the kernel's algorithmic work of the step / its launches per step
    roof = roofline_of(nbytes / launches, ops / launches, kind, dom_us * 1e-6, L.groups != 1)
    tr = TRAFFIC.get((args.config, args.layer, dom))
    roof["traffic"] = tr[0] if tr else None
    roof["traffic_source"] = ("stored figure, not measured by this run: " + tr[1]) if tr else None
    roof["kernel"] = dom
    roof["launches_per_step"] = per_kernel[dom][0]
    roof["us_per_launch"] = dom_us
    roof["algorithmic_bytes_per_launch"] = nbytes / launches
    roof["algorithmic_ops_per_launch"] = ops / launches
    two_streams = overlap is None and period == 1 and two_stream_default(L)
    if two_streams:
        # In the timed region the kernel may share the compute units with the second stream's kernels;
        # what it does with the machine to itself comes from the untimed one-stream pass.
        roof["us_per_launch_one_stream"] = per_kernel[dom][1]

    single_ms = None
    if rotate > 1:
        single_ms = timed_steps(sets[:1], max(50, args.steps // 4), 50)[0] * 1e3

    out = {
        "metric": "INT8 conv TOPS (fwd+bwd-data+bwd-weight incl. quantize); % int8 MFMA peak",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": warm_total + 20,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config {args.config} layer {args.layer}: {L.name} N={L.N} C={L.C} "
                               f"H=W={L.H}x{L.W} K={L.K} {L.R}x{L.S} stride {L.stride[0]} pad {L.pad} "
                               f"groups {L.groups}; DSGC 32 candidates " + ("every step" if period == 1 else f"every {period} steps"),
                   "streams": ("2: quantization of a, W and the forward convolution beside the clip search"
                               if two_streams else "1"),
                   "buffer_sets": rotate, "single_set_ms_per_step": single_ms,
                   "warmup_requested": args.warmup,
                   "pct_int8_mfma_peak": 100.0 * tops / INT8_MFMA_PEAK_TOPS,
                   "kernel_choice": kernel_choice,
                   "us_per_kernel": {k: {"launches_per_step": v[0], "us_per_launch": round(v[1], 2)}
                                     for k, v in sorted(per_kernel.items(), key=lambda kv: -kv[1][0] * kv[1][1])},
                   "sum_kernels_us": sum(v[0] * v[1] for v in per_kernel.values()),
                   "passes": passes},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        n_img = args.cpu_images or max(1, min(L.N, int(L.N * 1.5e11 / (3 * L.macs + 1))))
        out["cpu_baseline"] = cpu_baseline(L, *host, ratios, n_img)
    del sets
    torch.cuda.empty_cache()

    # ---- every benchmark layer against its own rooflines ------------------------------------------
    if not args.no_layers:
        rows = []
        for cfg in sorted(c for c in inputs.CONFIGS if 1 <= c <= 4):
            for li in range(len(inputs.CONFIGS[cfg])):
                Lx, _, sx = make_sets(cfg, li, rotate)
                ts, _ = timed_steps(sx, max(100, args.steps // 5), 150)
                prow, _ = pass_table(Lx, sx[0])
                row = {"layer": f"{cfg}.{li} {Lx.name}", "ms_per_step": round(ts * 1e3, 4),
                       "TOPS": round(6 * Lx.macs / ts / 1e12, 2),
                       "pct_int8_mfma_peak": round(600 * Lx.macs / ts / 1e12 / INT8_MFMA_PEAK_TOPS, 3),
                       "passes": {p["pass"]: {"us": p["us"], "bound": p["bound"], "achieved": round(p["achieved"], 1),
                                              "unit": p["unit"], "frac": round(p["frac"], 4)} for p in prow}}
                rows.append(row)
                if args.all_layers:
                    print(json.dumps({"layer": row["layer"], "passes": prow}), file=sys.stderr, flush=True)
                del sx
                torch.cuda.empty_cache()
        out["config"]["layers"] = rows

    # what the matrix cores sustain on this GPU: published peak needs all-zero operands; random int8 operands
    # pull the clock down (power limit), and that is the ceiling of a convolution on real codes
    ceil = {}
    for name, rnd, lds in (("zero_operands_from_registers", 0, 0), ("random_operands_from_registers", 1, 0),
                           ("random_operands_from_lds", 1, 1)):
        t, ghz = B.int8t_profile_mfma_ceiling(rnd, lds, 20000)
        ceil[name] = {"TOPS": round(t, 1), "shader_clock_GHz": round(ghz, 3)}
    out["config"]["int8_mfma_ceiling_measured"] = ceil
    if roof["bound"] == "mfma":
        roof["frac_of_measured_ceiling_random_operands_from_lds"] = roof["achieved"] / ceil["random_operands_from_lds"]["TOPS"]

    if args.copy_calibration > 0:
        src = torch.ones(args.copy_calibration * (1 << 20) // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)       # one elementwise kernel: reads and writes the stated size once
        torch.cuda.synchronize()

    def sweep(title, batch, layers, seed_cfg):
        """One step per distinct layer shape; the network's time is the sum over shapes x multiplicity."""
        total_ms, total_ops = 0.0, 0
        for i, (count, Lx) in enumerate(layers):
            # the first layer's input is the image: no backward-data pass there (4 of the 6 MAC passes counted)
            st = LayerStep(Lx, n_cand=n_cand, keep_acc=False, requantize_deviation=False, input_grad=i > 0)
            npass = 6 if i > 0 else 4
            st.upload(inputs.make_x(Lx, seed_cfg, i), inputs.make_w(Lx, seed_cfg, i), inputs.make_dy(Lx, seed_cfg, i), ratios)
            nst = max(20, args.steps // 10)
            for k in range(80):          # the first few dozen steps on fresh buffers run at up to twice the steady time
                st.run(seed=k, overlap=overlap)
            if overlap is None:
                st.tune()                # one or two streams for this layer, by measurement (untimed)
            if args.variant_table:
                # every variant the library admits, per pass (microseconds); the library's own rule is restored afterwards
                table = st.tune_kernels()
                for op in (B.OP_CONV_FWD, B.OP_CONV_BWD_DATA, B.OP_CONV_BWD_WEIGHT):
                    B.int8t_conv_select_variant(op, st.desc, B.VARIANT_AUTO)
                st.refresh_scratch()
                if table:
                    print(json.dumps({"variants": Lx.name, **{k: v[1] for k, v in table.items()}}), file=sys.stderr, flush=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(nst):
                st.run(seed=k, search=(k % period == 0), overlap=overlap)
            torch.cuda.synchronize()
            ts = (time.perf_counter() - t0) / nst
            total_ms += count * ts * 1e3
            total_ops += count * Lx.macs * npass
            print(json.dumps({"layer": Lx.name, "count": count, "C": Lx.C, "HW": Lx.H, "K": Lx.K, "RS": [Lx.R, Lx.S],
                              "stride": Lx.stride[0], "groups": Lx.groups, "ms_per_step": round(ts * 1e3, 4),
                              "TOPS": round(npass * Lx.macs / ts / 1e12, 1)}), file=sys.stderr, flush=True)
            del st
        print(json.dumps({"network": title, "batch": batch, "ms_per_iteration": round(total_ms, 3),
                          "TOPS": round(total_ops / total_ms / 1e9, 1),
                          "images_per_s": round(batch / total_ms * 1e3, 1)}), file=sys.stderr, flush=True)

    if args.fused_forward:
        # the quantization-convolution fused kernel (Suppl. "INT8 Convolution") against the separate passes:
        # 1x1 stride-1 layers, one stream, wall clock over 300 repetitions after 150 untimed ones
        def timeit(fn, reps=300):
            for _ in range(150):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps * 1e6

        def r50(C, HW, K):
            return inputs.Layer("r50_1x1", 64, C, HW, HW, K, 1, 1, x_dist="relu", dy_scale=1e-4)
        cases = [("config 3 layer 2 (MobileNetV2 144 -> 24, 56x56, N=64)", inputs.CONFIGS[3][2], 3, 2),
                 ("config 3 layer 0 (MobileNetV2 24 -> 144, 56x56, N=64)", inputs.CONFIGS[3][0], 3, 0),
                 ("config 2 layer 0 (ResNet-50 1024 -> 256, 14x14, N=128)", inputs.CONFIGS[2][0], 2, 0),
                 ("config 2 layer 2 (ResNet-50 256 -> 1024, 14x14, N=128)", inputs.CONFIGS[2][2], 2, 2),
                 ("ResNet-50 256 -> 64, 56x56, N=64", r50(256, 56, 64), 7, 0),
                 ("ResNet-50 64 -> 64, 56x56, N=64", r50(64, 56, 64), 7, 1),
                 ("ResNet-50 512 -> 128, 28x28, N=64", r50(512, 28, 128), 7, 2)]
        for name, Lx, cfg_i, li_i in cases:
            xx, ww, dd = inputs.make_x(Lx, cfg_i, li_i), inputs.make_w(Lx, cfg_i, li_i), inputs.make_dy(Lx, cfg_i, li_i)
            res = {}
            for fused in (False, True):
                st = LayerStep(Lx, requantize_deviation=False, fused_fwd=fused)
                st.upload(xx, ww, dd, ratios)
                st.run(seed=0, overlap=False)
                torch.cuda.synchronize()
                sp = B.stream_pointer(None)
                if fused:
                    chain = lambda: (st._k_w(sp), st._k_fwd_fused(sp))
                else:
                    chain = lambda: (st._k_xw(sp), st._k_fwd(sp))
                res[fused] = (timeit(chain), timeit(lambda: st.run(seed=1, overlap=False)))
                del st
            print(json.dumps({"layer": name, "quantize_aW_plus_fwd_us": round(res[False][0], 1), "fused_us": round(res[True][0], 1),
                              "whole_step_us": round(res[False][1], 1), "whole_step_fused_fwd_us": round(res[True][1], 1)}),
                  file=sys.stderr, flush=True)

    if args.resnet50 > 0:
        sweep("ResNet-50 convolutions + classifier", args.resnet50, inputs.resnet50_layers(args.resnet50), 50)
    if args.mobilenetv2 > 0:
        sweep("MobileNetV2 convolutions", args.mobilenetv2, inputs.mobilenetv2_layers(args.mobilenetv2), 51)
    if args.inceptionv3 > 0:
        sweep("InceptionV3, one layer of each kind", args.inceptionv3, inputs.inceptionv3_layers(args.inceptionv3), 52)

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
