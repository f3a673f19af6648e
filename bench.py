#!/usr/bin/env python3
"""FPROP convolution benchmark: TFLOP/s by the complexity formula of Section 2
of the maxDNN paper, and the fraction of MI355X's FP32 matrix peak (the
"computational efficiency" of Section 3.3, credited only for required FLOPs).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vgg]
                    [--variant NAME] [--no-layers] [--no-cpu-baseline] [--no-probe]

A step is one whole FPROP convolution of the named layer (one launch of
mdnn_conv_fprop) on seeded synthetic tensors already resident in HBM.  One
JSON line goes to stdout; progress goes to stderr.
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

PEAK_FP32_MATRIX_TFLOPS = 157.3      # 256 CUs x 256 FLOP/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0
# An idle MI355X needs about 30 ms of load before its clocks stop ramping: every timed region is
# preceded by the requested warm-up launches and, if those were shorter, by more launches up to this.
WARM_MS_FLOOR = 100.0

# HBM-side bytes per launch (fetched + written), measured with rocprofv3 --pmc FETCH_SIZE and
# --pmc WRITE_SIZE (one counter per run) on this kernel and scaled by what the same counters read
# for a plain 256 MiB device copy in the same run (--copy-calibration): factor 2.000 for
# FETCH_SIZE, 1.000 for WRITE_SIZE.  Not measurable from inside this script: each figure is recorded
# together with the launch plan it was taken with (the summary with the commands is SOURCE), and is
# reported only when the plan launched now is that plan; otherwise `traffic` is null.
TRAFFIC_SOURCE = "profiles/conv_fprop_hbm_traffic_pmc.txt"
PLAN_KEYS = ("variant", "tiles", "whole", "halved", "thirded", "quartered", "eighthed", "pieces_first", "table_entries")
RECORDED_TRAFFIC = {
    "vgg":   {"bytes": 740.0e6, "plan": {"variant": "o128m128k8", "tiles": 3136, "whole": 3072, "halved": 0, "thirded": 0,
                                         "quartered": 64, "eighthed": 0, "pieces_first": 256, "table_entries": 2304}},
    "conv1": {"bytes": 265.5e6, "plan": {"variant": "o96m256", "tiles": 1513, "whole": 1513, "halved": 0, "thirded": 0,
                                         "quartered": 0, "eighthed": 0, "pieces_first": 0, "table_entries": 368}},
    "conv2": {"bytes": 291.0e6, "plan": {"variant": "o128m128k8", "tiles": 1458, "whole": 1280, "halved": 0, "thirded": 0,
                                         "quartered": 178, "eighthed": 0, "pieces_first": 256, "table_entries": 2400}},
    "conv3": {"bytes": 105.4e6, "plan": {"variant": "o128m128", "tiles": 507, "whole": 507, "halved": 0, "thirded": 0,
                                         "quartered": 0, "eighthed": 0, "pieces_first": 0, "table_entries": 2304}},
}


def recorded_traffic(workload, plan):
    """The recorded HBM bytes per launch if the launch plan is the one they were measured with, else None."""
    rec = RECORDED_TRAFFIC.get(workload)
    if rec is None or any(plan.get(k) != rec["plan"][k] for k in PLAN_KEYS):
        return None
    return rec["bytes"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_layer(torch, B, layer, d_in, d_f, out, steps, warmup, variant, min_warm_ms=0.0):
    """Events on the launch stream (torch's current stream) around `steps` launches.
    `warmup` untimed launches first, and more until `min_warm_ms` of GPU time has
    passed: the clocks of an idle GPU need tens of milliseconds of load to ramp up."""
    def launch(n):
        for _ in range(n):
            B.mdnn_conv_fprop(d_in, d_f, layer.stride, layer.pad, layer.alpha, out=out, variant=variant)
    w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    w0.record()
    launch(max(warmup, 1))
    w1.record()
    torch.cuda.synchronize()
    warm_ms = w0.elapsed_time(w1)
    if warm_ms < min_warm_ms:
        per = warm_ms / max(warmup, 1)
        launch(int((min_warm_ms - warm_ms) / max(per, 1e-3)) + 1)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    launch(steps)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def layer_report(torch, B, W, name, steps, warmup, variant=None, min_warm_ms=0.0):
    L = W.LAYERS[name] if name in W.LAYERS else W.TABLE1[name][0]
    inp, filt = W.make_inputs(L)
    d_in, d_f = torch.from_numpy(inp).cuda(), torch.from_numpy(filt).cuda()
    st, Wo, Ho = B.mdnn_out_dims(L.Wi, L.Hi, L.Sk, L.stride, L.pad)
    assert st == 0
    out = torch.empty((L.No, Ho, Wo, L.Nb), dtype=torch.float32, device="cuda")
    flops = B.mdnn_conv_flops(L.Nb, Wo, Ho, L.Nc, L.No, L.Sk)
    ev_ms, wall_ms = time_layer(torch, B, L, d_in, d_f, out, steps, warmup, variant, min_warm_ms)
    tflops = flops / (ev_ms * 1e-3) / 1e12
    nbytes = 4 * (inp.size + filt.size + out.numel())
    rep = {
        "variant": variant or B.mdnn_choose_variant(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad),
        "ms": round(ev_ms, 5), "wall_ms": round(wall_ms, 5), "steps": steps,
        "tflops": round(tflops, 3), "frac_peak": round(tflops / PEAK_FP32_MATRIX_TFLOPS, 4),
        "flops": flops, "compulsory_bytes": nbytes,
        "compulsory_GBps": round(nbytes / (ev_ms * 1e-3) / 1e9, 1),
    }
    return rep, (L, inp, filt, out)


def parity(B, W, L, inp, filt, out, variant=None):
    """Untimed check of a buffer the timed launches wrote: at least two outputs in every 16-row by
    half-tile-wide block of the launch grid (so in every tile and in every piece a tile may have
    been cut into), first and last element of each block among them, against the oracle's
    one-by-one evaluation.  Returns max |gpu - oracle| / (|alpha| * sum |x w|) and the count."""
    import numpy as np
    import oracle

    plan = B.mdnn_describe_launch(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad, variant)
    to, tm = map(int, plan["tile"].split("x"))
    No, Ho, Wo, Nb = out.shape
    idx = W.output_points((No, Nb), Ho, Wo, min(16, to), max(tm // 2, 4), 2, L.seed % 1000)
    want, absum = oracle.conv_fprop_points(inp, filt, idx, L.stride, L.pad, L.alpha)
    import torch
    t = torch.from_numpy(idx.astype(np.int64)).to(out.device)
    got = out[t[:, 0], t[:, 1], t[:, 2], t[:, 3]].cpu().numpy()
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    scale = abs(L.alpha) * absum
    zero = scale == 0
    ratio = np.zeros_like(err)
    np.divide(err, scale, out=ratio, where=~zero)
    ok = bool(np.isfinite(got).all() and (got[zero] == 0).all() and float(ratio.max()) <= 1e-4)
    return {"max_err_over_A": float(ratio.max()), "points": int(idx.shape[0]), "bound": 1e-4, "ok": ok,
            "sampling": f"2 per {min(16, to)}x{max(tm // 2, 4)} block of the No x M output, block corners included"}


def cpu_baseline(W, name):
    """The oracle as it stands on the whole layer, one pass (all output filters, all positions,
    whole batch): a few seconds on 16 host cores, about 15 s on 8."""
    import numpy as np
    import oracle

    L = W.LAYERS[name]
    inp, filt = W.make_inputs(L)
    No_s = L.No          # whole layer: a few seconds on 16 cores, ~15 s on 8
    fs = np.ascontiguousarray(filt[..., :No_s])
    Wo, Ho = oracle.out_dims(L.Wi, L.Hi, L.Sk, L.stride, L.pad)
    flops = oracle.flops(L.Nb, Wo, Ho, L.Nc, No_s, L.Sk)
    t0 = time.perf_counter()
    oracle.conv_fprop(inp, fs, L.stride, L.pad, L.alpha, want_abs=False)
    dt = time.perf_counter() - t0
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.max_threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"whole layer {name}: all {No_s} output filters, all positions, whole batch, one pass"}


def cpu_baseline_gradient(W, name, kind):
    """The oracle's gradient function on the whole layer, one pass (same role as cpu_baseline)."""
    import numpy as np
    import oracle

    L = W.LAYERS[name]
    inp, filt = W.make_inputs(L)
    Wo, Ho = oracle.out_dims(L.Wi, L.Hi, L.Sk, L.stride, L.pad)
    dout = np.random.Generator(np.random.PCG64(L.seed + 99)).standard_normal(
        size=(L.No, Ho, Wo, L.Nb), dtype=np.float32)
    flops = oracle.flops(L.Nb, Wo, Ho, L.Nc, L.No, L.Sk)
    t0 = time.perf_counter()
    if kind == "data":
        oracle.conv_bprop_data(dout, filt, (L.Hi, L.Wi), L.stride, L.pad, L.alpha, want_abs=False)
    else:
        oracle.conv_bprop_filter(inp, dout, L.Sk, L.stride, L.pad, L.alpha, want_abs=False)
    dt = time.perf_counter() - t0
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.max_threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"whole layer {name}, {kind} gradient, one pass"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="vgg", choices=["tiny", "conv1", "conv2", "conv3", "vgg"])
    ap.add_argument("--variant", default=None, help="pin a tile variant for the headline workload")
    ap.add_argument("--no-layers", action="store_true", help="skip the per-layer table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true", help="skip the register-only MFMA ceiling")
    ap.add_argument("--no-parity", action="store_true",
                    help="skip the check of the timed output buffers against the oracle (stratified points)")
    ap.add_argument("--vgg16", action="store_true",
                    help="time the nine distinct 3x3 shapes of a VGG-16 style network at minibatch 64")
    ap.add_argument("--tail-cuts", action="store_true",
                    help="time layers with 280 ... 1568 tiles of 128x128 under every way of cutting the last "
                         "partial round of tiles (pinned through the variant name) beside the library's own choice")
    ap.add_argument("--tail-map", action="store_true",
                    help="the measurement behind the tail-cut rules: layers with 1 ... 8 rounds of 256 tiles of 128x128 "
                         "plus every 32nd remainder, on two layer families, each under the library's plan and under "
                         "every pinned cut of both 128x128 kernels (about a minute)")
    ap.add_argument("--minibatch", action="store_true",
                    help="time the headline layer's geometry at minibatch sizes 4 ... 256")
    ap.add_argument("--block-sizes", action="store_true",
                    help="time the headline workload with every 16-byte tile variant: the block-size "
                         "experiment Section 3.4 of the paper asks for")
    ap.add_argument("--rotating", action="store_true",
                    help="also time the headline workload cycling through enough (in, filt, out) buffer sets "
                         "to exceed L2 + Infinity Cache (>= 1.2 GB), so no launch finds its operands cached")
    ap.add_argument("--bprop-data", action="store_true",
                    help="also time the data gradient (BPROP w.r.t. the input, computed by the FPROP kernels on "
                         "the turned-over filter bank) of the five layers; each call includes the filter "
                         "rearrangement and, for stride > 1, the gather of the residue classes")
    ap.add_argument("--bprop-filter", action="store_true",
                    help="also time the filter gradient (BPROP w.r.t. the weights) of the five layers; each call "
                         "is the partial-gradient kernel plus the kernel that sums the partials")
    ap.add_argument("--no-bprop", action="store_true",
                    help="leave the two gradients out of the per-layer table (they are timed by default, "
                         "unless --no-layers)")
    ap.add_argument("--bprop-layers", default="tiny,conv1,conv2,conv3,vgg",
                    help="comma-separated layers for --bprop-data / --bprop-filter (default: all five)")
    ap.add_argument("--sgemm", action="store_true",
                    help="time the 1x1 / stride-1 special case, which is a plain SGEMM (the calibration the "
                         "paper's conclusion leans on), next to the vendor library's fp32 matmul")
    ap.add_argument("--table1", action="store_true",
                    help="also time the ten layer shapes of the paper's Table 1 (minibatch 128, synthetic "
                         "data) and print MI355X efficiency beside the paper's GTX 980 column")
    ap.add_argument("--variant-sweep", action="store_true",
                    help="time every 16-byte tile variant on 48 layer shapes (minibatch 16 ... 128, 7x7 ... 56x56 "
                         "pixels, 96 ... 512 channels, 3x3) and report how far the library's own choice is from "
                         "the best of them")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy three times (known HBM traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU by design (one convolution on one MI355X); "
                 "run with --gpus 1")

    import torch
    from paper_1501_06633_amd import binding as B
    from paper_1501_06633_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    B.lib()
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    log(f"[bench] device={props.name} CUs={props.multi_processor_count}")

    # ---- headline: K timed steps of the named workload
    log(f"[bench] workload={args.workload} steps={args.steps} warmup={args.warmup}")
    rep, ctx = layer_report(torch, B, W, args.workload, args.steps, args.warmup, args.variant,
                          min_warm_ms=WARM_MS_FLOOR)
    L = W.LAYERS[args.workload]
    log(f"[bench] {args.workload}: {rep['ms']} ms/step, {rep['tflops']} TFLOP/s "
        f"({100 * rep['frac_peak']:.1f}% of {PEAK_FP32_MATRIX_TFLOPS}) variant={rep['variant']}")

    result = {
        "metric": "conv FPROP TFLOP/s and % of MI355X FP32 matrix peak per layer shape",
        "value": rep["tflops"], "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "warmup_ms_floor": WARM_MS_FLOOR, "ms_per_step": rep["ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, **L.dims(), "variant": rep["variant"],
                   "plan": B.mdnn_describe_launch(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad, args.variant),
                   "layout": "in CHWN, filt (C,Sk,Sk,No), out (No,Ho,Wo,Nb)"},
        "roofline": {"bound": "mfma", "achieved": rep["tflops"], "peak": PEAK_FP32_MATRIX_TFLOPS,
                     "unit": "TFLOP/s", "frac": rep["frac_peak"],
                     "traffic": None, "traffic_source": TRAFFIC_SOURCE,
                     "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE+WRITE_SIZE, copy-calibrated), recorded "
                                     "with the launch plan it was measured on; null when the plan differs",
                     "algorithmic_bytes": rep["compulsory_bytes"]},
        "frac_of_fp32_matrix_peak": rep["frac_peak"],
        "max_err_over_A": None,
        "paper_context": {"best_computational_efficiency": 0.963, "machine": "NVIDIA GTX 980 (Maxwell), Table 1",
                          "note": "another machine and another peak: context, not the target"},
    }

    result["roofline"]["traffic"] = recorded_traffic(args.workload, result["config"]["plan"])
    if not args.no_parity:
        # the buffer the timed launches wrote, checked after the clock has stopped
        _, inp_h, filt_h, out_h = ctx
        result["parity"] = parity(B, W, L, inp_h, filt_h, out_h, args.variant)
        result["max_err_over_A"] = result["parity"]["max_err_over_A"]
        log(f"[bench] parity of the timed buffer: {result['parity']}")
        if not result["parity"]["ok"]:
            sys.exit(f"bench.py: the timed output of {args.workload} does not match the oracle: {result['parity']}")

    if args.copy_calibration:
        src = torch.rand(64 * 1024 * 1024, device="cuda")          # 256 MiB read, 256 MiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        log("[bench] copy calibration: 3 x copy of 268435456 bytes")

    # ---- register-only MFMA loop: what the matrix cores sustain with no memory traffic
    if not args.no_probe:
        sink = torch.zeros(2048 * 4 * 64, device="cuda")
        for _ in range(2):
            B.mdnn_mfma_peak_probe(sink, 2048, 4, 20000)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fl = 0
        for _ in range(5):
            fl += B.mdnn_mfma_peak_probe(sink, 2048, 4, 20000)
        e1.record()
        torch.cuda.synchronize()
        ceiling = fl / (e0.elapsed_time(e1) * 1e-3) / 1e12
        result["mfma_f32_sustained_tflops"] = round(ceiling, 2)
        result["frac_of_sustained"] = round(rep["tflops"] / ceiling, 4)
        # the matrix rate with every SIMD busy and no memory traffic, read as a clock:
        # sustained FLOP/s / (CUs x 4 SIMDs x 64 FLOP per clock)
        result["mfma_clock_equivalent_ghz"] = round(ceiling * 1e12 / (256 * 4 * 64) / 1e9, 3)
        log(f"[bench] register-only FP32 MFMA loop: {ceiling:.1f} TFLOP/s sustained "
            f"(= {result['mfma_clock_equivalent_ghz']} GHz on every SIMD)")

    # ---- the headline workload launch by launch (one event pair each): median and minimum
    if not args.no_layers:
        L0, inp0, filt0, out0 = ctx
        d_in0, d_f0 = torch.from_numpy(inp0).cuda(), torch.from_numpy(filt0).cuda()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
        for _ in range(int(WARM_MS_FLOOR / max(rep["ms"], 1e-3)) + 1):
            B.mdnn_conv_fprop(d_in0, d_f0, L0.stride, L0.pad, L0.alpha, out=out0, variant=args.variant)
        for a, b in evs:
            a.record()
            B.mdnn_conv_fprop(d_in0, d_f0, L0.stride, L0.pad, L0.alpha, out=out0, variant=args.variant)
            b.record()
        torch.cuda.synchronize()
        per = sorted(a.elapsed_time(b) for a, b in evs)
        result["per_launch_ms"] = {"launches": 50, "median": round(per[25], 5), "min": round(per[0], 5),
                                   "note": "one event pair per launch; includes the gap between the two events"}
        del d_in0, d_f0

    # ---- the other layer shapes (same launch path, fewer steps)
    if not args.no_layers:
        layers = {}
        for name in W.ORDER:
            if name == args.workload and args.variant is None:
                layers[name] = rep
                continue
            steps = {"tiny": 200, "conv1": 50, "conv2": 50, "conv3": 100, "vgg": 30}[name]
            r, lctx = layer_report(torch, B, W, name, steps, 5, min_warm_ms=WARM_MS_FLOOR)
            if not args.no_parity:
                pr = parity(B, W, *lctx)
                r["max_err_over_A"], r["parity_points"] = pr["max_err_over_A"], pr["points"]
                if not pr["ok"]:
                    sys.exit(f"bench.py: the timed output of {name} does not match the oracle: {pr}")
            layers[name] = r
            log(f"[bench] {name}: {r['ms']} ms, {r['tflops']} TFLOP/s ({100 * r['frac_peak']:.1f}%) "
                f"variant={r['variant']}")
        if not args.no_parity and args.workload in layers and "parity" in result:
            layers[args.workload]["max_err_over_A"] = result["parity"]["max_err_over_A"]
            layers[args.workload]["parity_points"] = result["parity"]["points"]
        result["layers"] = {k: {kk: v[kk] for kk in ("variant", "ms", "tflops", "frac_peak", "compulsory_GBps",
                                                     "max_err_over_A", "parity_points") if kk in v}
                            for k, v in layers.items()}

    if args.block_sizes:
        rows = {}
        for v in B.mdnn_variant_names():
            if v[-1] in "sab":                               # 4-byte copies of one or both operands
                continue
            r, _ = layer_report(torch, B, W, args.workload, 30, 5, v, min_warm_ms=WARM_MS_FLOOR)
            plan = B.mdnn_describe_launch(L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad, v)
            to, tm = map(int, plan["tile"].split("x"))
            rows[v] = {"tile": plan["tile"], "tiles": plan["tiles"], "split": plan["split"],
                       "ms": r["ms"], "tflops": r["tflops"], "frac_peak": r["frac_peak"],
                       # operand bytes a workgroup pulls from L2 per FLOP it performs
                       "l2_bytes_per_flop": round(4.0 * (to + tm) / (2.0 * to * tm), 4),
                       "l2_to_lds_TBps": round(r["tflops"] * 4.0 * (to + tm) / (2.0 * to * tm), 2)}
            log(f"[bench] block {v:11s} tile {plan['tile']:8s} {r['ms']:8.4f} ms {r['tflops']:7.2f} TFLOP/s "
                f"{100 * r['frac_peak']:5.1f}%  L2->LDS {rows[v]['l2_to_lds_TBps']:.2f} TB/s")
        result["block_sizes"] = rows

    if args.minibatch:
        # the headline layer's geometry at other minibatch sizes (Section 3.4 of the paper: its kernel
        # exists for minibatches of 64 and 128 only); flat-column tiles take any multiple of 4
        rows = {}
        # 50 and 100 are not multiples of 4: those take the 4-byte-copy tiles (Table 1's caption: sizes off
        # the block size cost efficiency), and so does a filter count of No - 6 at the layer's own minibatch
        for nb, no in [(n, L.No) for n in (4, 8, 16, 32, 50, 64, 100, 128, 256)] + [(L.Nb, L.No - 6)]:
            name = f"{args.workload}_nb{nb}_no{no}"
            W.LAYERS[name] = W.custom(name, nb, L.Hi, L.Wi, L.Nc, no, L.Sk, L.stride, L.pad, L.alpha)
            r, _ = layer_report(torch, B, W, name, 30, 5, None, min_warm_ms=WARM_MS_FLOOR)
            del W.LAYERS[name]
            key = str(nb) if no == L.No else f"{nb}, No={no}"
            rows[key] = {"ms": r["ms"], "tflops": r["tflops"], "frac_peak": r["frac_peak"], "variant": r["variant"]}
            log(f"[bench] minibatch {key:>12s}: {r['ms']:8.4f} ms {r['tflops']:7.2f} TFLOP/s "
                f"{100 * r['frac_peak']:5.1f}%  variant={r['variant']}")
        result["minibatch"] = rows

    if args.rotating:
        inp, filt = W.make_inputs(L)
        st, Wo, Ho = B.mdnn_out_dims(L.Wi, L.Hi, L.Sk, L.stride, L.pad)
        set_bytes = rep["compulsory_bytes"]
        nsets = max(2, min(64, -(-1_200_000_000 // set_bytes)))
        sets = [(torch.from_numpy(inp).cuda(), torch.from_numpy(filt).cuda(),
                 torch.empty((L.No, Ho, Wo, L.Nb), dtype=torch.float32, device="cuda")) for _ in range(nsets)]

        def launch(n):
            for k in range(n):
                a, f, o = sets[k % nsets]
                B.mdnn_conv_fprop(a, f, L.stride, L.pad, L.alpha, out=o, variant=args.variant)
        launch(max(args.warmup, nsets))
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        launch(args.steps)
        e1.record()
        torch.cuda.synchronize()
        rms = e0.elapsed_time(e1) / args.steps
        result["rotating"] = {"sets": nsets, "bytes_per_set": set_bytes, "ms_per_step": round(rms, 5),
                              "tflops": round(rep["flops"] / rms / 1e9, 3),
                              "frac_peak": round(rep["flops"] / rms / 1e9 / PEAK_FP32_MATRIX_TFLOPS, 4)}
        log(f"[bench] rotating {nsets} buffer sets: {rms:.5f} ms/step, {result['rotating']['tflops']} TFLOP/s")
        del sets

    def time_gradient(kind, Lb, steps):
        """ms per call of one gradient of layer Lb (all kernels of the call), after a timed warm-up."""
        st, Wo, Ho = B.mdnn_out_dims(Lb.Wi, Lb.Hi, Lb.Sk, Lb.stride, Lb.pad)
        inp, filt = W.make_inputs(Lb)
        d_g = torch.randn((Lb.No, Ho, Wo, Lb.Nb), device="cuda")
        dims = (Lb.Nb, Lb.Wi, Lb.Hi, Lb.Nc, Lb.No, Lb.Sk, Lb.stride, Lb.pad)
        if kind == "data":
            d_f = torch.from_numpy(filt).cuda()
            res = torch.empty((Lb.Nc, Lb.Hi, Lb.Wi, Lb.Nb), device="cuda")
            st, need = B.mdnn_conv_bprop_data_workspace(*dims)
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            call = lambda: B.mdnn_conv_bprop_data(d_g, d_f, (Lb.Hi, Lb.Wi), Lb.stride, Lb.pad, Lb.alpha,
                                                  din=res, workspace=ws)
        else:
            d_in = torch.from_numpy(inp).cuda()
            res = torch.empty((Lb.Nc, Lb.Sk, Lb.Sk, Lb.No), device="cuda")
            st, need = B.mdnn_conv_bprop_filter_workspace(*dims)
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            call = lambda: B.mdnn_conv_bprop_filter(d_in, d_g, Lb.Sk, Lb.stride, Lb.pad, Lb.alpha,
                                                    dfilt=res, workspace=ws)

        def launch(n):
            for _ in range(n):
                call()
        launch(5)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); launch(10); e1.record(); torch.cuda.synchronize()
        per = e0.elapsed_time(e1) / 10
        launch(int(WARM_MS_FLOOR / max(per, 1e-3)) + 1)
        torch.cuda.synchronize()
        e0.record(); launch(steps); e1.record(); torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        # required work: every forward multiply-add has one counterpart in the gradient
        fl = B.mdnn_conv_flops(Lb.Nb, Wo, Ho, Lb.Nc, Lb.No, Lb.Sk)
        return {"ms": round(ms, 5), "tflops": round(fl / ms / 1e9, 3),
                "frac_peak": round(fl / ms / 1e9 / PEAK_FP32_MATRIX_TFLOPS, 4),
                "stride": Lb.stride, "workspace_bytes": need}

    with_table = not args.no_layers and not args.no_bprop
    do_data, do_filter = args.bprop_data or with_table, args.bprop_filter or with_table
    for kind, flag in (("data", do_data), ("filter", do_filter)):
        if not flag:
            continue
        rows = {}
        for name in [x for x in W.ORDER if x in args.bprop_layers.split(",")]:
            Lb = W.LAYERS[name]
            steps = {"tiny": 200, "conv1": 20 if kind == "data" else 100, "conv2": 50, "conv3": 100, "vgg": 30}[name]
            rows[name] = time_gradient(kind, Lb, steps)
            log(f"[bench] bprop-{kind} {name:6s} {rows[name]['ms']:9.5f} ms {rows[name]['tflops']:8.3f} TFLOP/s "
                f"({100 * rows[name]['frac_peak']:.1f}% of peak, required FLOPs) stride={Lb.stride} "
                f"workspace {rows[name]['workspace_bytes'] / 1e6:.1f} MB")
        if not args.no_cpu_baseline and args.workload in rows:
            log(f"[bench] timing the CPU oracle's {kind} gradient on {args.workload} ...")
            rows[args.workload]["cpu_baseline"] = cpu_baseline_gradient(W, args.workload, kind)
            log(f"[bench] oracle: {rows[args.workload]['cpu_baseline']}")
        for r in rows.values():
            r["roofline"] = {"bound": "mfma", "achieved": r["tflops"], "peak": PEAK_FP32_MATRIX_TFLOPS,
                             "unit": "TFLOP/s", "frac": r["frac_peak"]}
        result["bprop_" + kind] = rows

    if args.sgemm:
        # c (N x M) = a^T (N x K) . b (K x M) through the library's SGEMM entry point, which runs the
        # convolution kernel on the 1x1 geometry; the vendor library's fp32 matmul beside it
        rows = {}
        for (Mg, Ng, Kg) in [(4096, 4096, 4096), (8192, 8192, 4096), (16384, 4096, 2304)]:
            b2 = torch.rand((Kg, Mg), device="cuda") - 0.5
            a_kn = torch.randn((Kg, Ng), device="cuda") * 0.01
            c2 = torch.empty((Ng, Mg), device="cuda")

            def timed(fn, n):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(n):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / n

            ours = lambda: B.mdnn_sgemm_tn(a_kn, b2, 1.0, c=c2)
            warm = timed(ours, 5)
            timed(ours, int(WARM_MS_FLOOR / max(warm, 1e-3)) + 1)
            ms = timed(ours, 30)
            fl = 2.0 * Mg * Ng * Kg
            a2 = a_kn.t().contiguous()
            ref = torch.empty((Ng, Mg), device="cuda")
            vendor = lambda: torch.matmul(a2, b2, out=ref)
            timed(vendor, 10)
            lib_ms = timed(vendor, 30)
            same = bool(torch.allclose(c2, ref, rtol=1e-3, atol=1e-3))
            rows[f"{Ng}x{Mg}x{Kg}"] = {"ms": round(ms, 4), "tflops": round(fl / ms / 1e9, 2),
                                       "frac_peak": round(fl / ms / 1e9 / PEAK_FP32_MATRIX_TFLOPS, 4),
                                       "vendor_fp32_matmul_ms": round(lib_ms, 4),
                                       "vendor_fp32_matmul_tflops": round(fl / lib_ms / 1e9, 2),
                                       "agrees_with_vendor": same,
                                       "variant": B.mdnn_choose_variant(Mg, 1, 1, Kg, Ng, 1, 1, 0)}
            log(f"[bench] sgemm {Ng}x{Mg}x{Kg}: mdnn_sgemm_tn {ms:.4f} ms {fl / ms / 1e9:.1f} TFLOP/s | "
                f"vendor fp32 matmul {lib_ms:.4f} ms {fl / lib_ms / 1e9:.1f} TFLOP/s | agree={same}")
        result["sgemm"] = rows

    if args.table1:
        rows = {}
        for name in W.TABLE1:
            L1, paper_ce = W.TABLE1[name]
            r, _ = layer_report(torch, B, W, name, 40, 5, min_warm_ms=WARM_MS_FLOOR)
            rows[name] = {"variant": r["variant"], "ms": r["ms"], "tflops": r["tflops"],
                          "frac_peak": r["frac_peak"], "paper_gtx980_efficiency": paper_ce / 100.0}
            log(f"[bench] table1 {name:18s} {r['ms']:8.4f} ms {r['tflops']:7.2f} TFLOP/s "
                f"{100 * r['frac_peak']:5.1f}% of peak   (paper, GTX 980: {paper_ce}%)  variant={r['variant']}")
            for kind, flag in (("data", args.bprop_data), ("filter", args.bprop_filter)):
                if flag:
                    g = time_gradient(kind, L1, 5 if (kind == "data" and L1.stride > 1) else 40)
                    rows[name]["bprop_" + kind] = g
                    log(f"[bench] table1 {name:18s} bprop-{kind}: {g['ms']:8.4f} ms {g['tflops']:7.2f} TFLOP/s "
                        f"{100 * g['frac_peak']:5.1f}% of peak")
        result["table1"] = rows

    if args.variant_sweep:
        def timed(fn, n):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n
        rows, worst = {}, 0.0
        for nb in (16, 32, 64, 128):
            for hw in (7, 14, 28, 56):
                for nc, no in ((96, 256), (256, 384), (512, 512)):
                    d_in = torch.rand((nc, hw, hw, nb), device="cuda") - 0.5
                    d_f = torch.randn((nc, 3, 3, no), device="cuda") * 0.01
                    out = torch.empty((no, hw, hw, nb), device="cuda")
                    fl = B.mdnn_conv_flops(nb, hw, hw, nc, no, 3)
                    auto = B.mdnn_choose_variant(nb, hw, hw, nc, no, 3, 1, 1)
                    res = {}
                    for v in B.mdnn_variant_names():
                        if v[-1] in "sab" or v == "o64m512":             # 4-byte copies; the output-bound tile
                            continue
                        fn = lambda: B.mdnn_conv_fprop(d_in, d_f, 1, 1, 1.0, out=out, variant=v)
                        w = timed(fn, 3)
                        timed(fn, int(30.0 / max(w, 1e-3)) + 1)
                        res[v] = min(timed(fn, 10), timed(fn, 10))
                    best = min(res, key=res.get)
                    loss = res[auto] / res[best] - 1.0
                    worst = max(worst, loss)
                    name = f"nb{nb}.{hw}x{hw}.{nc}to{no}"
                    rows[name] = {"auto": auto, "auto_frac_peak": round(fl / res[auto] / 1e9 / PEAK_FP32_MATRIX_TFLOPS, 4),
                                  "best": best, "best_frac_peak": round(fl / res[best] / 1e9 / PEAK_FP32_MATRIX_TFLOPS, 4),
                                  "auto_slower_by": round(loss, 4)}
                    log(f"[bench] sweep {name:24s} auto {auto:11s} {100 * rows[name]['auto_frac_peak']:5.1f}%   "
                        f"best {best:11s} {100 * rows[name]['best_frac_peak']:5.1f}%   auto slower by {100 * loss:4.1f}%")
                    del d_in, d_f, out
        result["variant_sweep"] = {"shapes": rows, "worst_auto_slower_by": round(worst, 4)}
        log(f"[bench] sweep: the library's choice is at most {100 * worst:.1f}% slower than the best variant")

    if args.tail_cuts:
        # Section 3.4's smaller blocks, used for the last partial round of tiles only: 3x3 layers
        # with 256 input channels whose count of 128x128 tiles leaves r = 24 ... 150 tiles beyond
        # whole rounds of 256, each timed with the library's plan and with every pinned cut the two
        # 128x128 kernels offer for that r (w: none, h/t/q/e: halves, thirds, quarters, eighths,
        # m/n/p: pairings of two piece sizes per compute unit).
        def timed(fn, n):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n
        shapes = [  # name, Nb, Hi, Wi, Nc, No
            ("280 tiles (r = 24)", 128, 10, 14, 256, 256), ("338 tiles (r = 82; AlexNet-v2 conv5)", 128, 13, 13, 256, 256),
            ("352 tiles (r = 96)", 128, 11, 16, 256, 256), ("392 tiles (r = 136; VGG conv5_1)", 64, 14, 14, 512, 512),
            ("406 tiles (r = 150)", 128, 7, 29, 256, 256), ("540 tiles (2 rounds + 28)", 128, 12, 15, 256, 384),
            ("800 tiles (3 rounds + 32; Overfeat L2 geometry)", 128, 20, 20, 256, 256),
            ("1568 tiles (6 rounds + 32; VGG conv4_1)", 64, 28, 28, 256, 512)]
        rows = {}
        for name, nb, hi, wi, nc, no in shapes:
            d_in = torch.rand((nc, hi, wi, nb), device="cuda") - 0.5
            d_f = torch.randn((nc, 3, 3, no), device="cuda") * 0.01
            out = torch.empty((no, hi, wi, nb), device="cuda")
            fl = B.mdnn_conv_flops(nb, wi, hi, nc, no, 3)
            res = {}
            for v in [None] + [f"{k}:{c}" for k in ("o128m128", "o128m128k8") for c in "whtqemnp"]:
                try:
                    plan = B.mdnn_describe_launch(nb, wi, hi, nc, no, 3, 1, 1, v)
                except B.MdnnError:
                    continue                      # this kernel has no such cut for this tile count
                fn = lambda: B.mdnn_conv_fprop(d_in, d_f, 1, 1, 1.0, out=out, variant=v)
                w = timed(fn, 3)
                timed(fn, int(40.0 / max(w, 1e-3)) + 1)
                ms = min(timed(fn, 20), timed(fn, 20), timed(fn, 20))
                cut = "/".join(f"{plan[k]}{k[0]}" for k in ("halved", "thirded", "quartered", "eighthed") if plan[k]) or "uncut"
                res[v or "library"] = {"ms": round(ms, 4), "frac_peak": round(fl / ms / 1e9 / PEAK_FP32_MATRIX_TFLOPS, 4),
                                       "variant": plan["variant"], "cut": cut, "pieces_first": plan["pieces_first"]}
            rows[name] = res
            best = min(res, key=lambda k: res[k]["ms"])
            log(f"[bench] tail cuts, {name}: library = {res['library']['variant']} {res['library']['cut']} "
                f"{100 * res['library']['frac_peak']:.1f}%; best = {best} {100 * res[best]['frac_peak']:.1f}%")
            for k, r in res.items():
                log(f"[bench]     {k:14s} {r['ms'] * 1e3:8.1f} us {100 * r['frac_peak']:5.1f}%  {r['cut']}")
            del d_in, d_f, out
        result["tail_cuts"] = rows

    if args.tail_map:
        # For every tile count n = 256 R + r (R = 1 ... 8, r = 16, 48, ... 240) of two layer families
        # at minibatch 128 -- 3x3 with 128 channels and 256 filters, 5x5 with 96 channels and 256
        # filters (two filter tiles per pixel) -- the library's plan and every pinned cut.
        def timed(fn, n):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n
        def letter(p):
            h, t, q, e = p["halved"], p["thirded"], p["quartered"], p["eighthed"]
            return ("w" if not (h or t or q or e) else "n" if h and e else "m" if h and q else "p" if q and e
                    else "h" if h else "t" if t else "q" if q else "e")
        families = {"3x3, 128 -> 256": (128, 256, 3), "5x5, 96 -> 256": (96, 256, 5)}
        out_map = {}
        for fam, (nc, no, sk) in families.items():
            rows = {}
            for n in range(256 + 16, 9 * 256, 32):
                px = n // (no // 128)
                hi = next(h for h in range(int(px ** 0.5), 0, -1) if px % h == 0)
                wi = px // hi
                d_in = torch.rand((nc, hi, wi, 128), device="cuda") - 0.5
                d_f = torch.randn((nc, sk, sk, no), device="cuda") * 0.01
                out = torch.empty((no, hi, wi, 128), device="cuda")
                fl = B.mdnn_conv_flops(128, wi, hi, nc, no, sk)
                res, lib = {}, None
                for v in [None] + [f"{k}:{c}" for k in ("o128m128", "o128m128k8") for c in "whtqemnp"]:
                    try:
                        plan = B.mdnn_describe_launch(128, wi, hi, nc, no, sk, 1, sk // 2, v)
                    except B.MdnnError:
                        continue
                    if v is None:
                        lib = f"{plan['variant']}:{letter(plan)}"
                        continue                  # the library's plan is one of the pinned ones: timed once
                    fn = lambda: B.mdnn_conv_fprop(d_in, d_f, 1, sk // 2, 1.0, out=out, variant=v)
                    timed(fn, 20)
                    res[v] = round(fl / min(timed(fn, 10), timed(fn, 10)) / 1e9 / PEAK_FP32_MATRIX_TFLOPS, 4)
                best = max(res, key=res.get)
                rows[n] = {"library": lib, "library_frac_peak": res.get(lib), "best": best, "best_frac_peak": res[best], "all": res}
                log(f"[bench] tail map {fam}: n={n:5d} R={n // 256} r={n % 256:3d} library {lib:14s} "
                    f"{100 * (res.get(lib) or 0):5.1f}%  best {best:14s} {100 * res[best]:5.1f}%")
                del d_in, d_f, out
            out_map[fam] = rows
        result["tail_map"] = out_map

    if args.vgg16:
        # the nine distinct 3x3 shapes of a VGG-16 style network at minibatch 64; random data made on
        # the device (the first layers' tensors are 0.8 GB each; timing does not depend on the values)
        rows = {}
        tot_ms, tot_fl = 0.0, 0.0
        for name, Lv in W.VGG16.items():
            d_in = torch.rand((Lv.Nc, Lv.Hi, Lv.Wi, Lv.Nb), device="cuda")
            d_f = torch.randn((Lv.Nc, Lv.Sk, Lv.Sk, Lv.No), device="cuda") * 0.01
            out = torch.empty((Lv.No, Lv.Hi, Lv.Wi, Lv.Nb), device="cuda")
            ms, _ = time_layer(torch, B, Lv, d_in, d_f, out, 20, 3, None, min_warm_ms=WARM_MS_FLOOR)
            fl = B.mdnn_conv_flops(Lv.Nb, Lv.Wi, Lv.Hi, Lv.Nc, Lv.No, Lv.Sk)
            nbytes = 4 * (Lv.Nc * Lv.Hi * Lv.Wi * Lv.Nb + Lv.Nc * Lv.Sk * Lv.Sk * Lv.No + Lv.No * Lv.Hi * Lv.Wi * Lv.Nb)
            rows[name] = {"ms": round(ms, 4), "tflops": round(fl / ms / 1e9, 2),
                          "frac_peak": round(fl / ms / 1e9 / PEAK_FP32_MATRIX_TFLOPS, 4),
                          "variant": B.mdnn_choose_variant(Lv.Nb, Lv.Wi, Lv.Hi, Lv.Nc, Lv.No, Lv.Sk, Lv.stride, Lv.pad)}
            # which roof binds: FLOPs per compulsory byte against the ridge 157.3 TFLOP/s / 8 TB/s = 19.7
            if fl / nbytes < PEAK_FP32_MATRIX_TFLOPS * 1e3 / PEAK_HBM_GBS:
                gbs = nbytes / ms / 1e6
                rows[name]["roofline"] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                          "frac": round(gbs / PEAK_HBM_GBS, 4), "algorithmic_bytes": nbytes,
                                          "written_GBps": round(4 * Lv.No * Lv.Hi * Lv.Wi * Lv.Nb / ms / 1e6, 1)}
            else:
                rows[name]["roofline"] = {"bound": "mfma", "achieved": rows[name]["tflops"], "peak": PEAK_FP32_MATRIX_TFLOPS,
                                          "unit": "TFLOP/s", "frac": rows[name]["frac_peak"]}
            tot_ms += ms
            tot_fl += fl
            log(f"[bench] vgg16 {name:8s} {Lv.Nc:4d}->{Lv.No:4d} @{Lv.Hi:3d}: {ms:8.4f} ms {fl / ms / 1e9:7.2f} TFLOP/s "
                f"{100 * fl / ms / 1e9 / PEAK_FP32_MATRIX_TFLOPS:5.1f}%  variant={rows[name]['variant']}")
            del d_in, d_f, out
        rows["nine_shapes_once_each"] = {"ms": round(tot_ms, 3), "tflops": round(tot_fl / tot_ms / 1e9, 2),
                                         "frac_peak": round(tot_fl / tot_ms / 1e9 / PEAK_FP32_MATRIX_TFLOPS, 4)}
        log(f"[bench] vgg16 nine shapes once each: {tot_ms:.3f} ms, {tot_fl / tot_ms / 1e9:.1f} TFLOP/s")
        result["vgg16"] = rows

    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a bounded sample ...")
        result["cpu_baseline"] = cpu_baseline(W, args.workload)
        log(f"[bench] oracle: {result['cpu_baseline']}")

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
