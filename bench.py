#!/usr/bin/env python3
"""Benchmark of the DHQ W8A8 SIREN forward on one MI355X.

A step is one pass of the whole hot path (coordinates in, signal values out: rotation,
quantizer, int8 GEMM, dequantize + bias + sine for every layer) over one synthetic coordinate
grid that is already resident in device memory.  The workload is the largest configuration,
C5 (SIREN 2 -> 512 x 6 hidden -> 3 on a 2048 x 2048 grid); other configurations can be selected
with --workload, and the default run also times C2, C3 and C4 and reports them under
"other_workloads".  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8 MFMA peak, 5.0 POP/s
VALU_LANE_RATE = 256 * 4 * 16 * 2.4e9  # 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz fp32 lane-ops/s


# Figures stored from rocprofv3 --pmc runs of this script (profiles/ has the summaries and the commands):
# HBM bytes per launch of the fused kernel (FETCH_SIZE / WRITE_SIZE, each counter scaled by what it reads for
# a plain 256 MiB device copy in the same run), and the fraction of SIMD cycles the vector ALU and the matrix
# unit were busy.  Valid only for the kernel sources they were taken with: the hash below is compared with
# the current sources and the figures are dropped if they differ.
TRAFFIC_SOURCES = ("dhq_fused.hip", "dhq_fused_pair.hip", "dhq_fused_common.h", "dhq_device.h")
TRAFFIC_SHA256 = "65b13a8ddb13a56b6236e6b308681aa04ecb6c6338faa39a6fb6bfdb11c2315a"
TRAFFIC_BYTES = {"C2": 2593792 + 786432, "C5": 45164544 + 50331648}
COUNTER_BUSY = {"C2": {"valu": 0.655, "mfma": 0.260}, "C4": {"valu": 0.886, "mfma": 0.369}, "C5": {"valu": 0.693, "mfma": 0.437}}


def kernel_sources_sha256():
    import hashlib
    h = hashlib.sha256()
    for name in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, "paper_2508_13478_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def time_forward(model, x, out, flags, steps, warmup):
    import torch
    import paper_2508_13478_amd as dhq
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        dhq.dhq_forward(model.handle, x, out, stream, flags)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        dhq.dhq_forward(model.handle, x, out, stream, flags)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def cpu_baseline(name, max_coords, two_sided=False, wavelet_s0=None):
    """The CPU oracle's quantized forward (static scales) timed on a bounded sample."""
    import numpy as np
    from oracle import dhq_oracle as o
    from paper_2508_13478_amd import synth
    wl, coords, W, b = synth.make(name)
    stride = max(1, -(-coords.shape[0] // max_coords))
    sample = coords[::stride]
    net = o.quantize_net(wl.dims, wl.omega0, 8, 8, W, b, two_sided=two_sided, gabor_s0=wavelet_s0)
    o.forward(net, sample, calibrate=True)   # the oracle's own scales (untimed); nothing from the GPU goes into it
    # repeat the sample until about ten seconds of oracle time have been spent
    runs, t0 = 0, time.perf_counter()
    while True:
        o.forward(net, sample)
        runs += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or runs >= 50:
            break
    try:
        threads = ctypes.CDLL("libgomp.so.1").omp_get_max_threads()
    except OSError:
        threads = os.cpu_count() or 1
    return {"value": runs * sample.shape[0] / dt, "unit": "coords/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{name} grid, every {stride}th coordinate ({sample.shape[0]} coords), {runs} runs, "
                      f"{dt:.2f} s, quantized forward with static scales (weight quantization and "
                      f"calibration excluded)"}


def cpu_baseline_complex(name, max_coords, s0):
    """The CPU oracle's quantized forward of the complex-valued wavelet network (as a real network of interleaved
    features) on a bounded sample."""
    from oracle import dhq_oracle as o
    from paper_2508_13478_amd import synth
    wl, coords, _, _ = synth.make(name)
    dims_c = [wl.dims[0]] + [d // 2 for d in wl.dims[1:-1]] + [wl.dims[-1]]
    Wc, bc = synth.wire_init(dims_c, wl.omega0, wl.seed)
    dims, W, b = o.complex_net_to_real(dims_c, Wc, bc)
    stride = max(1, -(-coords.shape[0] // max_coords))
    sample = coords[::stride]
    net = o.quantize_net(dims, wl.omega0, 8, 8, W, b, gabor_s0=o.ComplexSpread(s0))
    o.forward(net, sample, calibrate=True)
    runs, t0 = 0, time.perf_counter()
    while True:
        o.forward(net, sample)
        runs += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or runs >= 50:
            break
    try:
        threads = ctypes.CDLL("libgomp.so.1").omp_get_max_threads()
    except OSError:
        threads = os.cpu_count() or 1
    return {"value": runs * sample.shape[0] / dt, "unit": "coords/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{name} grid, every {stride}th coordinate ({sample.shape[0]} coords), {runs} runs, {dt:.2f} s, "
                      f"quantized forward with static scales"}


def cpu_baseline_float(name, max_coords, wavelet_s0=None):
    """The CPU oracle's plain fp64/fp32 MLP timed on a bounded sample."""
    from oracle import dhq_oracle as o
    from paper_2508_13478_amd import synth
    wl, coords, W, b = synth.make(name)
    stride = max(1, -(-coords.shape[0] // max_coords))
    sample = coords[::stride]
    runs, t0 = 0, time.perf_counter()
    while True:
        o.mlp_float(wl.dims, wl.omega0, W, b, sample, gabor_s0=wavelet_s0)
        runs += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or runs >= 50:
            break
    try:
        threads = ctypes.CDLL("libgomp.so.1").omp_get_max_threads()
    except OSError:
        threads = os.cpu_count() or 1
    return {"value": runs * sample.shape[0] / dt, "unit": "coords/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{name} grid, every {stride}th coordinate ({sample.shape[0]} coords), {runs} runs, {dt:.2f} s, "
                      f"plain MLP evaluated in fp64 and fp32 side by side"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C5")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the extra timings of C2, C3 and C4 that the default run adds to its line")
    ap.add_argument("--variant", default="base", choices=["base", "two_sided", "dynamic", "two_sided_dynamic", "w8a32", "w32a32"],
                    help="base: input-side rotation, static scales (fused kernel where there is one); "
                         "two_sided: weights rotated on both sides, un-rotation in int32; "
                         "dynamic / two_sided_dynamic: activation scales measured on line per call (one fused kernel "
                         "per layer where there is one); "
                         "w8a32 / w32a32: the comparison networks with fp32 activations (fused fp32 kernel)")
    ap.add_argument("--activation", default="sine", choices=["sine", "wavelet", "wavelet_complex"],
                    help="sine: the SIREN of the workload; wavelet: the same shapes and weights with the activation "
                         "cos(omega0 y) exp(-(s0 y)^2) of the second architecture the paper evaluates (same fused kernels); "
                         "wavelet_complex: that architecture with complex-valued hidden layers of half the workload's "
                         "width (the same real width, seeded complex weights), base variant only")
    ap.add_argument("--wavelet-s0", type=float, default=10.0, help="spread of the wavelet's Gaussian envelope")
    ap.add_argument("--path", default="auto", choices=["auto", "layerwise"],
                    help="auto: the fused kernel where the model has one; layerwise: force the layer-by-layer path")
    ap.add_argument("--wide-kernel", type=int, default=0, choices=[0, 1, 2],
                    help="hidden width 512 only: 0 the library's default whole-network kernel, 1 the one with one wave "
                         "per SIMD, 2 the one with two waves per SIMD that split the features")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-coords", type=int, default=32768, help="cap of the CPU-baseline sample")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this benchmark runs on one GPU; --gpus must be 1 (the coordinate grid shards "
              "trivially, but no multi-GPU path is part of it)", file=sys.stderr)
        return 2

    import torch
    import paper_2508_13478_amd as dhq
    from paper_2508_13478_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)
    wl, coords, W, b = synth.make(args.workload)
    two_sided = args.variant.startswith("two_sided")
    dynamic = args.variant.endswith("dynamic")
    floating = args.variant in ("w8a32", "w32a32")
    mode = dhq.DHQ_ROTATE_BOTH if two_sided else dhq.DHQ_ROTATE_IN
    if floating:
        mode = dhq.DHQ_W8A32 if args.variant == "w8a32" else dhq.DHQ_W32A32
    s0 = args.wavelet_s0 if args.activation == "wavelet" else None
    cplx = args.activation == "wavelet_complex"
    if cplx:
        if args.variant != "base":
            print("bench.py: --activation wavelet_complex runs the base variant only", file=sys.stderr)
            return 2
        dims_c = [wl.dims[0]] + [d // 2 for d in wl.dims[1:-1]] + [wl.dims[-1]]
        Wc, bc = synth.wire_init(dims_c, wl.omega0, wl.seed)
        model = dhq.Model.complex_wavelet(dims_c, wl.omega0, Wc, bc, args.wavelet_s0, 8, 8)
    else:
        model = dhq.Model(wl.dims, wl.omega0, W, b, 8, 8, mode=mode, wavelet_s0=s0)
    if args.wide_kernel:
        model.select_wide_kernel(args.wide_kernel)
    x = torch.from_numpy(coords).to("cuda")
    out = torch.empty((x.shape[0], wl.dims[-1]), dtype=torch.float32, device="cuda")
    if not floating:
        model.calibrate(x)
    fused = model.has_fused() and not dynamic and args.path == "auto"
    flags = dhq.DHQ_FUSED if fused else dhq.DHQ_LAYERWISE
    # dynamic scales: one fused kernel per layer where the library has a whole-network kernel (two-sided: up to
    # hidden width 256), the layer-by-layer kernels otherwise or with --path layerwise
    dyn_fused = dynamic and args.path == "auto" and model.has_fused()
    if dynamic:
        flags = (dhq.DHQ_FUSED if dyn_fused else dhq.DHQ_LAYERWISE) | dhq.DHQ_DYNAMIC

    ms, wall_ms = time_forward(model, x, out, flags, args.steps, args.warmup)
    n = x.shape[0]
    ops = wl.int8_ops_per_coord() * n
    tops = ops / (ms * 1e-3) / 1e12
    res = {
        "metric": "W8A8 SIREN forward coords/sec",
        "value": n / (ms * 1e-3),
        "unit": "coords/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "i8",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: SIREN {'-'.join(map(str, wl.dims))}, omega0={wl.omega0:g}, "
                               f"{wl.side}x{wl.side} grid ({n} coords), W8A8, static per-layer scales "
                               f"from absmax calibration on the same grid",
                   "path": "fused" if fused else "layerwise", "variant": args.variant, "coords": n},
        "int8_tops": tops,
        "pct_int8_mfma_peak": 100.0 * tops / INT8_MFMA_PEAK_TOPS,
        "wall_ms_per_step": wall_ms,
        # dominant kernel = the fused whole-network kernel: one launch per step, so its average
        # duration is the event-timed step; algorithmic work = 2 ops per MAC over the un-padded
        # layer shapes
        "roofline": {"bound": "mfma", "achieved": tops, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": tops / INT8_MFMA_PEAK_TOPS,
                     "traffic": (TRAFFIC_BYTES.get(wl.name) if fused and not two_sided and s0 is None and not cplx and args.wide_kernel != 1
                                 and kernel_sources_sha256() == TRAFFIC_SHA256
                                 else None),
                     "traffic_unit": "HBM bytes per launch, stored from the rocprofv3 --pmc runs summarised in "
                                     "profiles/dhq_fused_hbm_traffic_pmc.md (null when the kernel sources have changed since)",
                     "kernel": ((f"dhq_fused2_kernel<{wl.dims[1]}>" if two_sided else
                                 (f"dhq_fused_wide_kernel<512, {2 if s0 is not None else 1}>" if args.wide_kernel == 1 else
                                  f"dhq_fused_pair_kernel<{2 if s0 is not None else 1}>") if wl.dims[1] == 512 else
                                 f"dhq_fused_kernel<{wl.dims[1]}, {2 if s0 is not None else 1}>")
                                if fused else "layerwise kernels"),
                     "algorithmic_hbm_bytes_per_launch": 4 * (wl.dims[0] + wl.dims[-1]) * n,
                     "algorithmic_ops_per_launch": ops},
    }
    # Secondary view: the vector ALU, which is what actually limits this path.  Per feature and
    # sine layer the fused kernels issue convert, fma, sine, the transform, fma, median, and three
    # byte-permute/or instructions per four codes.  The
    # transform: the fused kernels give its 32-row factor to the matrix unit (two vector
    # instructions to split an activation into binary16 pieces) and keep log2(n / 32) add/sub
    # (the one-wave width-512 kernel: plus one move out of the accumulation registers).
    # A SIMD issues one wave64 vector instruction per 4 clocks, i.e. 256 CUs x 4 SIMDs x 2.4 GHz / 4
    # per second.
    import math
    nf = wl.dims[1]
    per_feature = 3 + 2 + math.log2(nf / 32) + (1 if nf == 512 and args.wide_kernel == 1 else 0) + 2.75
    if two_sided:
        per_feature += math.log2(nf) + 0.5   # the integer un-rotation: log2(n) add/sub and half a lane swap
    lane_instr = sum(wl.dims[l + 1] for l in range(len(wl.dims) - 2)) * per_feature * n
    valu_peak = 256 * 4 * 2.4e9 / 4
    res["alu"] = {"bound": "alu", "achieved": lane_instr / 64 / (ms * 1e-3), "peak": valu_peak,
                  "unit": "wave64 instr/s", "frac": lane_instr / 64 / (ms * 1e-3) / valu_peak,
                  "model": f"{per_feature:.1f} vector instructions per feature and sine layer"}
    if fused and not two_sided and s0 is None and not cplx and args.wide_kernel != 1 and kernel_sources_sha256() == TRAFFIC_SHA256:
        busy = COUNTER_BUSY.get(wl.name)
        if busy:
            res["alu"]["counter_valu_busy_frac"] = busy["valu"]
            res["alu"]["counter_mfma_busy_frac"] = busy["mfma"]
            res["alu"]["counter_source"] = "stored from the rocprofv3 --pmc run summarised in profiles/dhq_fused_utilisation_pmc.md"
    if floating:
        # fp32 activations: the same multiply-adds on the fp32 MFMA (157.3 TFLOP/s dense)
        tf = ops / (ms * 1e-3) / 1e12
        res["metric"] = "fp32-activation SIREN forward coords/sec"
        res["dtype"] = "f32"
        res["config"]["workload"] = res["config"]["workload"].replace("W8A8, static per-layer scales from absmax calibration on the same grid", args.variant.upper())
        res.pop("int8_tops"); res.pop("pct_int8_mfma_peak"); res.pop("alu")
        res["roofline"] = {"bound": "mfma", "achieved": tf, "peak": 157.3, "unit": "TFLOP/s", "frac": tf / 157.3,
                           "traffic": None,
                           "kernel": (f"dhq_float_kernel<{wl.dims[1]}>" if fused else "float_layer_kernel, all launches of one forward"),
                           "algorithmic_hbm_bytes_per_launch": 4 * (wl.dims[0] + wl.dims[-1]) * n,
                           "algorithmic_ops_per_launch": ops}
    if not fused and not floating:
        # The layer-by-layer path is bound by device-memory traffic: per coordinate and layer the
        # transform reads 4 K bytes (twice when the scale is measured on line) and writes Kp codes,
        # the GEMM reads them and writes 4 M bytes of activations (two-sided: 4 Mp of accumulators,
        # which the un-rotation kernel reads back before it writes the 4 M).
        def p2(k):
            return 1 << (k - 1).bit_length() if k > 1 else 1
        per_coord = 0
        for l in range(len(wl.dims) - 1):
            K, M = wl.dims[l], wl.dims[l + 1]
            per_coord += 4 * K * (2 if dynamic else 1) + 2 * p2(K) + 4 * M + (8 * p2(M) if two_sided else 0)
        if two_sided and not dynamic:
            # static scales: a layer's un-rotation kernel also rotates and quantizes the next layer's input, so only
            # the coordinates, codes and rotated accumulators cross device memory
            nl = len(wl.dims) - 1
            per_coord = 4 * wl.dims[0] + p2(wl.dims[0])
            for l in range(nl):
                K, M = wl.dims[l], wl.dims[l + 1]
                per_coord += p2(K) + 8 * p2(M) + (p2(M) if l < nl - 1 else 4 * M)
        if dyn_fused:
            # one kernel per layer: the coordinates are read twice (scale of the input layer, then the layer),
            # every hidden boundary is one write and one read of the transformed activations (fp32)
            per_coord = 2 * 4 * wl.dims[0] + 4 * wl.dims[-1] + sum(2 * 4 * p2(k) for k in wl.dims[1:-1])
            res["config"]["path"] = "one fused kernel per layer"
        gbs = per_coord * n / (ms * 1e-3) / 1e9
        res["roofline"] = {"bound": "hbm", "achieved": gbs, "peak": 8000.0, "unit": "GB/s", "frac": gbs / 8000.0,
                           "traffic": None,
                           "kernel": (("dhq_fused2_layer_kernel" if two_sided else
                                       "dhq_fused_pair_layer_kernel" if wl.dims[1] == 512 else "dhq_fused_layer_kernel") +
                                      ", all launches of one forward" if dyn_fused
                                      else "layer-by-layer path, all kernels of one forward"),
                           "algorithmic_hbm_bytes_per_launch": per_coord * n,
                           "algorithmic_ops_per_launch": ops}
        res.pop("alu", None)
    if fused and not floating:
        ms_lw, _ = time_forward(model, x, out, dhq.DHQ_LAYERWISE, max(10, args.steps // 20), 5)
        res["layerwise_ms_per_step"] = ms_lw
    if not floating and not two_sided and not dynamic and not cplx:
        # the paper's W32A32-versus-W8A8 comparison (Table 2) on this GPU: the plain fp32 network through
        # the library's own fp32 kernels (one fused kernel up to width 256, layer by layer beyond), and how
        # far the quantized output is from it
        ref_model = dhq.Model(wl.dims, wl.omega0, W, b, 8, 8, mode=dhq.DHQ_W32A32, wavelet_s0=s0)
        ref_out = torch.empty_like(out)
        ms_f, _ = time_forward(ref_model, x, ref_out, dhq.DHQ_AUTO, max(10, args.steps // 20), 5)
        dhq.dhq_forward(model.handle, x, out, torch.cuda.current_stream(), flags)
        torch.cuda.synchronize()
        mse = float(((out.double() - ref_out.double()) ** 2).mean())
        peak = float(ref_out.max() - ref_out.min())
        res["w32a32_ms_per_step"] = ms_f
        res["w32a32_path"] = "fused" if ref_model.has_fused() else "layer by layer"
        res["speedup_vs_w32a32"] = ms_f / ms
        res["psnr_vs_w32a32_db"] = 10.0 * math.log10(peak * peak / mse) if mse > 0 else float("inf")
        ref_model.close()
    if args.workload == "C5" and args.variant == "base" and s0 is None and args.path == "auto" and not args.no_other_workloads:
        # the smaller configurations on the same kernels, for the record (not the headline)
        others = {}
        for name, steps in (("C2", 2000), ("C3", 400), ("C4", 100)):
            wl2, coords2, W2, b2 = synth.make(name)
            m2 = dhq.Model(wl2.dims, wl2.omega0, W2, b2, 8, 8)
            x2 = torch.from_numpy(coords2).to("cuda")
            out2 = torch.empty((x2.shape[0], wl2.dims[-1]), dtype=torch.float32, device="cuda")
            m2.calibrate(x2)
            ms2, _ = time_forward(m2, x2, out2, dhq.DHQ_FUSED, steps, 10)
            tops2 = wl2.int8_ops_per_coord() * x2.shape[0] / (ms2 * 1e-3) / 1e12
            others[name] = {"ms_per_step": ms2, "coords_per_s": x2.shape[0] / (ms2 * 1e-3), "int8_tops": tops2,
                            "frac_int8_mfma_peak": tops2 / INT8_MFMA_PEAK_TOPS, "steps": steps, "coords": x2.shape[0],
                            "dims": list(wl2.dims)}
            m2.close()
            del x2, out2
        res["other_workloads"] = others
    if cplx:
        res["config"]["workload"] = res["config"]["workload"].replace(
            "SIREN", f"complex-valued wavelet MLP (s0={args.wavelet_s0:g}, {wl.dims[1] // 2} complex features per hidden layer), real dims")
        res["config"]["activation"] = "wavelet_complex"
        res["metric"] = res["metric"].replace("SIREN", "complex-wavelet-MLP")
        res["roofline"]["traffic"] = None
        if fused:
            res["roofline"]["kernel"] = "dhq_fused_pair_kernel<3>" if wl.dims[1] == 512 else f"dhq_fused_kernel<{wl.dims[1]}, 3>"
        res["alu"]["model"] += " (sine model; the complex wavelet takes 4.5 instructions per value where the sine takes 1)"
    if s0 is not None:
        res["config"]["workload"] = res["config"]["workload"].replace("SIREN", f"wavelet MLP (s0={s0:g})")
        res["config"]["activation"] = "wavelet"
        res["metric"] = res["metric"].replace("SIREN", "wavelet-MLP")
    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline and cplx:
        res["cpu_baseline"] = cpu_baseline_complex(args.workload, args.cpu_coords, args.wavelet_s0)
    elif not args.no_cpu_baseline:
        res["cpu_baseline"] = (cpu_baseline_float(args.workload, args.cpu_coords, s0) if floating else
                               cpu_baseline(args.workload, args.cpu_coords, two_sided, s0))
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
