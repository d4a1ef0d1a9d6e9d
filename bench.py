#!/usr/bin/env python3
"""Benchmark of the ConvLinear4bit forward path on one MI355X.

A step is one pass of the whole hot path - rotate + quantise + pack the activations, W4A4 GEMM,
dequantise to bf16 (`convlinear4bit_forward`, weights prepared beforehand as the paper does
offline) - over one batch of synthetic input of the headline shape M4608 x K3072 x N12288, g = 16.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--calibrate-copy]

--calibrate-copy additionally runs a plain device-to-device copy of known size, so that a
rocprofv3 --pmc run of this command holds the reference the HBM byte counters are scaled by.
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

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
FP6_MFMA_PEAK_TOPS = 10100.0  # MI355X dense FP6 MFMA, published (the GEMM's operand type)
I8_MFMA_PEAK_TOPS = 5000.0    # MI355X dense int8 MFMA, published (the figure the build's target is phrased in)

# HBM bytes per launch of the headline shape from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per
# dispatch), each scaled by what the same counter reads for a plain copy of known size (x2.0 and
# x1.0); the runs are in profiles/gemm_w4a4_and_rotquant_headline_hbm_traffic_and_mfma_busy.md.
# These are stored measurements, not taken live (bench.py cannot run the profiler on itself): TRAFFIC_SOURCE
# says which build of the kernels they were taken on.
MEASURED_TRAFFIC_BYTES = {"gemm_w4a4_kernel": 83177 * 1024 * 2.0 + 110613 * 1024 * 1.0,
                          "rotquant_kernel": 13883 * 1024 * 2.0 + 10386 * 1024 * 1.0}
TRAFFIC_SOURCE = ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of `python bench.py --calibrate-copy`, library version 500 "
                  "(kernel sources as of commit 1f837fa); see profiles/")
# What a register-only loop of the GEMM's MFMA sustains on this chip on operands with the workload's bit
# statistics (8 wavefronts per compute unit, no memory traffic; 9.9 POP/s on all-zero operands): the chip lowers its
# clock with operand activity, so this, not the nominal figure, is what a perfect kernel could reach on this data.
MEASURED_FP6_MFMA_LOOP_TOPS = 6600.0
MFMA_LOOP_SOURCE = "register-only v_mfma_f32_32x32x64_f8f6f4 loop on workload-like FP6 operands, MI355X of this pool"
PREWARM_MS = 200.0           # load put on the device before anything is timed, whatever --warmup says
COPY_BYTES = 512 << 20       # size of the calibration copy (--calibrate-copy)
COLD_FOOTPRINT = 768 << 20   # kernel A, cold: bytes touched between two uses of one buffer set


def time_region(fn, steps: int, torch, stream) -> float:
    """Milliseconds per call: HIP events on the stream the kernels are launched on."""
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(steps):
        fn()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) / steps


def time_region_chunks(fn, steps: int, torch, stream, chunks: int = 10):
    """As time_region, with an event recorded after every steps / chunks calls as well (recording syncs nothing): returns
    (ms per call over the whole region, median and minimum of the per-chunk ms per call)."""
    chunks = max(1, min(chunks, steps))
    bounds = [steps * c // chunks for c in range(chunks + 1)]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(chunks + 1)]
    ev[0].record(stream)
    for c in range(chunks):
        for _ in range(bounds[c + 1] - bounds[c]):
            fn()
        ev[c + 1].record(stream)
    ev[-1].synchronize()
    per = sorted(ev[c].elapsed_time(ev[c + 1]) / (bounds[c + 1] - bounds[c]) for c in range(chunks))
    return ev[0].elapsed_time(ev[-1]) / steps, per[len(per) // 2], per[0]


def cpu_baseline(spec, x_bits, w_bits, budget_s: float = 15.0):
    """The oracle, untuned, on the host cores: same forward (weights prepared untimed) on a row sample."""
    import numpy as np
    import oracle

    qw, sw = oracle.rotquant(w_bits, spec.group)          # offline in the paper: not timed
    probe = min(128, spec.M)

    def fwd(rows_bits):
        qx, sx = oracle.rotquant(rows_bits, spec.group)
        return oracle.dequant(oracle.int_gemm(qx, qw), sx, sw)

    t0 = time.perf_counter()
    fwd(x_bits[:probe])
    t_probe = time.perf_counter() - t0
    rows = int(min(spec.M, max(probe, budget_s / max(t_probe, 1e-6) * probe)))
    passes = int(max(1, min(8, budget_s / max(t_probe / probe * rows, 1e-6))))
    t0 = time.perf_counter()
    for _ in range(passes):
        fwd(x_bits[:rows])
    dt = (time.perf_counter() - t0) / passes
    tops = 2.0 * rows * spec.K * spec.N / dt / 1e12
    return {"value": tops, "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {rows} of {spec.M} token rows, all {spec.N} output channels, mean of {passes} "
                      f"passes ({dt:.2f} s each; rotate+quantise, int GEMM, dequant; weight prep untimed)",
            "ms_per_step": dt / rows * spec.M * 1e3}


def measure_layer(spec, cr, wl, torch, np, steps: int, warmup: int, bits: int = 4):
    """Kernel A, kernel B, the fused forward and the offline weight preparation of one layer (ms, rates); bits = 8:
    the W8A8 variant of the layer (int8 codes, int8 MFMA)."""
    stream = torch.cuda.current_stream()
    M, K, N, g = spec.M, spec.K, spec.N, spec.group
    prepare, rotquant, gemm, forward, wsbytes = (
        (cr.convrot_prepare_weight, cr.convrot_rotquant_act, cr.convrot_w4a4_gemm_dequant, cr.convlinear4bit_forward,
         cr.workspace_bytes) if bits == 4 else
        (cr.convrot_prepare_weight8, cr.convrot_rotquant_act8, cr.convrot_w8a8_gemm_dequant, cr.convlinear8bit_forward,
         cr.workspace_bytes8))
    x_bits, w_bits = wl.make_layer(spec)
    X = torch.from_numpy(x_bits.view(np.int16)).cuda().view(torch.bfloat16)
    W = torch.from_numpy(w_bits.view(np.int16)).cuda().view(torch.bfloat16)
    Wq, Ws = prepare(W, g)
    Xq, Xs = rotquant(X, g)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty((wsbytes(M, K),), dtype=torch.uint8, device="cuda")
    fns = {"forward": lambda: forward(X, Wq, Ws, g, Y, ws),
           "gemm": lambda: gemm(Xq, Xs, Wq, Ws, K, Y),
           "rotquant": lambda: rotquant(X, g, Xq, Xs),
           "prepare_weight": lambda: prepare(W, g, Wq, Ws)}
    for _ in range(warmup):
        fns["forward"]()
    ms = {}
    for name, fn in fns.items():
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        ms[name] = time_region(fn, steps, torch, stream)
    torch.cuda.synchronize()
    code_bytes = 0.75 if bits == 4 else 1.0
    ops, bytes_a, bytes_w = 2.0 * M * K * N, (2.0 + code_bytes) * M * K + 4.0 * M, (2.0 + code_bytes) * N * K + 4.0 * N
    out = {"layer": spec.name, "M": M, "K": K, "N": N, "group": g,
           "forward_ms": ms["forward"], "forward_TOPS": ops / ms["forward"] / 1e9,
           "gemm_ms": ms["gemm"], "gemm_TOPS": ops / ms["gemm"] / 1e9}
    if bits == 4:
        out["gemm_frac_fp6_mfma_peak"] = ops / ms["gemm"] / 1e9 / FP6_MFMA_PEAK_TOPS
        out["gemm_vs_i8_mfma_peak"] = ops / ms["gemm"] / 1e9 / I8_MFMA_PEAK_TOPS
    else:
        out["gemm_frac_i8_mfma_peak"] = ops / ms["gemm"] / 1e9 / I8_MFMA_PEAK_TOPS
    out.update({"rotquant_ms_warm": ms["rotquant"], "rotquant_GB/s_warm": bytes_a / ms["rotquant"] / 1e6,
                "rotquant_frac_hbm_peak_warm": bytes_a / ms["rotquant"] / 1e6 / HBM_PEAK_GBS,
                "prepare_weight_ms": ms["prepare_weight"], "prepare_weight_GB/s": bytes_w / ms["prepare_weight"] / 1e6})
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--all-configs", action="store_true",
                    help="also time every layer of the five benchmark configurations and the next-row layers (adds a "
                         "'configs' list) and the W8A8 variant on four of them ('configs_w8a8')")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (token rows are independent, so the path would shard over "
              "tokens without any exchange); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2512_03673_amd import binding as cr
    from paper_2512_03673_amd import workloads as wl

    cr.load()  # raises if the HIP library is not built: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    spec = wl.HEADLINE
    M, K, N, g = spec.M, spec.K, spec.N, spec.group
    x_bits, w_bits = wl.make_layer(spec)

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    X, W = dev(x_bits), dev(w_bits)
    Wq, Ws = cr.convrot_prepare_weight(W, g)
    del W
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty((cr.workspace_bytes(M, K),), dtype=torch.uint8, device="cuda")
    Xq = torch.empty((cr.packed_bytes(M, K),), dtype=torch.uint8, device="cuda")
    Xs = torch.empty((M,), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        cr.convlinear4bit_forward(X, Wq, Ws, g, Y, ws)

    # The clocks of an idle MI355X need tens of milliseconds of load to settle (the first hundred launches run
    # a quarter slower): load the device for PREWARM_MS before the warm-up steps the caller asked for.
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < PREWARM_MS:
        for _ in range(50):
            step()
        torch.cuda.synchronize()
    prewarm_ms = (time.perf_counter() - t0) * 1e3
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms_step, ms_step_median, ms_step_min = time_region_chunks(step, args.steps, torch, stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-kernel durations, same launch configuration, same stream
    def kern_a():
        cr.convrot_rotquant_act(X, g, Xq, Xs)

    def kern_b():
        cr.convrot_w4a4_gemm_dequant(Xq, Xs, Wq, Ws, K, Y)

    for _ in range(max(5, args.warmup // 4)):
        kern_a(); kern_b()
    torch.cuda.synchronize()
    ms_b, ms_b_median, ms_b_min = time_region_chunks(kern_b, args.steps, torch, stream)
    ms_a = time_region(kern_a, args.steps, torch, stream)
    torch.cuda.synchronize()

    # kernel A again with nothing of its working set left in the 256 MB Infinity Cache: a ring of
    # buffer sets, COLD_FOOTPRINT bytes touched between two uses of the same set
    bytes_a = 2.75 * M * K + 4.0 * M         # bf16 in, 6-bit code out, one fp32 scale per row
    nset = int(COLD_FOOTPRINT // bytes_a) + 1
    ring = [(X.clone(), torch.empty_like(Xq), torch.empty_like(Xs)) for _ in range(nset)]
    state = {"i": 0}

    def kern_a_cold():
        x, q, sc = ring[state["i"] % nset]
        state["i"] += 1
        cr.convrot_rotquant_act(x, g, q, sc)

    for _ in range(nset):
        kern_a_cold()
    torch.cuda.synchronize()
    ms_a_cold = time_region(kern_a_cold, max(args.steps, 2 * nset), torch, stream)
    torch.cuda.synchronize()
    del ring

    if args.calibrate_copy:
        src = torch.empty((COPY_BYTES,), dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    ops = 2.0 * M * K * N
    tops_step = ops / (ms_step * 1e-3) / 1e12
    tops_b = ops / (ms_b * 1e-3) / 1e12
    gbs_a = bytes_a / (ms_a * 1e-3) / 1e9
    gbs_a_cold = bytes_a / (ms_a_cold * 1e-3) / 1e9
    bytes_a_nibble = 2.5 * M * K + 4.0 * M    # what the same pass would move with two codes per byte
    bytes_b_min = 0.75 * M * K + 0.75 * N * K + 4.0 * (M + N) + 2.0 * M * N

    out = {
        "metric": "ConvLinear4bit forward throughput at M4608xK3072xN12288 (rotate+quantise+W4A4 GEMM+dequant)",
        "value": tops_step, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp6", "data": "synthetic",
        "config": {"workload": "cfg3_mlp/mlp_up: FLUX-style MLP up-projection", "M": M, "K": K, "N": N,
                   "group": g, "codes": "4-bit integers stored as FP6 E2M3, FP6 MFMA with exact fp32 accumulation, bf16 in/out",
                   "weights": "prepared offline (convrot_prepare_weight), not timed"},
        "ms_per_step_median_of_tenths": ms_step_median, "ms_per_step_min_of_tenths": ms_step_min,
        "wall_ms_per_step": wall_ms, "prewarm_ms": prewarm_ms, "build": cr.build_info(),
        "kernels": {
            "rotquant_act": {"ms_cold": ms_a_cold, "GB/s_cold": gbs_a_cold, "frac_hbm_peak_cold": gbs_a_cold / HBM_PEAK_GBS,
                             "ms_warm": ms_a, "GB/s_warm": gbs_a, "frac_hbm_peak_warm": gbs_a / HBM_PEAK_GBS,
                             "algorithmic_bytes": bytes_a,
                             "frac_hbm_peak_cold_at_2.5B_per_elem": bytes_a_nibble / (ms_a_cold * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "traffic": MEASURED_TRAFFIC_BYTES["rotquant_kernel"], "traffic_source": TRAFFIC_SOURCE,
                             "note": f"cold: {nset} buffer sets in rotation ({COLD_FOOTPRINT >> 20} MiB between reuses); "
                                     "warm: one set, its 35 MB fit the 256 MB Infinity Cache"},
            "w4a4_gemm_dequant": {"ms": ms_b, "ms_median_of_tenths": ms_b_median, "ms_min_of_tenths": ms_b_min, "TOPS": tops_b, "frac_fp6_mfma_peak": tops_b / FP6_MFMA_PEAK_TOPS,
                                  "vs_i8_mfma_peak": tops_b / I8_MFMA_PEAK_TOPS,
                                  "min_bytes": bytes_b_min},
        },
        "roofline": {"kernel": "gemm_w4a4_kernel", "bound": "mfma", "achieved": tops_b, "peak": FP6_MFMA_PEAK_TOPS,
                     "unit": "TOP/s", "frac": tops_b / FP6_MFMA_PEAK_TOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES["gemm_w4a4_kernel"], "traffic_source": TRAFFIC_SOURCE,
                     "frac_vs_measured_peak": tops_b / MEASURED_FP6_MFMA_LOOP_TOPS,
                     "measured_peak": MEASURED_FP6_MFMA_LOOP_TOPS, "measured_peak_source": MFMA_LOOP_SOURCE},
    }
    if args.all_configs:
        del X, Wq, Ws, Y, ws, Xq, Xs
        out["configs"] = [dict(config=name, **measure_layer(sp, cr, wl, torch, np, min(args.steps, 100), min(args.warmup, 100)))
                          for name, layers in list(wl.CONFIGS.items()) + list(wl.NEXT_CONFIGS.items()) for sp in layers]
        # the W8A8 variant of the layer (int8 codes on the int8 MFMA) on the large FLUX shapes
        w8 = [sp for name, layers in list(wl.CONFIGS.items()) + list(wl.NEXT_CONFIGS.items()) for sp in layers
              if sp.name in ("mlp_up", "mlp_down", "hires_down", "fused_out")]
        out["configs_w8a8"] = [measure_layer(sp, cr, wl, torch, np, min(args.steps, 100), min(args.warmup, 100), bits=8)
                               for sp in w8]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(spec, x_bits, w_bits)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
