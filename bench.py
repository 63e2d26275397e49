#!/usr/bin/env python3
"""Benchmark of the fused W4A4 + low-rank linear layer (arXiv 2411.05007, Eq. 5) on one MI355X.

One "step" is one pass of the whole hot path - activation kernel (smooth + INT4 quantize + down
projection) and W4A4 GEMM (with up projection, bias and bf16 store) - over one batch of synthetic
FLUX-MLP-shaped input (M=4608, K=3072, N=12288, r=32) already resident in HBM.

`--format fp4` and `--format w8a8` time the MXFP4 variant and the 8-bit setting of the same layer instead (their GEMMs
against the FP4 and INT8 MFMA peaks), `--lora R` appends an adapter first; the default line is the INT4 metric.

Prints ONE JSON line with the headline metric (TOPS of the 4-bit branch, 2*M*N*K per layer time),
the roofline of the dominant kernel (the GEMM, against the INT8 MFMA peak) measured live with HIP
events on the stream the kernels run on, and the CPU oracle timed on a bounded row sample.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0       # MI355X dense INT8, published
FP4_MFMA_PEAK_TFLOPS = 10100.0     # MI355X dense FP4 / FP6, published
HBM_PEAK_GBS = 8000.0

# HBM-side traffic of one GEMM launch at the headline shape from `rocprofv3 --pmc FETCH_SIZE` /
# `--pmc WRITE_SIZE` (profiles/flux_mlp_up_kernel_stats.md), each scaled by what the same counter
# reads for a plain 256 MiB copy (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0): 301.6 MB read + 113.2 MB written.
GEMM_TRAFFIC_BYTES = 414.9e6


class Hip:
    """The few HIP runtime calls the timing needs (events on a given stream)."""

    def __init__(self):
        self.rt = C.CDLL("libamdhip64.so")
        self.rt.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.rt.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.rt.hipEventSynchronize.argtypes = [C.c_void_p]
        self.rt.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.rt.hipEventDestroy.argtypes = [C.c_void_p]

    def event(self):
        e = C.c_void_p()
        assert self.rt.hipEventCreate(C.byref(e)) == 0
        return e

    def record(self, e, stream):
        assert self.rt.hipEventRecord(e, C.c_void_p(stream)) == 0

    def sync(self, e):
        assert self.rt.hipEventSynchronize(e) == 0

    def ms(self, a, b):
        out = C.c_float()
        assert self.rt.hipEventElapsedTime(C.byref(out), a, b) == 0
        return float(out.value)


def cpu_baseline(case, L, prep_canon, rows=768, fmt="int4"):
    """The oracle as it stands, timed on the host cores over the first `rows` tokens of the same workload."""
    import numpy as np
    if fmt == "fp4":
        from oracle import svdq_fp4_oracle as O
    elif fmt == "w8a8":
        from oracle import svdq_w8a8_oracle as O
    else:
        from oracle import svdq_oracle as O

    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    xb = L["x_bf16"][:rows]
    best = float("inf")
    for _ in range(2):
        t0 = time.perf_counter()
        O.forward(xb, prep_canon)
        best = min(best, time.perf_counter() - t0)
    ops = 2.0 * rows * case.N * case.K
    return {"value": ops / best / 1e12, "unit": "TOPS", "cores": int(threads), "kind": "oracle",
            "sample": f"first {rows} of {case.M} tokens, all K and N, best of 2 ({best:.2f} s); scaled by 2*rows*N*K",
            "us_per_layer_extrapolated": best * case.M / rows * 1e6}


def bench_w4a16(args, np, torch, S, hip):
    """The W4A16 forward on a synthetic modulation layer: weight-stream bandwidth against the HBM roofline."""
    from paper_2411_05007_amd import inputs as I
    K, N, r, M = 3072, 18432, 32, args.w4a16
    G = K // 64
    rng = np.random.default_rng(241105016)
    # the forward's speed does not depend on the values: seeded random codes and scales stand in for a prepared layer
    # (preparing one needs an SVD of a 3072 x 18432 matrix on the host, which this mode does not time)
    prep = S.svdq_pack((1.0 / (np.abs(rng.standard_normal(K)) + 0.5)).astype(np.float32),
                       I.f32_to_bf16_bits((rng.standard_normal((K, r)) * 0.05).astype(np.float32)),
                       I.f32_to_bf16_bits((rng.standard_normal((r, N)) * 0.05).astype(np.float32)),
                       rng.integers(-8, 8, size=(K, N), dtype=np.int8),
                       (np.abs(rng.standard_normal((G, N))) * 0.01 + 1e-3).astype(np.float16),
                       bias=(rng.standard_normal(N) * 0.1).astype(np.float32))
    nsets = 10                                           # 10 x 30 MB of weights rotate: past the 256 MB last-level cache
    layers = [S.DeviceLayer(prep, "cuda:0") for _ in range(nsets)]
    x = S.bf16_tensor_from_bits(I.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)), "cuda:0")
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda:0")
    ws = layers[0].workspace(M)
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    for i in range(args.warmup):
        layers[i % nsets].forward_w4a16(x, out=y, workspace=ws, stream=stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        layers[i % nsets].forward_w4a16(x, out=y, workspace=ws, stream=stream)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ev = [(hip.event(), hip.event(), hip.event()) for _ in range(args.steps)]
    for i, (a, m, b) in enumerate(ev):
        S.svdq_profile_event(m.value)
        hip.record(a, sh)
        layers[i % nsets].forward_w4a16(x, out=y, workspace=ws, stream=stream)
        hip.record(b, sh)
    torch.cuda.synchronize()
    S.svdq_profile_event(None)
    proj_us = float(np.mean([hip.ms(a, m) for a, m, b in ev])) * 1e3
    main_us = float(np.mean([hip.ms(m, b) for a, m, b in ev])) * 1e3
    # algorithmic bytes of the weight-streaming kernel: codes, scales, L2 and bias once; X, H and Y are a few KB
    nbytes = K * N // 2 + G * N * 2 + N * r * 2 + N * 4 + M * K * 2 + M * r * 4 + M * N * 2
    gbs = nbytes / (main_us * 1e-6) / 1e9
    print(json.dumps({
        "metric": f"W4A16 linear (16-bit activations, INT4 weights + low-rank branch) us/layer, M={M} K={K} N={N} r={r}",
        "value": ms * 1e3, "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 codes widened to fp32, fp32 FMA and accumulate, bf16 out", "data": "synthetic",
        "config": {"workload": f"FLUX.1 modulation linear: M={M} K={K} N={N} r={r} g=64, weights rotated over {nsets} copies"},
        "kernels": {"projection_us": proj_us, "w4a16_us": main_us},
        "roofline": {"bound": "hbm", "kernel": "w4a16_stream_kernel" if M <= 2 else "w4a16_kernel",
                     "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": None},
    }), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=100, help="untimed steps; the clocks need tens of milliseconds of load to settle")
    ap.add_argument("--case", default="flux_mlp_up", help="layer name from paper_2411_05007_amd.inputs (default: the metric shape)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tile", type=int, default=0, help="GEMM tile configuration id (0 = library default)")
    ap.add_argument("--breakdown", action="store_true", help="also time naive INT4 (no low-rank) and the unfused 4-kernel pipeline")
    ap.add_argument("--format", choices=["int4", "fp4", "w8a8"], default="int4",
                    help="int4 = the metric's format (group 64, fp16 scales, INT8 MFMA); fp4 = the MXFP4 variant "
                         "(E2M1, blocks of 32, power-of-two scales) on the block-scaled MFMA; w8a8 = the paper's 8-bit setting "
                         "(per-token / per-channel INT8, rank 16)")
    ap.add_argument("--lora", type=int, default=0, metavar="R",
                    help="append a synthetic rank-R adapter to the layer's 16-bit branch (no re-quantization) and time that")
    ap.add_argument("--w4a16", type=int, default=0, metavar="ROWS",
                    help="time the 16-bit-activation forward (the adaptive-normalization linears) instead: ROWS conditioning "
                         "rows through a FLUX.1 modulation layer, 3072 -> 18432, rank 32; a memory-bound side path, not the metric")
    ap.add_argument("--pmc-run", action="store_true",
                    help="for `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`: a few forwards plus one plain copy of 256 MiB "
                         "(the known-size kernel the counters are scaled by), no timing, no JSON")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X per box); run with --gpus 1. "
              "Rows of X are independent, so N GPUs would each take M/N tokens with replicated weights.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2411_05007_amd import inputs as I
    from paper_2411_05007_amd import svdq as S

    S.lib()   # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    if args.w4a16 > 0:
        bench_w4a16(args, np, torch, S, Hip())
        return
    case = I.case_by_name(args.case)
    L = I.make_layer(case)
    fp4 = args.format == "fp4"
    w8 = args.format == "w8a8"
    rank = 16 if w8 else case.rank                       # the paper's 8-bit setting uses rank 16
    prep = (S.svdq_fp4_prepare if fp4 else S.svdq_w8a8_prepare if w8 else S.svdq_prepare)(L["w"], L["x_absmax"], rank, bias=L["bias"])
    if args.lora > 0:
        rng = np.random.default_rng(241105999)
        down = (rng.standard_normal((case.K, args.lora)) * 0.02).astype(np.float32)
        up = (rng.standard_normal((args.lora, case.N)) * 0.02).astype(np.float32)
        prep = S.svdq_append_lora(prep, down, up, 1.0)
    layer = S.DeviceLayer(prep, dev)

    # >= 3 independent (X, Y, workspace) sets so the footprint exceeds the 256 MB last-level cache
    nsets = 3
    xs, ys, wss = [], [], []
    for i in range(nsets):
        xb = L["x_bf16"] if i == 0 else np.roll(L["x_bf16"], 17 * i, axis=0)
        xs.append(S.bf16_tensor_from_bits(np.ascontiguousarray(xb), dev))
        ys.append(torch.empty((case.M, case.N), dtype=torch.bfloat16, device=dev))
        wss.append(layer.workspace(case.M))

    hip = Hip()
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream

    if args.pmc_run:
        S.svdq_forward_options(args.tile << S.OPT_TILE_SHIFT)
        for i in range(4):
            layer.forward(xs[i % nsets], out=ys[i % nsets], workspace=wss[i % nsets], stream=stream)
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        torch.cuda.synchronize()
        print("pmc-run done: 4 forwards, 2 copies of 268435456 bytes", flush=True)
        return

    def run(flags, steps, warmup, split):
        S.svdq_forward_options(flags | (args.tile << S.OPT_TILE_SHIFT))
        for i in range(warmup):
            layer.forward(xs[i % nsets], out=ys[i % nsets], workspace=wss[i % nsets], stream=stream)
        torch.cuda.synchronize()
        ev = [(hip.event(), hip.event(), hip.event()) for _ in range(steps)] if split else None
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            j = i % nsets
            if split:
                a, m, b = ev[i]
                S.svdq_profile_event(m.value)
                hip.record(a, sh)
                layer.forward(xs[j], out=ys[j], workspace=wss[j], stream=stream)
                hip.record(b, sh)
            else:
                layer.forward(xs[j], out=ys[j], workspace=wss[j], stream=stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        S.svdq_profile_event(None)
        res = {"ms_per_step": wall * 1e3 / steps}
        if split:
            act = [hip.ms(a, m) for a, m, b in ev]
            gemm = [hip.ms(m, b) for a, m, b in ev]
            for a, m, b in ev:
                for e in (a, m, b):
                    hip.rt.hipEventDestroy(e)
            res.update(act_ms=float(np.mean(act)), gemm_ms=float(np.mean(gemm)),
                       gemm_ms_min=float(np.min(gemm)), act_ms_min=float(np.min(act)))
        return res

    # The timed region proper: K forwards back to back, nothing else on the stream.  The per-kernel durations
    # come from a second pass over the same K steps with three HIP events per step on the launch stream (one of
    # them recorded by the library between its two kernels); the events cost a few microseconds per step, which
    # is why they stay out of the pass that `value` is computed from.
    timed = run(0, args.steps, args.warmup, split=False)
    main_res = run(0, args.steps, min(args.warmup, 20), split=True)
    main_res["ms_per_step_with_events"] = main_res["ms_per_step"]
    main_res["ms_per_step"] = timed["ms_per_step"]
    ms = main_res["ms_per_step"]
    ops = float(case.ops)
    tops = ops / (ms * 1e-3) / 1e12
    gemm_tops = ops / (main_res["gemm_ms"] * 1e-3) / 1e12
    G = case.K // 64
    act_bytes = case.M * case.K * (2 + 0.5 + 2.0 / 64) + 4.0 * case.M * case.rank     # algorithmic bytes of the activation pass
    out = {
        "metric": ("fused W4A4+low-rank linear TOPS & us/layer, FLUX MLP M=4608 K=3072 N=12288 r=32"
                   if case.name == "flux_mlp_up" else f"fused W4A4+low-rank linear TOPS & us/layer, {case.name}")
                  + (" [MXFP4 variant]" if fp4 else " [W8A8 setting, r=16]" if w8 else ""),
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "us_per_layer": ms * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp4 (E2M1) block-scaled MFMA, fp32 accumulate, bf16 out" if fp4
                 else "int8 MFMA (int8 codes), exact int32 sums, one fp32 rescale, bf16 out" if w8
                 else "int8 MFMA (int4 codes), int32 group sums, fp32 rescale, bf16 out",
        "data": "synthetic",
        "config": {"workload": f"{case.name}: M={case.M} K={case.K} N={case.N} r={case.rank} g=64"
                               + (" MXFP4 (blocks of 32)" if fp4 else " W8A8 (per token / per channel, branch rank 16)" if w8 else "")
                               + (f" + LoRA r={args.lora} (branch rank {prep.shape.rank})" if args.lora else "")
                               + (" (the FLUX MLP up projection the metric is quoted on)" if case.name == "flux_mlp_up" else ""),
                   "tile": args.tile, "sets_rotated": nsets},
        "kernels": {"act_us": main_res["act_ms"] * 1e3, "gemm_us": main_res["gemm_ms"] * 1e3,
                    "gemm_us_min": main_res["gemm_ms_min"] * 1e3,
                    "us_per_layer_with_events": main_res["ms_per_step_with_events"] * 1e3,
                    "act_GBps": act_bytes / (main_res["act_ms"] * 1e-3) / 1e9,
                    "act_frac_hbm_peak": act_bytes / (main_res["act_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "roofline": {"bound": "mfma",
                     "kernel": ("gemm_fp4_kernel (MXFP4 GEMM" if fp4 else "gemm_w8a8_kernel (INT8 GEMM" if w8 else "gemm_kernel (W4A4 GEMM")
                               + " + fused up projection, bias, bf16 store)",
                     "achieved": gemm_tops, "peak": FP4_MFMA_PEAK_TFLOPS if fp4 else INT8_MFMA_PEAK_TOPS, "unit": "TFLOP/s",
                     "note": ("FP4" if fp4 else "INT8") + " tera-ops/s: 2*M*N*K per launch / mean launch duration (HIP events on the launch stream)",
                     "frac": gemm_tops / (FP4_MFMA_PEAK_TFLOPS if fp4 else INT8_MFMA_PEAK_TOPS),
                     "traffic": GEMM_TRAFFIC_BYTES if case.name == "flux_mlp_up" and args.format == "int4" else None},
    }
    if args.breakdown:
        naive = run(S.OPT_SKIP_LOWRANK, args.steps, 20, split=False)
        out["breakdown"] = {"fused_us": ms * 1e3, "naive_int4_us": naive["ms_per_step"] * 1e3,
                            "lowrank_overhead_fused": ms / naive["ms_per_step"] - 1.0}
        if not fp4 and not w8:                           # the unfused pipeline exists for the INT4 path only
            unfused = run(S.OPT_UNFUSED, max(20, args.steps // 2), 20, split=False)
            out["breakdown"].update(unfused_us=unfused["ms_per_step"] * 1e3,
                                    lowrank_overhead_unfused=unfused["ms_per_step"] / naive["ms_per_step"] - 1.0)
        again = run(0, args.steps, 20, split=False)      # the fused path once more, after the others: drift check
        out["breakdown"]["fused_us_again"] = again["ms_per_step"] * 1e3
    S.svdq_forward_options(0)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(case, L, (S.svdq_fp4_unpack if fp4 else S.svdq_w8a8_unpack if w8 else S.svdq_unpack)(prep),
                                           fmt=args.format)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
