#!/usr/bin/env python3
"""Benchmark of the fused W4A4 + low-rank linear layer (arXiv 2411.05007, Eq. 5) on one MI355X.

One "step" is one pass of the whole hot path - activation kernel (smooth + INT4 quantize + down
projection) and W4A4 GEMM (with up projection, bias and bf16 store) - over one batch of synthetic
FLUX-MLP-shaped input (M=4608, K=3072, N=12288, r=32) already resident in HBM.

`--format fp4` and `--format w8a8` time the MXFP4 variant and the 8-bit setting of the same layer instead (their GEMMs
against the FP4 and INT8 MFMA peaks), `--lora R` appends an adapter first; the default line is the INT4 metric.

Prints ONE JSON line with the headline metric (TOPS of the 4-bit branch, 2*M*N*K per layer time),
the roofline of the dominant kernel (the GEMM, against the published INT8 MFMA peak and against what a
register-only MFMA loop sustains in the same run) measured live with HIP events on the stream the kernels
run on, the fused / naive / unfused breakdown of Sec. 4.3, and the CPU oracle timed on all rows of the workload.

Timing protocol: before anything is timed the layer runs untimed until the clocks have settled (at least
150 ms of GPU work, and two consecutive windows of 20 steps within 2 % of each other), whatever --warmup says;
then --warmup further untimed steps; then exactly --steps steps, each bracketed by HIP events.  `value` comes
from the MEDIAN step; the mean and the wall-clock mean of the same pass are reported beside it.
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

# HBM-side traffic of one GEMM launch at the headline shape: NOT measured by this script.  It is the figure of
# `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` runs of `bench.py --pmc-run`, each counter scaled by what it reads
# for a plain 256 MiB copy; the summary with the commands is profiles/flux_mlp_up_pmc_counters.md.
GEMM_TRAFFIC_BYTES = 347.9e6         # 234.7 MB read (FETCH_SIZE x 2.000) + 113.2 MB written (WRITE_SIZE x 1.000) per launch
GEMM_TRAFFIC_SOURCE = "profiles/flux_mlp_up_pmc_counters.md"


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


def cpu_baseline(case, L, prep_canon, fmt="int4", reps=3):
    """The oracle as it stands, timed on the host cores over ALL tokens of the same workload, best of `reps`."""
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
    xb = L["x_bf16"]
    times = []
    for _ in range(reps):
        t0 = time.perf_counter()
        O.forward(xb, prep_canon)
        times.append(time.perf_counter() - t0)
    best = min(times)
    ops = float(case.ops)
    return {"value": ops / best / 1e12, "unit": "TOPS", "cores": int(threads), "kind": "oracle",
            "sample": f"all {case.M} tokens, all K and N: the oracle's forward (quantize, per-group integer products, low-rank branch, "
                      f"bias), prepare excluded; best of {reps} ({', '.join(f'{t:.2f}' for t in times)} s)",
            "us_per_layer": best * 1e6}


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
                       rng.integers(-7, 8, size=(K, N), dtype=np.int8),
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
    ap.add_argument("--warmup", type=int, default=20, help="untimed steps after the clock-settling phase (which runs whatever this says)")
    ap.add_argument("--case", default="flux_mlp_up", help="layer name from paper_2411_05007_amd.inputs (default: the metric shape)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-breakdown", action="store_true", help="skip the naive-INT4 / unfused-pipeline passes (Sec. 4.3 / Fig. 6)")
    ap.add_argument("--format", choices=["int4", "fp4", "w8a8"], default="int4",
                    help="int4 = the metric's format (group 64, fp16 scales, INT8 MFMA); fp4 = the MXFP4 variant "
                         "(E2M1, blocks of 32, power-of-two scales) on the block-scaled MFMA; w8a8 = the paper's 8-bit setting "
                         "(per-token / per-channel INT8, rank 16)")
    ap.add_argument("--lora", type=int, default=0, metavar="R",
                    help="append a synthetic rank-R adapter to the layer's 16-bit branch (no re-quantization) and time that")
    ap.add_argument("--w4a16", type=int, default=0, metavar="ROWS",
                    help="time the 16-bit-activation forward (the adaptive-normalization linears) instead: ROWS conditioning "
                         "rows through a FLUX.1 modulation layer, 3072 -> 18432, rank 32; a memory-bound side path, not the metric")
    ap.add_argument("--act-chunk", type=int, default=0, metavar="GROUPS",
                    help="int4 only: groups of 64 channels per activation-kernel workgroup (255 = all of K), 0 = the library's choice")
    ap.add_argument("--ksplit", type=int, default=0, metavar="S", help="int4 only: workgroups per output tile along K, 0 = the library's choice")
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
    base_opts = ((args.act_chunk & 0xff) << S.OPT_ACT_CHUNK_SHIFT) | ((args.ksplit & 0xf) << S.OPT_KSPLIT_SHIFT)
    S.svdq_forward_options(base_opts)      # before the workspaces are sized

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
        S.svdq_forward_options(base_opts)
        for i in range(4):
            layer.forward(xs[i % nsets], out=ys[i % nsets], workspace=wss[i % nsets], stream=stream)
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        torch.cuda.synchronize()
        print("pmc-run done: 4 forwards, 2 copies of 268435456 bytes", flush=True)
        return

    def step(i):
        j = i % nsets
        layer.forward(xs[j], out=ys[j], workspace=wss[j], stream=stream)

    def settle(max_ms=3000.0):
        """Untimed steps until the clocks have settled: windows of 20 steps, each timed with a pair of events, until
        at least 150 ms of GPU work have passed and two consecutive windows agree within 2 %."""
        done_ms, steps, prev, stable = 0.0, 0, None, False
        e0, e1 = hip.event(), hip.event()
        while done_ms < max_ms:
            hip.record(e0, sh)
            for i in range(20):
                step(steps + i)
            hip.record(e1, sh)
            hip.sync(e1)
            w = hip.ms(e0, e1)
            steps += 20
            done_ms += w
            stable = prev is not None and abs(w - prev) <= 0.02 * prev
            prev = w
            if done_ms >= 150.0 and stable:
                break
        for e in (e0, e1):
            hip.rt.hipEventDestroy(e)
        return {"settle_ms": done_ms, "settle_steps": steps, "settled": bool(stable), "last_window_us_per_step": prev * 1e3 / 20}

    def run(flags, steps, warmup):
        """Settle, `warmup` more untimed steps, then `steps` timed steps: three HIP events per step on the launch stream
        (one of them recorded by the library between its two kernels)."""
        S.svdq_forward_options(flags | base_opts)
        st = settle()
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        ev = [(hip.event(), hip.event(), hip.event()) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            a, m, b = ev[i]
            S.svdq_profile_event(m.value)
            hip.record(a, sh)
            step(i)
            hip.record(b, sh)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        S.svdq_profile_event(None)
        # a step's interval runs from the end of the step before it (its first event follows that step's last kernel
        # on the stream) to the end of its own GEMM, so the intervals add up to the whole pass
        per = np.array([hip.ms(a, b) for a, m, b in ev])
        act = np.array([hip.ms(a, m) for a, m, b in ev])
        gemm = np.array([hip.ms(m, b) for a, m, b in ev])
        for a, m, b in ev:
            for e in (a, m, b):
                hip.rt.hipEventDestroy(e)
        res = dict(st)
        res.update(ms_per_step=float(np.median(per)), ms_per_step_mean=float(np.mean(per)), ms_per_step_wall=wall * 1e3 / steps,
                   ms_per_step_min=float(np.min(per)), act_ms=float(np.mean(act)), gemm_ms=float(np.mean(gemm)),
                   act_ms_median=float(np.median(act)), gemm_ms_median=float(np.median(gemm)), gemm_ms_min=float(np.min(gemm)))
        return res

    def measured_peak(kind):
        """TOPS of the register-only MFMA loop (kind 0: int8 32x32x32, 1: 6-bit operands 32x32x64), best of 5 launches of ~1 ms."""
        sink = torch.empty(512 * 256, dtype=torch.float32, device=dev)
        e0, e1 = hip.event(), hip.event()
        iters = 4000
        for _ in range(3):
            S.svdq_mfma_peak_probe(kind, iters, sink, stream)
        best = float("inf")
        ops = 0.0
        for _ in range(5):
            hip.record(e0, sh)
            ops = S.svdq_mfma_peak_probe(kind, iters, sink, stream)
            hip.record(e1, sh)
            hip.sync(e1)
            best = min(best, hip.ms(e0, e1))
        for e in (e0, e1):
            hip.rt.hipEventDestroy(e)
        return ops / (best * 1e-3) / 1e12

    main_res = run(0, args.steps, args.warmup)
    ms = main_res["ms_per_step"]
    ops = float(case.ops)
    tops = ops / (ms * 1e-3) / 1e12
    gemm_tops = ops / (main_res["gemm_ms"] * 1e-3) / 1e12
    peak_pub = FP4_MFMA_PEAK_TFLOPS if fp4 else INT8_MFMA_PEAK_TOPS
    peak_int8_measured = measured_peak(0)
    peak_fp6_measured = measured_peak(1)
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
                 else "int4 codes as exact 6-bit floats on the block-scaled MFMA, exact fp32 group sums, fp32 rescale, bf16 out",
        "data": "synthetic",
        "config": {"workload": f"{case.name}: M={case.M} K={case.K} N={case.N} r={case.rank} g=64"
                               + (" MXFP4 (blocks of 32)" if fp4 else " W8A8 (per token / per channel, branch rank 16)" if w8 else "")
                               + (f" + LoRA r={args.lora} (branch rank {prep.shape.rank})" if args.lora else "")
                               + (" (the FLUX MLP up projection the metric is quoted on)" if case.name == "flux_mlp_up" else ""),
                   "sets_rotated": nsets},
        "timing": {"value_from": "median step of the timed pass (HIP events around every step)",
                   "us_per_step_median": ms * 1e3, "us_per_step_mean": main_res["ms_per_step_mean"] * 1e3,
                   "us_per_step_min": main_res["ms_per_step_min"] * 1e3, "us_per_step_wall_clock": main_res["ms_per_step_wall"] * 1e3,
                   "settle_ms": main_res["settle_ms"], "settle_steps": main_res["settle_steps"], "settled": main_res["settled"]},
        "kernels": {"act_us": main_res["act_ms"] * 1e3, "gemm_us": main_res["gemm_ms"] * 1e3,
                    "act_us_median": main_res["act_ms_median"] * 1e3, "gemm_us_median": main_res["gemm_ms_median"] * 1e3,
                    "gemm_us_min": main_res["gemm_ms_min"] * 1e3,
                    "act_GBps": act_bytes / (main_res["act_ms"] * 1e-3) / 1e9,
                    "act_frac_hbm_peak": act_bytes / (main_res["act_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "roofline": {"bound": "mfma",
                     "kernel": ("gemm_fp4_kernel (MXFP4 GEMM" if fp4 else "gemm_w8a8_kernel (INT8 GEMM" if w8 else "gemm_w4a4_kernel (W4A4 GEMM")
                               + " + fused up projection, bias, bf16 store)",
                     "achieved": gemm_tops, "peak": peak_pub, "unit": "TFLOP/s",
                     "note": ("FP4" if fp4 else "INT8") + " tera-ops/s: 2*M*N*K per launch / mean launch duration (HIP events on the launch stream); "
                             "peak = the published dense rate the metric is quoted against",
                     "frac": gemm_tops / peak_pub,
                     "peak_measured_int8": peak_int8_measured, "frac_measured_peak": gemm_tops / peak_int8_measured,
                     "peak_measured_fp6_instruction": peak_fp6_measured, "peak_published_fp6_instruction": FP4_MFMA_PEAK_TFLOPS,
                     "frac_of_fp6_instruction_published": gemm_tops / FP4_MFMA_PEAK_TFLOPS,
                     "measured_peak_note": "register-only loops of v_mfma_i32_32x32x32_i8 and of v_mfma_scale_f32_32x32x64_f8f6f4 (6-bit operands), "
                                           "two wavefronts per SIMD, timed in this run",
                     "traffic": GEMM_TRAFFIC_BYTES if case.name == "flux_mlp_up" and args.format == "int4" else None,
                     "traffic_note": f"not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE figure from {GEMM_TRAFFIC_SOURCE}"},
    }
    if not args.no_breakdown:
        # Sec. 4.3 / Fig. 6 and App. "Latency Results": the 4-bit branch alone ("naive INT4"), and the low-rank branch run
        # as separate kernels (down projection, quantize, GEMM, up projection)
        naive = run(S.OPT_SKIP_LOWRANK, max(20, args.steps // 2), 10)
        out["breakdown"] = {"fused_us": ms * 1e3, "naive_int4_us": naive["ms_per_step"] * 1e3,
                            "lowrank_overhead_fused": ms / naive["ms_per_step"] - 1.0}
        if not fp4 and not w8:                           # the unfused pipeline exists for the INT4 path only
            unfused = run(S.OPT_UNFUSED, max(20, args.steps // 2), 10)
            out["breakdown"].update(unfused_us=unfused["ms_per_step"] * 1e3,
                                    lowrank_overhead_unfused=unfused["ms_per_step"] / naive["ms_per_step"] - 1.0)
        again = run(0, max(20, args.steps // 2), 10)     # the fused path once more, after the others: drift check
        out["breakdown"]["fused_us_again"] = again["ms_per_step"] * 1e3
    S.svdq_forward_options(0)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(case, L, (S.svdq_fp4_unpack if fp4 else S.svdq_w8a8_unpack if w8 else S.svdq_unpack)(prep),
                                           fmt=args.format)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
