#!/usr/bin/env python3
"""Benchmark of the 2:4 structured-sparse linear-layer path on one MI355X.

One step = one pass of the whole path over the ViT-Base MLP fc1 workload at batch 64 (M = 64*197, K = 768,
N = 3072): prune 2:4 -> per-channel INT8 weights -> compress -> pack, per-tensor INT8 activations, sparse INT8 GEMM
with fused dequantise + bias + GELU and fp16 output.  Inputs (fp32 weights, fp16 activations, fp32 bias) are
synthetic, seeded, and resident in HBM before the timed region.

Prints ONE JSON line.  `value` is dense-equivalent TOPS (2*M*N*K per step / step time) of the whole step; the
sparse GEMM kernel alone, its dense twin, the FP16 pair and the other kernels are reported beside it.
"""
import argparse
import json
import os
import sys
import time

import numpy as np


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU-oracle timing leg")
    ap.add_argument("--only-step", action="store_true", help="run only the timed full-path steps")
    ap.add_argument("--profile-mode", action="store_true",
                    help="for rocprofv3 runs: the timed steps, then 3 launches of the fp32->fp16 streaming kernel on 2^26 "
                         "elements (reads 256 MiB, writes 128 MiB) that calibrate the FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def time_kernel(fn, iters, torch, warm=5):
    """average ms per launch of fn over `iters` back-to-back launches, HIP events on the current stream"""
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path shards over M with no exchange step, and this build runs on a "
              "single MI355X; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2305_10727_amd import gpusq, synth
    from paper_2305_10727_amd.pipeline import SparseLinear

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    gpusq.lib()  # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS["c1"]
    M = cfg["M"]
    _, K, N, gelu, dist = cfg["layers"][0]
    ids = (1, 0)
    X32 = synth.activations(M, K, dist, seed=cfg["seed"], ids=ids)
    W32 = synth.weights(N, K, seed=cfg["seed"], ids=ids)
    b32 = synth.bias(N, seed=cfg["seed"], ids=ids)
    Xh = torch.from_numpy(X32.astype(np.float16)).to(dev)
    W = torch.from_numpy(W32).to(dev)
    bias = torch.from_numpy(b32).to(dev)

    lin = SparseLinear(M, K, N, "int8", gelu=gelu, bias=True, out_dtype=torch.float16)
    eff_ops = 2.0 * M * N * K

    # ---- the timed region: W warm-up steps, then exactly K steps of the whole path --------------------------------
    lin.prepare_weights(W)  # once with every optional output: the dense twin below reads the masked INT8 weights
    for _ in range(args.warmup):
        lin.prepare_weights(W, intermediates=False)
        lin.forward(Xh, bias)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        # prune -> quantise -> compress -> pack in one launch; it writes the packed operand and the scales, the
        # intermediate tensors of the unfused chain are not materialised
        lin.prepare_weights(W, intermediates=False)
        lin.quantize_activations(Xh)
        lin.gemm(Xh, bias)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = e0.elapsed_time(e1) / args.steps
    # The same K steps once more with a pair of events around every GEMM launch, for the launch duration of the dominant
    # kernel inside the step (same stream, same predecessors and cache state as in the timed pass).  The events stay out
    # of the timed pass: each one is a command of its own in the queue, and two per step cost about 8 us of a 64 us step.
    gemm_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    e2, e3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e2.record()
    for i in range(args.steps):
        lin.prepare_weights(W, intermediates=False)
        lin.quantize_activations(Xh)
        gemm_ev[i][0].record()
        lin.gemm(Xh, bias)
        gemm_ev[i][1].record()
    e3.record()
    torch.cuda.synchronize()
    gemm_ms_in_step = float(np.mean([a.elapsed_time(b) for a, b in gemm_ev]))
    ms_per_step_with_events = e2.elapsed_time(e3) / args.steps
    if args.profile_mode:
        calib_in = torch.ones(1 << 26, dtype=torch.float32, device=dev)
        calib_out = torch.empty(1 << 26, dtype=torch.float16, device=dev)
        for _ in range(3):
            gpusq.cast_f16(calib_in, out=calib_out)
        torch.cuda.synchronize()
    if args.only_step or args.profile_mode:
        print(json.dumps({"ms_per_step": ms_per_step, "gemm_ms_in_step": gemm_ms_in_step}))
        return

    # ---- per-kernel timings (back-to-back launches, same buffers) ---------------------------------------------------
    it = max(20, min(args.steps, 200))
    t_gemm = time_kernel(lambda: lin.gemm(Xh, bias), it, torch)
    t_dense = time_kernel(lambda: lin.gemm_dense(Xh, bias), it, torch)
    t_qact = time_kernel(lambda: lin.quantize_activations(Xh), it, torch)
    t_wprep = time_kernel(lambda: lin.prepare_weights(W, intermediates=False), it, torch)
    t_wprep_all = time_kernel(lambda: lin.prepare_weights(W), it, torch)
    lin16 = SparseLinear(M, K, N, "fp16", gelu=gelu, bias=True)
    lin16.prepare_weights(W)
    t_gemm16 = time_kernel(lambda: lin16.gemm(Xh, bias), it, torch)
    t_dense16 = time_kernel(lambda: lin16.gemm_dense(Xh, bias), it, torch)
    lin8o = SparseLinear(M, K, N, "int8", gelu=gelu, bias=True, out_dtype=torch.int8)
    lin8o.prepare_weights(W)
    lin8o.quantize_activations(Xh)
    out_scale = torch.full((1,), 0.05, dtype=torch.float32, device=dev)
    t_gemm8o = time_kernel(lambda: lin8o.gemm(Xh, bias, out_scale), it, torch)

    # algorithmic HBM bytes of one sparse INT8 GEMM launch: X int8 + kept values + metadata + scales + bias + Y fp16
    gemm_bytes = M * K + N * K // 2 + N * K // 8 + 8 * N + 4 + 2 * M * N
    gemm_s = gemm_ms_in_step * 1e-3
    roofline = {"bound": "hbm", "achieved": gemm_bytes / gemm_s / 1e9, "peak": 8000.0, "unit": "GB/s",
                "frac": gemm_bytes / gemm_s / 1e9 / 8000.0, "traffic": None, "kernel": "spgemm_tile_kernel<int8, GELU, fp16 out> (fused epilogue)",
                "algorithmic_bytes": gemm_bytes, "avg_launch_ms": gemm_ms_in_step,
                "measured": "HIP events around each GEMM launch in a second pass of the same %d steps" % args.steps}
    traffic_file = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "spgemm_int8_c1_traffic.json")
    if os.path.exists(traffic_file):  # HBM bytes per launch from committed rocprofv3 --pmc runs (FETCH_SIZE + WRITE_SIZE)
        roofline["traffic"] = json.load(open(traffic_file)).get("hbm_bytes_per_launch")

    out = {
        "metric": "2:4-sparse INT8 GEMM TOPS on ViT-B shapes (dense-equivalent 2*M*N*K ops / step time; step = whole path)",
        "value": eff_ops / (ms_per_step * 1e-3) / 1e12, "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "c1: ViT-Base MLP fc1, batch 64 (M=12608, K=768, N=3072), 2:4 INT8 per-channel weights, "
                               "per-tensor INT8 activations from fp16, fused bias+GELU, fp16 output",
                   "M": M, "K": K, "N": N, "step": "prune+quantize_w+compress+pack (one fused launch, intermediates not written)+quantize_act+spgemm_int8"},
        "wall_ms_per_step": wall_ms / args.steps, "ms_per_step_with_gemm_events": ms_per_step_with_events,
        "roofline": roofline,
        "kernels": {
            "spgemm_int8_ms": t_gemm, "spgemm_int8_tops": eff_ops / (t_gemm * 1e-3) / 1e12,
            "spgemm_int8_frac_of_sparse_peak_10070": eff_ops / (t_gemm * 1e-3) / 1e12 / 10070.0,
            "gemm_int8_dense_ms": t_dense, "gemm_int8_dense_tops": eff_ops / (t_dense * 1e-3) / 1e12,
            "int8_speedup_vs_dense": t_dense / t_gemm,
            "spgemm_int8_int8out_ms": t_gemm8o, "spgemm_int8_int8out_tops": eff_ops / (t_gemm8o * 1e-3) / 1e12,
            "spgemm_fp16_ms": t_gemm16, "spgemm_fp16_tflops": eff_ops / (t_gemm16 * 1e-3) / 1e12,
            "spgemm_fp16_frac_of_sparse_peak_5030": eff_ops / (t_gemm16 * 1e-3) / 1e12 / 5030.0,
            "gemm_fp16_dense_ms": t_dense16, "gemm_fp16_dense_tflops": eff_ops / (t_dense16 * 1e-3) / 1e12,
            "fp16_speedup_vs_dense": t_dense16 / t_gemm16,
            "quantize_act_ms": t_qact, "weight_prep_ms": t_wprep, "weight_prep_with_intermediate_outputs_ms": t_wprep_all,
        },
        "paper_context": "A100 INT8 2:4 vs FP32 dense end-to-end: 1.26-1.47x latency, 2.40-2.60x throughput (Table 2); "
                         "no GEMM-level figure is published",
    }

    if not args.no_cpu_baseline:
        import oracle
        P, _ = oracle.prune_2to4(W32)
        Wq, s_w = oracle.quantize_rows_int8(P)
        Xq, s_a = oracle.quantize_tensor_int8(X32.astype(np.float16).astype(np.float32))
        vals, meta, _ = oracle.compress(Wq)
        best, spent, reps = None, 0.0, 0
        while spent < 10.0 and reps < 8:
            t = time.perf_counter()
            oracle.linear_int8_sparse(Xq, vals, meta, s_a, s_w, b32, gelu)
            dt = time.perf_counter() - t
            best = dt if best is None else min(best, dt)
            spent += dt
            reps += 1
        out["cpu_baseline"] = {"value": eff_ops / best / 1e12, "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "sparse-form INT8 GEMM + epilogue of the full c1 workload (all %d rows), best of %d runs, "
                                         "%.1f s of CPU time in total" % (M, reps, spent)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
