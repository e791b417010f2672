"""Launches one linear layer's GEMM of a workload configuration a number of times and exits: the program to put behind
`rocprofv3 --kernel-trace --stats` or `rocprofv3 --pmc <counters>` when a kernel is to be looked at on its own.

    python3 -m paper_2305_10727_amd.gemm_loop --config c2 --layer fc2 --path int8 --kind sparse --iters 20

Random device tensors of the configuration's shapes and distributions; every launch goes through the C ABI.  With
--calibrate the fp32 -> fp16 streaming kernel runs three times on 2^26 elements at the end (256 MiB read, 128 MiB
written: the known traffic the FETCH_SIZE / WRITE_SIZE counters are scaled by).
"""
import argparse

import torch

from . import gpusq as G
from . import synth
from .pipeline import SparseLinear


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="c1")
    ap.add_argument("--layer", default="fc1")
    ap.add_argument("--path", default="int8", choices=["int8", "fp16"])
    ap.add_argument("--kind", default="sparse", choices=["sparse", "dense"])
    ap.add_argument("--out", default="fp16", choices=["fp16", "int8"], help="output type of the int8 path")
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--calibrate", action="store_true")
    a = ap.parse_args()
    cfg = synth.CONFIGS[a.config]
    M = cfg["M"]
    _, K, N, gelu, dist = [l for l in cfg["layers"] if l[0] == a.layer][0]
    dev = torch.device("cuda")
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    X = torch.randn(M, K, device=dev, generator=g)
    if dist == "gelu_normal":
        X = torch.nn.functional.gelu(X)
    X = X.half()
    W = torch.randn(N, K, device=dev, generator=g) * 0.02
    bias = torch.randn(N, device=dev, generator=g) * 0.01
    out_dtype = torch.int8 if (a.path == "int8" and a.out == "int8") else torch.float16
    lin = SparseLinear(M, K, N, a.path, gelu=gelu, bias=True, out_dtype=out_dtype)
    lin.prepare_weights(W, fused=K * 4 <= 64 * 1024)
    if a.path == "int8":
        lin.quantize_activations(X)
    out_scale = torch.full((1,), 0.05, dtype=torch.float32, device=dev) if out_dtype == torch.int8 else None
    fn = lin.gemm if a.kind == "sparse" else lin.gemm_dense
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn(X, bias, out_scale)
    e0.record()
    for _ in range(a.iters):
        fn(X, bias, out_scale)
    e1.record()
    torch.cuda.synchronize()
    if a.calibrate:
        cin = torch.ones(1 << 26, dtype=torch.float32, device=dev)
        cout = torch.empty(1 << 26, dtype=torch.float16, device=dev)
        for _ in range(3):
            G.cast_f16(cin, out=cout)
        torch.cuda.synchronize()
    us = e0.elapsed_time(e1) / a.iters * 1e3
    print("%s %s %s %s M=%d K=%d N=%d gelu=%d: %.2f us per launch, %.1f dense-equivalent TOPS" %
          (a.config, a.layer, a.path, a.kind, M, K, N, gelu, us, 2.0 * M * N * K / us / 1e6))


if __name__ == "__main__":
    main()
