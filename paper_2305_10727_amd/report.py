"""Per-GEMM timing table over the linear-layer shapes of all workload configurations (c0 ... c4): sparse INT8 and FP16
against their dense twins, with buffers that stay in the memory-side cache ("hot") and with a rotation of buffer sets
larger than it ("cold").  `python -m paper_2305_10727_amd.report [--out FILE]` on a GPU machine; prints a markdown table.

Inputs are random device tensors of the configurations' shapes and distributions (N(0,1) activations, N(0, 0.02)
weights); every number is a sparse or dense GEMM launch through the C ABI, timed with HIP events on the launch stream.
"""
import argparse

import torch

from . import gpusq as G
from . import synth
from .pipeline import EncoderBlockLinears, SparseLinear, SparsePatchEmbed

SPARSE_PEAK = {"int8": 10070.0, "fp16": 5030.0}  # nominal dense-equivalent T(FL)OP/s of the gfx950 sparse matrix instructions
DENSE_PEAK = {"int8": 5035.0, "fp16": 2515.0}
HBM_PEAK = 8000.0  # GB/s
INFINITY_CACHE = 256 << 20


def measured_peaks():
    """sparse matrix rates measured by `python -m paper_2305_10727_amd.probes` (committed run), or None"""
    import json
    import os
    f = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "hardware_probes.json")
    if not os.path.exists(f):
        return {}
    d = {k: v["value"] for k, v in json.load(open(f)).items()}
    return {"int8": d.get("sparse_int8_16x16x128_rate"), "fp16": d.get("sparse_fp16_16x16x64_rate")}


def ideal_speedup(M, K, N, prec):
    """sparse / dense ratio with each side on its own roofline at the nominal peaks: max(matrix time, HBM time of the
    algorithmic bytes); the dense side reads N*K*e weight bytes and no metadata"""
    e = 1 if prec == "int8" else 2
    ops = 2.0 * M * N * K
    io = M * K * e + 8 * N + M * N * 2
    t_s = max(ops / (SPARSE_PEAK[prec] * 1e12), (io + N * K * e // 2 + N * K // 8) / (HBM_PEAK * 1e9))
    t_d = max(ops / (DENSE_PEAK[prec] * 1e12), (io + N * K * e) / (HBM_PEAK * 1e9))
    return t_d / t_s


def _time(fns, iters):
    """average us per launch cycling through `fns` (one per buffer set)"""
    for f in fns:
        f()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(iters):
        fns[i % len(fns)]()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e3


def layer_rows(M, K, N, gelu, iters):
    dev = torch.device("cuda")
    rows = []
    for prec in ("int8", "fp16"):
        e = 1 if prec == "int8" else 2
        per_set = M * K * e + M * N * 2
        n_sets = max(3, -(-2 * INFINITY_CACHE // per_set))  # cold: the sets together exceed twice the cache
        n_sets = min(n_sets, max(3, (6 << 30) // per_set))
        W = torch.randn(N, K, device=dev) * 0.02
        bias = torch.randn(N, device=dev) * 0.01
        sets = []
        for _ in range(n_sets):
            lin = SparseLinear(M, K, N, prec, gelu=gelu, bias=True)
            if sets:  # weights are shared between the sets: only the activations and the outputs rotate
                for name in ("W_low", "values", "meta", "packed", "W_pruned"):
                    setattr(lin, name, getattr(sets[0][0], name))
                if prec == "int8":
                    lin.w_scale = sets[0][0].w_scale
            else:
                lin.prepare_weights(W, fused=K * 4 <= 64 * 1024)
            X = torch.randn(M, K, device=dev).half()
            if prec == "int8":
                lin.quantize_activations(X)
            sets.append((lin, X))
        ops = 2.0 * M * N * K
        alg = M * K * e + N * K * e // 2 + N * K // 8 + 8 * N + M * N * 2
        kernel = G.spgemm_plan(torch.int8 if prec == "int8" else torch.float16, M, N, K, sets[0][0].epilogue)["kernel"]
        # The variants are timed in turn, three rounds of them, and each reports its median: the shader clock moves with
        # the load of the seconds before, so a variant timed once, after a pause or after a heavier kernel, is off by up
        # to 10 %.  `same` is the sparse instantiation of the dense twin's template (tile kernel 3), where the size rules
        # picked another kernel.
        hot = [lambda s=sets[0]: s[0].gemm(s[1], bias)]
        cold = [lambda s=s: s[0].gemm(s[1], bias) for s in sets]
        dense_hot = [lambda s=sets[0]: s[0].gemm_dense(s[1], bias)]
        dense_cold = [lambda s=s: s[0].gemm_dense(s[1], bias) for s in sets]
        with_twin = kernel != 3 and K * e % 128 == 0 and M * N > 256 * 1024
        samples = {name: [] for name in ("hot", "cold", "dense_hot", "dense_cold", "same")}
        for _round in range(3):
            samples["hot"].append(_time(hot, iters))
            samples["cold"].append(_time(cold, iters))
            if with_twin:
                G.force_kernel(3)
                samples["same"].append(_time(cold, iters))
                G.force_kernel(None)
            samples["dense_hot"].append(_time(dense_hot, iters))
            samples["dense_cold"].append(_time(dense_cold, iters))
        med = {name: sorted(v)[len(v) // 2] for name, v in samples.items() if v}
        t_hot, t_cold, td_hot, td_cold = med["hot"], med["cold"], med["dense_hot"], med["dense_cold"]
        t_same = med.get("same", t_cold)
        mp = measured_peaks().get(prec)
        rows.append(dict(prec=prec, t_hot=t_hot, t_cold=t_cold, td_hot=td_hot, td_cold=td_cold, tops=ops / t_cold / 1e6,
                         frac=ops / t_cold / 1e6 / SPARSE_PEAK[prec], hbm=alg / t_cold / 1e6 / 8.0, sets=n_sets, kernel=kernel,
                         t_same=t_same, ideal=ideal_speedup(M, K, N, prec), frac_measured=(ops / t_cold / 1e6 / mp) if mp else float("nan")))
        del sets
        torch.cuda.empty_cache()
    return rows


def full_depth_row(cfg, prec, iters):
    """every linear layer of the model, depth times, each layer with weights of its own"""
    dev = torch.device("cuda")
    M, depth = cfg["M"], cfg["depth"]
    kinds = []  # per GEMM kind: one SparseLinear per layer (sharing activations, codes and output), its input, its bias
    weights_bytes = 0
    ops = 0.0
    for name, K, N, gelu, _dist in cfg["layers"]:
        X = torch.randn(M, K, device=dev).half()
        bias = torch.randn(N, device=dev) * 0.01
        lins = []
        for layer in range(depth):
            lin = SparseLinear(M, K, N, prec, gelu=gelu, bias=True)
            if lins:  # the activation-side buffers are shared between the layers of a kind
                for nm in ("Y", "Xq", "act_scale", "workspace", "W_pruned", "values", "meta"):
                    if hasattr(lins[0], nm):
                        setattr(lin, nm, getattr(lins[0], nm))
            lin.prepare_weights(torch.randn(N, K, device=dev) * 0.02, fused=K * 4 <= 64 * 1024)
            weights_bytes += lin.packed.numel()
            lins.append(lin)
        if prec == "int8":
            lins[0].quantize_activations(X)
        kinds.append((lins, X, bias))
        ops += 2.0 * M * N * K * depth

    def sparse_pass():
        for layer in range(depth):
            for lins, X, bias in kinds:
                lins[layer].gemm(X, bias)

    def dense_pass():
        for layer in range(depth):
            for lins, X, bias in kinds:
                lins[layer].gemm_dense(X, bias)
    t_s = _time([sparse_pass], iters)
    t_d = _time([dense_pass], iters)
    del kinds
    torch.cuda.empty_cache()
    return dict(t_sparse=t_s, t_dense=t_d, ops=ops, launches=4 * depth, weights_mb=weights_bytes / 1e6)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="")
    ap.add_argument("--iters", type=int, default=30)
    ap.add_argument("--configs", default="c0,c1,c2,c3,c4_vitl,c4_vith")
    ap.add_argument("--only-blocks", action="store_true", help="skip the per-layer and patch-embedding tables")
    ap.add_argument("--only-int4", action="store_true", help="only the INT4 format table")
    a = ap.parse_args()
    lines = ["Sparse GEMM against its dense twin per linear layer.  The dense twin is the dense instantiation of tile kernel 3 (two workgroups "
             "per CU); `same template` is the sparse instantiation of that kernel, `sparse` the kernel the size rules pick (column `kernel`).  "
             "`ideal` = both sides on their own roofline at the nominal peaks (sparse 10.07 / 5.03, dense 5.03 / 2.52 P(FL)OP/s, 8 TB/s).", "",
             "| config | layer | M | K | N | GELU | path | kernel | sparse cold us | sparse hot us | same template cold us | dense cold us | dense hot us | "
             "speedup (cold) | same-template speedup | ideal | TOPS dense-equiv. (cold) | of nominal sparse peak | of measured sparse peak | "
             "of 8 TB/s (algorithmic bytes) |",
             "|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    totals = {}
    for cfg_name in ([] if a.only_blocks or a.only_int4 else a.configs.split(",")):
        cfg = synth.CONFIGS[cfg_name]
        M = cfg["M"]
        for name, K, N, gelu, _dist in cfg["layers"]:
            for r in layer_rows(M, K, N, gelu, a.iters):
                lines.append("| %s | %s | %d | %d | %d | %s | %s | %d | %.1f | %.1f | %.1f | %.1f | %.1f | %.2f | %.2f | %.2f | %.0f | %.3f | %.3f | %.3f |" % (
                    cfg_name, name, M, K, N, "yes" if gelu else "no", r["prec"], r["kernel"], r["t_cold"], r["t_hot"], r["t_same"], r["td_cold"],
                    r["td_hot"], r["td_cold"] / r["t_cold"], r["td_cold"] / r["t_same"], r["ideal"], r["tops"], r["frac"], r["frac_measured"],
                    r["hbm"]))
                key = (cfg_name, r["prec"])
                t = totals.setdefault(key, [0.0, 0.0, 0.0])
                t[0] += r["t_cold"] * cfg["depth"]
                t[1] += r["td_cold"] * cfg["depth"]
                t[2] += 2.0 * M * N * K * cfg["depth"]
                print(lines[-1], flush=True)
    lines += ["", "Whole configuration, sum of the per-layer times above x depth (cold activation buffers, one weight set):", "",
              "| config | path | sparse ms | dense ms | speedup | TOPS dense-equiv. |", "|---|---|---|---|---|---|"]
    for (cfg_name, prec), (ts, td, ops) in totals.items():
        lines.append("| %s | %s | %.3f | %.3f | %.2f | %.0f |" % (cfg_name, prec, ts / 1e3, td / 1e3, td / ts, ops / ts / 1e6))
    lines += ["", "Full-depth pass over all linear layers, timed as one sequence of 4 x depth launches with DISTINCT weights per layer (the "
              "weights of a layer are not cached from the layer before) and one activation / output buffer per kind of GEMM:", "",
              "| config | path | depth | launches | packed weights MB | sparse ms | dense ms | speedup | TOPS dense-equiv. |", "|---|---|---|---|---|---|---|---|---|"]
    for cfg_name in ([] if a.only_blocks or a.only_int4 else a.configs.split(",")):
        cfg = synth.CONFIGS[cfg_name]
        if cfg["depth"] <= 1:
            continue
        for prec in ("int8", "fp16"):
            r = full_depth_row(cfg, prec, max(3, a.iters // 10))
            lines.append("| %s | %s | %d | %d | %.0f | %.3f | %.3f | %.2f | %.0f |" % (cfg_name, prec, cfg["depth"], r["launches"], r["weights_mb"],
                                                                                r["t_sparse"] / 1e3, r["t_dense"] / 1e3, r["t_dense"] / r["t_sparse"],
                                                                                r["ops"] / r["t_sparse"] / 1e6))
            print(lines[-1], flush=True)
    lines += ["", "Patch embedding (a convolution with kernel = stride = P, run as quantise + im2col + sparse GEMM; images N(0,1) fp16, "
              "hot buffers):", "", "| model | images | P | M | K | N | path | quantise us | im2col us | sparse GEMM us | whole layer us | whole layer, patches "
              "gathered by the GEMM (P = 16) us |", "|---|---|---|---|---|---|---|---|---|---|---|---|"]
    dev = torch.device("cuda")
    for model, B, HW, P, D in [] if a.only_blocks or a.only_int4 else [("ViT-B/16, batch 64", 64, 224, 16, 768), ("ViT-L/16, batch 256", 256, 224, 16, 1024),
                                                      ("ViT-H/14, batch 256", 256, 224, 14, 1280)]:
        img = torch.randn(B, 3, HW, HW, device=dev).half()
        Wc = torch.randn(D, 3, P, P, device=dev) * 0.02
        bias = torch.randn(D, device=dev) * 0.01
        for prec in ("int8", "fp16"):
            t_fused = None
            if P == 16:
                pf = SparsePatchEmbed(B, 3, HW, HW, P, D, prec, fused=True)
                pf.prepare_weights(Wc)
                t_fused = _time([lambda: pf.forward(img, bias)], a.iters)
                del pf
            pe = SparsePatchEmbed(B, 3, HW, HW, P, D, prec, fused=False)
            pe.prepare_weights(Wc)
            pe.forward(img, bias)
            t_all = _time([lambda: pe.forward(img, bias)], a.iters)
            t_gemm = _time([lambda: pe.linear.gemm(pe.X, bias)], a.iters)
            src = pe.img_q if prec == "int8" else img
            t_i2c = _time([lambda: G.im2col_patches(src, P, pe.K_pad)], a.iters)
            t_q = _time([lambda: G.quantize_int8(img.reshape(1, -1), G.PER_TENSOR)], a.iters) if prec == "int8" else 0.0
            lines.append("| %s | %dx3x%dx%d | %d | %d | %d | %d | %s | %.1f | %.1f | %.1f | %.1f | %s |" % (
                model, B, HW, HW, P, pe.M, pe.K_pad, D, prec, t_q, t_i2c, t_gemm, t_all, "%.1f" % t_fused if t_fused else "-"))
            print(lines[-1], flush=True)
            del pe
            torch.cuda.empty_cache()
    lines += ["", "Linear layers of one encoder block on the INT8 path (qkv, proj, fc1 + GELU, fc2; attention and normalisation left out: "
              "proj and fc1 read buffers that nothing refreshes), us per block, hot buffers.  Unchained: every layer writes fp16 and the next "
              "one quantises it with a dynamic per-tensor scale (12 launches).  Chained: static scales, the re-quantisation fused into the "
              "producer's epilogue (6 launches), launched one by one or replayed as one HIP graph:", "",
              "| model | M | D | hidden | unchained us | chained us | chained, HIP graph us |", "|---|---|---|---|---|---|---|"]
    for model, M, D, hidden in [] if a.only_int4 else [("DeiT-Tiny, batch 1", 197, 192, 768), ("DeiT-Small, batch 1", 197, 384, 1536), ("ViT-B/16, batch 1", 197, 768, 3072),
                                ("ViT-B/16, batch 8", 1576, 768, 3072), ("ViT-B/16, batch 64", 12608, 768, 3072)]:
        shapes = [(3 * D, D), (D, D), (hidden, D), (D, hidden)]
        Ws = [torch.randn(n, k, device=dev) * 0.02 for n, k in shapes]
        bs = [torch.randn(n, device=dev) * 0.01 for n, k in shapes]
        x = torch.randn(M, D, device=dev).half()
        sc = {k: torch.full((1,), v, dtype=torch.float32, device=dev) for k, v in dict(x=0.03, qkv=0.01, attn=0.01, h=0.01, g=0.01).items()}
        blk = EncoderBlockLinears(M, D, hidden, sc)
        blk.prepare_weights(*Ws)
        nothing = lambda q, out: None
        t_chain = _time([lambda: blk.forward(x, bs, nothing)], a.iters)
        blk.capture(x, bs, nothing)
        t_graph = _time([blk.replay], a.iters)
        lins = [SparseLinear(M, k, n, "int8", gelu=(i == 2)) for i, (n, k) in enumerate(shapes)]
        for lin, W in zip(lins, Ws):
            lin.prepare_weights(W)
        xin = [x, torch.randn(M, D, device=dev).half(), torch.randn(M, D, device=dev).half(), None]

        def unchained():
            lins[0].forward(xin[0], bs[0])
            lins[1].forward(xin[1], bs[1])
            h = lins[2].forward(xin[2], bs[2])
            lins[3].forward(h, bs[3])
        t_un = _time([unchained], a.iters)
        lines.append("| %s | %d | %d | %d | %.1f | %.1f | %.1f |" % (model, M, D, hidden, t_un, t_chain, t_graph))
        print(lines[-1], flush=True)
        del blk, lins
        torch.cuda.empty_cache()
    lines += ["", "INT4 weights in the pair-wise 4:8 format (4 kept 4-bit codes + two 2-bit indices per chunk of 8 = 2.5 bits per weight); the "
              "product runs on the decoded INT8 operand with the dense kernel, or, for tensors pruned with one kept sub-chunk per group of 4 (pair-wise "
              "4:8 and 2:4 at once), on the sparse kernel after a direct conversion of the INT4 storage into its 2:4 INT8 operand.  Weight-side kernels (us, and GB/s over the bytes each must "
              "move), then one layer at M rows: decode + dense INT8 GEMM against the 2:4 INT8 sparse GEMM:", "",
              "| layer | N | K | prune us (GB/s) | quantise us (GB/s) | compress us (GB/s) | decode us (GB/s) | compressed bytes | M | "
              "decode + dense GEMM us | 2:4 INT8 sparse GEMM us | one kept sub-chunk per group of 4: INT4 storage -> 2:4 form us | pack us | "
              "sparse GEMM on it us |", "|---|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    for layer, N, K, M in [("ViT-B fc1", 3072, 768, 12608), ("ViT-B fc2", 768, 3072, 12608), ("ViT-H fc1", 5120, 1280, 65792)]:
        W = torch.randn(N, K, device=dev) * 0.02
        bias = torch.randn(N, device=dev) * 0.01
        P = G.prune_4to8_pairs(W)
        Q, s4 = G.quantize_rows_int4(P)
        v, m = G.compress_int4(Q)
        D = G.decompress_int4(v, m, K)
        L, st = G.lib(), G._stream
        from .pipeline import _p
        t_p = _time([lambda: L.gpusq_prune_4to8_pairs(_p(W), _p(P), None, 0, N, K, st())], a.iters)
        t_q = _time([lambda: L.gpusq_quantize_rows_int4(_p(P), G.F32, _p(Q), _p(s4), 0, N, K, st())], a.iters)
        t_c = _time([lambda: L.gpusq_compress_int4(_p(Q), _p(v), _p(m), None, N, K, st())], a.iters)
        t_d = _time([lambda: L.gpusq_decompress_int4(_p(v), _p(m), _p(D), N, K, st())], a.iters)
        comp = v.numel() + m.numel()
        lin = SparseLinear(M, K, N, "int8", gelu=False, bias=True)
        lin.prepare_weights(W, fused=K * 4 <= 64 * 1024)
        X = torch.randn(M, K, device=dev).half()
        lin.quantize_activations(X)
        t_sparse = _time([lambda: lin.gemm(X, bias)], a.iters)

        def int4_layer():
            L.gpusq_decompress_int4(_p(v), _p(m), _p(D), N, K, st())
            L.gpusq_gemm_int8_dense(_p(lin.Xq), _p(D), _p(lin.act_scale), _p(s4), _p(bias), _p(lin.Y), G.F16, None, M, N, K, G.EPI_BIAS, st())
        t_int4 = _time([int4_layer], a.iters)
        # the 2:4-compatible variant: the INT4 storage becomes the sparse kernel's operand
        Q1, s41 = G.quantize_rows_int4(G.prune_4to8_pairs(W, one_per_group=True))
        v1, m1 = G.compress_int4(Q1)
        v8, m8 = G.int4_to_sparse_int8(v1, m1, K)
        packed = G.pack(v8, m8, K)
        t_24 = _time([lambda: L.gpusq_int4_to_sparse_int8(_p(v1), _p(m1), _p(v8), _p(m8), None, N, K, st())], a.iters)
        t_pk = _time([lambda: L.gpusq_pack(_p(v8), _p(m8), _p(packed), G.I8, N, K, st())], a.iters)
        t_sp4 = _time([lambda: L.gpusq_spgemm_int8(_p(lin.Xq), _p(packed), _p(lin.act_scale), _p(s41), _p(bias), _p(lin.Y), G.F16, None,
                                                   M, N, K, G.EPI_BIAS, st())], a.iters)
        gbs = lambda nbytes, us: nbytes / us / 1e3
        lines.append("| %s | %d | %d | %.1f (%.0f) | %.1f (%.0f) | %.1f (%.0f) | %.1f (%.0f) | %d | %d | %.1f | %.1f | %.1f | %.1f | %.1f |" % (
            layer, N, K, t_p, gbs(8 * N * K, t_p), t_q, gbs(9 * N * K, t_q), t_c, gbs(N * K + comp, t_c), t_d, gbs(N * K + comp, t_d),
            comp, M, t_int4, t_sparse, t_24, t_pk, t_sp4))
        print(lines[-1], flush=True)
        del lin
        torch.cuda.empty_cache()
    text = "\n".join(lines) + "\n"
    print(text)
    if a.out:
        with open(a.out, "w") as fh:
            fh.write(text)


if __name__ == "__main__":
    main()
