"""One linear layer's full path with preallocated device buffers: prune -> quantise -> compress -> pack (weight
side), quantise activations, sparse GEMM with fused epilogue.  Every step is one call into libgpusq through ctypes;
this class only owns the buffers and passes pointers (PyTorch = device memory + current stream).
"""
import ctypes

import torch

from . import gpusq as G


def _p(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


class SparseLinear:
    """Buffers and call sequence for Y = act(X W^T + b) with 2:4-pruned W [N,K].

    precision 'int8': per-output-channel int8 weights, per-tensor int8 activations, int32 accumulation.
    precision 'fp16': fp16 weights and activations, fp32 accumulation.
    x_dtype: dtype of the activations handed in (fp16, or fp32 for the int8 path)."""

    def __init__(self, M, K, N, precision="int8", gelu=False, bias=True, out_dtype=torch.float16, x_dtype=torch.float16,
                 device="cuda"):
        assert precision in ("int8", "fp16")
        self.M, self.K, self.N, self.precision, self.gelu = M, K, N, precision, gelu
        self.out_dtype = out_dtype if precision == "int8" else torch.float16
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=device)
        self.W_pruned = e((N, K), torch.float32)
        self.epilogue = (G.EPI_BIAS if bias else 0) | (G.EPI_GELU if gelu else 0)
        wdt = torch.int8 if precision == "int8" else torch.float16
        self.W_low = e((N, K), wdt)  # quantised (int8) or rounded (fp16) masked weights: also the dense twin's operand
        self.values = e((N, K // 2), wdt)
        self.meta = e((N, G.meta_row_bytes(K)), torch.uint8)
        self.packed = e((G.packed_bytes(wdt, N, K),), torch.uint8)
        self.Y = e((M, N), self.out_dtype)
        if precision == "int8":
            self.w_scale = e((N,), torch.float32)
            self.act_scale = e((1,), torch.float32)
            self.Xq = e((M, K), torch.int8)
            self.workspace = e((max(G.lib().gpusq_quantize_workspace_bytes(G.PER_TENSOR, M, K), 16),), torch.uint8)
        self.x_dtype = x_dtype

    # ---- weight side (a1, a2, a3 + packing) -------------------------------------------------------------------
    def prepare_weights(self, W, fused=True, intermediates=True):
        """fused=True: one launch (gpusq_prepare_weights); fused=False: the four separate calls.
        intermediates=False (fused only): the pruned fp32 weights, the masked low-precision weights, the canonical values
        and metadata stay in the kernel's registers; only what the sparse GEMM reads (packed operand, scales) is written."""
        L, s = G.lib(), G._stream()
        N, K = self.N, self.K
        if fused and K * 4 <= 64 * 1024:
            keep = (lambda t: _p(t)) if intermediates else (lambda t: None)
            G._check(L.gpusq_prepare_weights(_p(W), G.I8 if self.precision == "int8" else G.F16, keep(self.W_pruned),
                                             keep(self.W_low), _p(self.w_scale) if self.precision == "int8" else None,
                                             keep(self.values), keep(self.meta), _p(self.packed), N, K, s), "gpusq_prepare_weights")
            return
        G._check(L.gpusq_prune_2to4(_p(W), _p(self.W_pruned), None, G.F32, N, K, s), "gpusq_prune_2to4")
        if self.precision == "int8":
            G._check(L.gpusq_quantize_int8(_p(self.W_pruned), G.F32, _p(self.W_low), _p(self.w_scale), G.PER_ROW, 0, N, K,
                                           None, s), "gpusq_quantize_int8")
            dt = G.I8
        else:
            G._check(L.gpusq_cast_f16(_p(self.W_pruned), _p(self.W_low), N * K, s), "gpusq_cast_f16")
            dt = G.F16
        G._check(L.gpusq_compress(_p(self.W_low), _p(self.values), _p(self.meta), None, dt, N, K, s), "gpusq_compress")
        G._check(L.gpusq_pack(_p(self.values), _p(self.meta), _p(self.packed), dt, N, K, s), "gpusq_pack")

    # ---- activation side + GEMM (a4, a5, a6) --------------------------------------------------------------------
    def quantize_activations(self, X, static=False):
        """static=True: act_scale already holds a calibrated scale and is used as it is (one launch, no range pass)"""
        G._check(G.lib().gpusq_quantize_int8(_p(X), G._TORCH_DT[X.dtype], _p(self.Xq), _p(self.act_scale), G.PER_TENSOR,
                                             1 if static else 0, self.M, self.K, _p(self.workspace), G._stream()),
                 "gpusq_quantize_int8")

    def gemm(self, X, bias, out_scale=None):
        L, s = G.lib(), G._stream()
        M, N, K = self.M, self.N, self.K
        if self.precision == "int8":
            G._check(L.gpusq_spgemm_int8(_p(self.Xq), _p(self.packed), _p(self.act_scale), _p(self.w_scale), _p(bias),
                                         _p(self.Y), G._TORCH_DT[self.out_dtype], _p(out_scale), M, N, K, self.epilogue, s),
                     "gpusq_spgemm_int8")
        else:
            G._check(L.gpusq_spgemm_fp16(_p(X), _p(self.packed), _p(bias), _p(self.Y), M, N, K, self.epilogue, s),
                     "gpusq_spgemm_fp16")
        return self.Y

    def takes_fp16_input(self):
        """True when the INT8 GEMM of this layer should quantise fp16 activations itself (static scale): the problem
        goes to the latency kernel, the only one that can, K is short and the rows are few (one round of workgroups).  Every workgroup quantises the X rows of its
        own tile, K step by K step, which costs it about 0.5 us per step; the launch this saves is worth 2.5-3 us
        (measured per block at batch 1: K = 192 29 -> 25 us, K = 384 30 -> 29 us, K = 768 34 -> 43 us)."""
        return (self.precision == "int8" and self.K <= 384 and self.M <= 256 and
                G.spgemm_plan(torch.int8, self.M, self.N, self.K, self.epilogue)["kernel"] < 2)

    def gemm_from_f16(self, X, bias, out_scale=None):
        """INT8 path with a static act_scale: quantise + GEMM in one launch (see takes_fp16_input)"""
        G._check(G.lib().gpusq_spgemm_int8_xf16(_p(X), _p(self.packed), _p(self.act_scale), _p(self.w_scale), _p(bias), _p(self.Y),
                                                G._TORCH_DT[self.out_dtype], _p(out_scale), self.M, self.N, self.K, self.epilogue,
                                                G._stream()), "gpusq_spgemm_int8_xf16")
        return self.Y

    def gemm_dense(self, X, bias, out_scale=None):
        """the dense twin on the same masked weights"""
        L, s = G.lib(), G._stream()
        M, N, K = self.M, self.N, self.K
        if self.precision == "int8":
            G._check(L.gpusq_gemm_int8_dense(_p(self.Xq), _p(self.W_low), _p(self.act_scale), _p(self.w_scale), _p(bias),
                                             _p(self.Y), G._TORCH_DT[self.out_dtype], _p(out_scale), M, N, K, self.epilogue,
                                             s), "gpusq_gemm_int8_dense")
        else:
            G._check(L.gpusq_gemm_fp16_dense(_p(X), _p(self.W_low), _p(bias), _p(self.Y), M, N, K, self.epilogue, s),
                     "gpusq_gemm_fp16_dense")
        return self.Y

    def forward(self, X, bias, out_scale=None):
        if self.precision == "int8":
            self.quantize_activations(X)
        return self.gemm(X, bias, out_scale)

    def full_path(self, W, X, bias, out_scale=None):
        """all steps of the path in order, as one benchmark step times them"""
        self.prepare_weights(W)
        return self.forward(X, bias, out_scale)


class SparsePatchEmbed:
    """Patch embedding (a convolution with kernel = stride = P) on the sparse GEMM: images [B,C,H,W] -> tokens
    [B*(H/P)*(W/P), D].  The weight [D,C,P,P] is flattened to [D, C*P*P] (zero-padded to whole 128-byte K steps) and
    prepared like a linear layer's; an image is (quantised per tensor and) cut into flattened patches by
    gpusq_im2col_patches, then multiplied by gpusq_spgemm_*; with P = 16 (and a problem large enough for the tile kernel)
    gpusq_patch_embed16_* lets the GEMM gather the patches itself (fused=True, the default where it applies: it saves
    the im2col pass, most on the fp16 path, where a patch row is 32 contiguous bytes; a 16-byte piece of an int8 patch
    row touches a cache line of its own, which gives part of the saving back)."""

    def __init__(self, B, C, H, W, P, D, precision="int8", bias=True, device="cuda", fused=None):
        self.shape = (B, C, H, W)
        can_fuse = P == 16 and B * (H // P) * (W // P) * D > 256 * 1024
        self.fused = can_fuse if fused is None else (fused and can_fuse)
        self.P, self.D, self.precision = P, D, precision
        self.K = C * P * P
        step = 128 if precision == "int8" else 64  # whole 128-byte K steps: the tile kernel's requirement
        self.K_pad = -(-self.K // step) * step
        self.M = B * (H // P) * (W // P)
        self.linear = SparseLinear(self.M, self.K_pad, D, precision, gelu=False, bias=bias, device=device)
        xdt = torch.int8 if precision == "int8" else torch.float16
        self.X = torch.empty((self.M, self.K_pad), dtype=xdt, device=device)
        if precision == "int8":
            n = B * C * H * W
            self.img_q = torch.empty((B, C, H, W), dtype=torch.int8, device=device)
            self.workspace = torch.empty((max(G.lib().gpusq_quantize_workspace_bytes(G.PER_TENSOR, 1, n), 16),), dtype=torch.uint8,
                                         device=device)

    def prepare_weights(self, Wc):
        """Wc [D,C,P,P] fp32"""
        Wflat = torch.zeros((self.D, self.K_pad), dtype=torch.float32, device=Wc.device)
        Wflat[:, :self.K] = Wc.reshape(self.D, self.K)
        self.linear.prepare_weights(Wflat, fused=self.K_pad * 4 <= 64 * 1024)

    def forward(self, img, bias):
        """img [B,C,H,W] fp16 (or fp32 on the int8 path)"""
        L, s = G.lib(), G._stream()
        B, C, H, W = self.shape
        if self.precision == "int8":
            G._check(L.gpusq_quantize_int8(_p(img), G._TORCH_DT[img.dtype], _p(self.img_q), _p(self.linear.act_scale), G.PER_TENSOR, 0,
                                           1, B * C * H * W, _p(self.workspace), s), "gpusq_quantize_int8")
            src, dt = self.img_q, G.I8
        else:
            src, dt = img, G.F16
        if self.fused:
            lin, epi = self.linear, self.linear.epilogue & G.EPI_BIAS
            if self.precision == "int8":
                G._check(L.gpusq_patch_embed16_int8(_p(src), _p(lin.packed), _p(lin.act_scale), _p(lin.w_scale), _p(bias), _p(lin.Y),
                                                    B, C, H, W, self.D, epi, s), "gpusq_patch_embed16_int8")
            else:
                G._check(L.gpusq_patch_embed16_fp16(_p(src), _p(lin.packed), _p(bias), _p(lin.Y), B, C, H, W, self.D, epi, s),
                         "gpusq_patch_embed16_fp16")
            return lin.Y
        G._check(L.gpusq_im2col_patches(_p(src), _p(self.X), dt, B, C, H, W, self.P, self.K_pad, s), "gpusq_im2col_patches")
        if self.precision == "int8":
            self.linear.Xq = self.X
        return self.linear.gemm(self.X, bias)


class EncoderBlockLinears:
    """The four linear layers of one encoder block (qkv, proj, fc1, fc2) on the INT8 path with static, calibrated
    activation scales, the deployment form with quantise / dequantise nodes around every linear layer: the
    re-quantisation of a layer's output with the next layer's input scale is fused into its epilogue (qkv -> int8,
    fc1 -> GELU -> int8, which fc2 reads directly), so one block is six launches of the library:
        quantise x, qkv, [attention], proj, [residual + norm], quantise h, fc1 (GELU), fc2;
    with few rows (problems of the latency kernel) qkv and fc1 quantise their fp16 input on the way in: four launches.
    Attention and the normalisation are not part of the library: `attention(qkv_int8 [M,3D], out_int8 [M,D])` and
    `norm(proj_fp16 [M,D]) -> fp16 [M,D]` are the caller's (stubs in the tests and the report).  capture() records the
    whole sequence into a HIP graph, which takes the host out of the loop.

    scales: dict of 1-element fp32 device tensors: x (block input), qkv (qkv output), attn (attention output),
    h (fc1 input), g (GELU output = fc2 input)."""

    def __init__(self, M, D, hidden, scales, device="cuda"):
        self.M, self.D, self.hidden = M, D, hidden
        self.qkv = SparseLinear(M, D, 3 * D, "int8", out_dtype=torch.int8, device=device)
        self.proj = SparseLinear(M, D, D, "int8", out_dtype=torch.float16, device=device)
        self.fc1 = SparseLinear(M, D, hidden, "int8", gelu=True, out_dtype=torch.int8, device=device)
        self.fc2 = SparseLinear(M, hidden, D, "int8", out_dtype=torch.float16, device=device)
        self.scales = scales
        self.qkv.act_scale = scales["x"]
        self.proj.act_scale = scales["attn"]
        self.fc1.act_scale = scales["h"]
        self.fc2.act_scale = scales["g"]
        self.fc2.Xq = self.fc1.Y  # fc2 reads the codes fc1's epilogue wrote: no pass in between
        # few rows (the latency kernel): qkv and fc1 quantise their fp16 input themselves, four launches per block
        self.fold_quantise = self.qkv.takes_fp16_input() and self.fc1.takes_fp16_input()
        self.graph = None

    def prepare_weights(self, Wqkv, Wproj, Wfc1, Wfc2):
        for lin, W in ((self.qkv, Wqkv), (self.proj, Wproj), (self.fc1, Wfc1), (self.fc2, Wfc2)):
            lin.prepare_weights(W)

    def forward(self, x, biases, attention, norm=None):
        """x fp16 [M,D]; biases: (b_qkv, b_proj, b_fc1, b_fc2); returns fc2's fp16 output [M,D] (a buffer of this object)"""
        if self.fold_quantise:
            self.qkv.gemm_from_f16(x, biases[0], self.scales["qkv"])
        else:
            self.qkv.quantize_activations(x, static=True)
            self.qkv.gemm(None, biases[0], self.scales["qkv"])
        attention(self.qkv.Y, self.proj.Xq)
        h = self.proj.gemm(None, biases[1])
        if norm is not None:
            h = norm(h)
        if self.fold_quantise:
            self.fc1.gemm_from_f16(h, biases[2], self.scales["g"])
        else:
            self.fc1.quantize_activations(h, static=True)
            self.fc1.gemm(None, biases[2], self.scales["g"])
        return self.fc2.gemm(None, biases[3])

    def capture(self, x, biases, attention, norm=None):
        """Records forward() on these buffers into a HIP graph (after one eager run that loads every kernel); replay()
        then reruns it on whatever x and the biases hold at that time."""
        self.forward(x, biases, attention, norm)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self.forward(x, biases, attention, norm)
        return self.graph

    def replay(self):
        self.graph.replay()
        return self.fc2.Y
