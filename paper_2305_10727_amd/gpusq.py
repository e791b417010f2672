"""Thin ctypes binding over libgpusq.so (include/gpusq.h).  Argument marshalling only: every step of the path runs
in the library's HIP kernels.  PyTorch supplies device memory (`torch.empty`) and the current HIP stream.

There is no fallback: if the library has not been built, or no GPU tensor is passed, the calls raise.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgpusq.so")

OK, ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_UNSUPPORTED, ERR_HIP = range(6)
F32, F16, I8, I32 = range(4)
EPI_NONE, EPI_BIAS, EPI_GELU = 0, 1, 2
PER_ROW, PER_TENSOR = 0, 1

_TORCH_DT = {torch.float32: F32, torch.float16: F16, torch.int8: I8, torch.int32: I32}
_DT_TORCH = {v: k for k, v in _TORCH_DT.items()}

EXPORTS = [
    "gpusq_status_string", "gpusq_last_hip_error", "gpusq_version", "gpusq_prune_2to4", "gpusq_cast_f16",
    "gpusq_quantize_workspace_bytes",
    "gpusq_quantize_int8", "gpusq_compress", "gpusq_check_2to4", "gpusq_decompress", "gpusq_packed_bytes", "gpusq_pack", "gpusq_prepare_weights", "gpusq_spgemm_fp16",
    "gpusq_spgemm_int8", "gpusq_spgemm_int8_xf16", "gpusq_spgemm_plan", "gpusq_im2col_patches", "gpusq_patch_embed16_int8", "gpusq_patch_embed16_fp16", "gpusq_gemm_fp16_dense", "gpusq_gemm_int8_dense",
    "gpusq_prune_4to8_pairs", "gpusq_quantize_rows_int4", "gpusq_compress_int4", "gpusq_decompress_int4",
    "gpusq_int4_to_sparse_int8", "gpusq_prune_n_of_m", "gpusq_force_kernel",
    "gpusq_quantize_tensor_int8_noalloc",
]


class GpusqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().gpusq_status_string(status).decode()
        if status == ERR_HIP:
            msg += " [hip error %d]" % lib().gpusq_last_hip_error()
        super().__init__("%s: %s" % (where, msg))


_lib = None


def lib():
    """Loads libgpusq.so (built by `python -m paper_2305_10727_amd.build`); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libgpusq.so is not built: run `python -m paper_2305_10727_amd.build` (needs hipcc)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.gpusq_status_string.restype = ctypes.c_char_p
        L.gpusq_status_string.argtypes = [ci]
        L.gpusq_last_hip_error.restype = ci
        L.gpusq_version.restype = ci
        L.gpusq_prune_2to4.argtypes = [vp, vp, vp, ci, i64, i64, vp]
        L.gpusq_cast_f16.argtypes = [vp, vp, i64, vp]
        L.gpusq_quantize_workspace_bytes.restype = ctypes.c_size_t
        L.gpusq_quantize_workspace_bytes.argtypes = [ci, i64, i64]
        L.gpusq_quantize_int8.argtypes = [vp, ci, vp, vp, ci, ci, i64, i64, vp, vp]
        L.gpusq_quantize_tensor_int8_noalloc.argtypes = [vp, ci, vp, vp, ci, i64, i64, vp]
        L.gpusq_quantize_tensor_int8_noalloc.restype = ci
        L.gpusq_compress.argtypes = [vp, vp, vp, vp, ci, i64, i64, vp]
        L.gpusq_check_2to4.argtypes = [vp, ci, vp, i64, i64, vp]
        L.gpusq_check_2to4.restype = ci
        L.gpusq_decompress.argtypes = [vp, vp, vp, ci, i64, i64, vp]
        L.gpusq_packed_bytes.restype = ctypes.c_size_t
        L.gpusq_packed_bytes.argtypes = [ci, i64, i64]
        L.gpusq_pack.argtypes = [vp, vp, vp, ci, i64, i64, vp]
        L.gpusq_prepare_weights.argtypes = [vp, ci, vp, vp, vp, vp, vp, vp, i64, i64, vp]
        L.gpusq_prepare_weights.restype = ci
        L.gpusq_spgemm_fp16.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp]
        L.gpusq_spgemm_int8.argtypes = [vp, vp, vp, vp, vp, vp, ci, vp, i64, i64, i64, ci, vp]
        L.gpusq_spgemm_int8_xf16.argtypes = [vp, vp, vp, vp, vp, vp, ci, vp, i64, i64, i64, ci, vp]
        L.gpusq_spgemm_int8_xf16.restype = ci
        L.gpusq_gemm_fp16_dense.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp]
        L.gpusq_gemm_int8_dense.argtypes = [vp, vp, vp, vp, vp, vp, ci, vp, i64, i64, i64, ci, vp]
        L.gpusq_im2col_patches.argtypes = [vp, vp, ci, i64, i64, i64, i64, i64, i64, vp]
        L.gpusq_patch_embed16_int8.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, ci, vp]
        L.gpusq_patch_embed16_fp16.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, ci, vp]
        L.gpusq_spgemm_plan.argtypes = [ci, i64, i64, i64, ci, ci, ctypes.POINTER(ctypes.c_int32)]
        L.gpusq_force_kernel.argtypes = [ci]
        L.gpusq_force_kernel.restype = ci
        L.gpusq_prune_4to8_pairs.argtypes = [vp, vp, vp, ci, i64, i64, vp]
        L.gpusq_prune_n_of_m.argtypes = [vp, vp, ci, ci, i64, i64, vp]
        L.gpusq_int4_to_sparse_int8.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp]
        L.gpusq_quantize_rows_int4.argtypes = [vp, ci, vp, vp, ci, i64, i64, vp]
        L.gpusq_compress_int4.argtypes = [vp, vp, vp, vp, i64, i64, vp]
        L.gpusq_decompress_int4.argtypes = [vp, vp, vp, i64, i64, vp]
        for name in ("gpusq_prune_2to4", "gpusq_cast_f16", "gpusq_quantize_int8", "gpusq_compress", "gpusq_check_2to4", "gpusq_decompress", "gpusq_pack",
                     "gpusq_spgemm_fp16", "gpusq_spgemm_int8", "gpusq_gemm_fp16_dense", "gpusq_gemm_int8_dense"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("gpusq works on device tensors only")
    if not t.is_contiguous():
        raise ValueError("gpusq needs contiguous tensors")
    return ctypes.c_void_p(t.data_ptr())


# torch's current stream as a raw hipStream_t.  The public route (torch.cuda.current_stream().cuda_stream) builds a Stream
# object per call and takes about 2.7 us, a third of the host time of a launch through this binding; torch's own raw
# accessor takes a tenth of that.  It is looked up once; without it the public route is used.
_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream():
    if _raw_stream is not None:
        return ctypes.c_void_p(_raw_stream(torch.cuda.current_device()))
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, where):
    if status != OK:
        raise GpusqError(status, where)


def meta_row_bytes(K):
    return (K // 4 + 1) // 2


def version():
    return lib().gpusq_version()


def prune_2to4(W, out=None, want_mask=False):
    """gpusq_prune_2to4: W [N,K] fp32/fp16 -> pruned W (and the [N,K/4] keep-mask bytes if asked)."""
    N, K = W.shape
    out = torch.empty_like(W) if out is None else out
    mask = torch.empty((N, max(K // 4, 1)), dtype=torch.uint8, device=W.device) if want_mask else None
    _check(lib().gpusq_prune_2to4(_ptr(W), _ptr(out), _ptr(mask), _TORCH_DT[W.dtype], N, K, _stream()), "gpusq_prune_2to4")
    return (out, mask) if want_mask else out


def cast_f16(X, out=None):
    """gpusq_cast_f16: fp32 tensor -> fp16 tensor of the same shape (round-to-nearest-even)."""
    out = torch.empty(X.shape, dtype=torch.float16, device=X.device) if out is None else out
    _check(lib().gpusq_cast_f16(_ptr(X), _ptr(out), X.numel(), _stream()), "gpusq_cast_f16")
    return out


def quantize_int8(X, mode, scale=None):
    """gpusq_quantize_int8: returns (Xq int8, scale tensor).  mode PER_ROW: scale [rows]; PER_TENSOR: scale [1].
    Pass `scale` (device fp32 tensor) to quantise with given scales."""
    rows, cols = X.shape
    Xq = torch.empty((rows, cols), dtype=torch.int8, device=X.device)
    given = scale is not None
    if not given:
        scale = torch.empty(rows if mode == PER_ROW else 1, dtype=torch.float32, device=X.device)
    ws_bytes = lib().gpusq_quantize_workspace_bytes(mode, rows, cols)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=X.device)
    _check(lib().gpusq_quantize_int8(_ptr(X), _TORCH_DT[X.dtype], _ptr(Xq), _ptr(scale), mode, int(given), rows, cols,
                                     _ptr(ws), _stream()), "gpusq_quantize_int8")
    return Xq, scale


def quantize_tensor_int8_noalloc(X, Xq, scale, scale_is_input=False):
    """gpusq_quantize_tensor_int8_noalloc: per-tensor codes into the caller's Xq [rows, cols] int8 and scale [1] fp32;
    nothing is allocated, here or in the library."""
    rows, cols = X.shape
    _check(lib().gpusq_quantize_tensor_int8_noalloc(_ptr(X), _TORCH_DT[X.dtype], _ptr(Xq), _ptr(scale), int(bool(scale_is_input)),
                                                    rows, cols, _stream()), "gpusq_quantize_tensor_int8_noalloc")
    return Xq, scale


def compress(W, want_violations=False):
    """gpusq_compress: W [N,K] fp16/int8 -> (values [N,K/2], meta [N,ceil(K/8)] uint8[, violations int32[1]])."""
    N, K = W.shape
    values = torch.empty((N, max(K // 2, 1)), dtype=W.dtype, device=W.device)
    meta = torch.empty((N, max(meta_row_bytes(K), 1)), dtype=torch.uint8, device=W.device)
    viol = torch.empty(1, dtype=torch.int32, device=W.device) if want_violations else None
    _check(lib().gpusq_compress(_ptr(W), _ptr(values), _ptr(meta), _ptr(viol), _TORCH_DT[W.dtype], N, K, _stream()),
           "gpusq_compress")
    return (values, meta, viol) if want_violations else (values, meta)


ERR_NOT_2TO4 = 6


def check_2to4(W):
    """gpusq_check_2to4: W [N,K] fp32/fp16/int8 -> (is_2to4, groups with more than two non-zeros); waits for the stream"""
    N, K = W.shape
    viol = torch.empty(1, dtype=torch.int32, device=W.device)
    st = lib().gpusq_check_2to4(_ptr(W), _TORCH_DT[W.dtype], _ptr(viol), N, K, _stream())
    if st not in (0, ERR_NOT_2TO4):
        _check(st, "gpusq_check_2to4")
    return st == 0, int(viol.item())


def decompress(values, meta, K):
    N = values.shape[0]
    W = torch.empty((N, K), dtype=values.dtype, device=values.device)
    _check(lib().gpusq_decompress(_ptr(values), _ptr(meta), _ptr(W), _TORCH_DT[values.dtype], N, K, _stream()),
           "gpusq_decompress")
    return W


def prune_n_of_m(W, n, m):
    """gpusq_prune_n_of_m: W [N,K] fp32 -> copy with the n largest magnitudes of every m contiguous elements kept"""
    N, K = W.shape
    out = torch.empty_like(W)
    _check(lib().gpusq_prune_n_of_m(_ptr(W), _ptr(out), n, m, N, K, _stream()), "gpusq_prune_n_of_m")
    return out


def prune_4to8_pairs(W, want_mask=False, one_per_group=False):
    """gpusq_prune_4to8_pairs: W [N,K] fp32 -> pruned copy (and the keep mask [N,K/8] uint8)"""
    N, K = W.shape
    out = torch.empty_like(W)
    mask = torch.empty((N, K // 8), dtype=torch.uint8, device=W.device) if want_mask else None
    _check(lib().gpusq_prune_4to8_pairs(_ptr(W), _ptr(out), _ptr(mask), int(one_per_group), N, K, _stream()),
           "gpusq_prune_4to8_pairs")
    return (out, mask) if want_mask else out


def int4_to_sparse_int8(values4, meta4, K, want_mismatches=False):
    """gpusq_int4_to_sparse_int8: INT4 pair-wise storage -> (values [N,K/2] int8, meta [N,K/8] uint8[, mismatches int32[1]])"""
    N = values4.shape[0]
    values8 = torch.empty((N, K // 2), dtype=torch.int8, device=values4.device)
    meta8 = torch.empty((N, K // 8), dtype=torch.uint8, device=values4.device)
    bad = torch.empty(1, dtype=torch.int32, device=values4.device) if want_mismatches else None
    _check(lib().gpusq_int4_to_sparse_int8(_ptr(values4), _ptr(meta4), _ptr(values8), _ptr(meta8), _ptr(bad), N, K, _stream()),
           "gpusq_int4_to_sparse_int8")
    return (values8, meta8, bad) if want_mismatches else (values8, meta8)


def quantize_rows_int4(X, scale=None):
    """gpusq_quantize_rows_int4: returns (4-bit codes in an int8 tensor, scale [rows])"""
    rows, cols = X.shape
    Xq = torch.empty((rows, cols), dtype=torch.int8, device=X.device)
    given = scale is not None
    if not given:
        scale = torch.empty(rows, dtype=torch.float32, device=X.device)
    _check(lib().gpusq_quantize_rows_int4(_ptr(X), _TORCH_DT[X.dtype], _ptr(Xq), _ptr(scale), int(given), rows, cols, _stream()),
           "gpusq_quantize_rows_int4")
    return Xq, scale


def compress_int4(Wq, want_violations=False):
    """gpusq_compress_int4: Wq [N,K] int8 (4-bit codes) -> (values [N,K/4] uint8, meta [N,ceil(K/16)] uint8[, violations])"""
    N, K = Wq.shape
    values = torch.empty((N, K // 4), dtype=torch.uint8, device=Wq.device)
    meta = torch.empty((N, (K // 8 + 1) // 2), dtype=torch.uint8, device=Wq.device)
    viol = torch.empty(1, dtype=torch.int32, device=Wq.device) if want_violations else None
    _check(lib().gpusq_compress_int4(_ptr(Wq), _ptr(values), _ptr(meta), _ptr(viol), N, K, _stream()), "gpusq_compress_int4")
    return (values, meta, viol) if want_violations else (values, meta)


def decompress_int4(values, meta, K):
    N = values.shape[0]
    W = torch.empty((N, K), dtype=torch.int8, device=values.device)
    _check(lib().gpusq_decompress_int4(_ptr(values), _ptr(meta), _ptr(W), N, K, _stream()), "gpusq_decompress_int4")
    return W


def im2col_patches(img, P, K_pad=None):
    """gpusq_im2col_patches: img [B,C,H,W] (int8 or fp16) -> flattened patches [B*(H/P)*(W/P), K_pad] (zero-padded columns)"""
    B, C, H, W = img.shape
    K = C * P * P
    K_pad = K if K_pad is None else K_pad
    X = torch.empty((B * (H // P) * (W // P), K_pad), dtype=img.dtype, device=img.device)
    _check(lib().gpusq_im2col_patches(_ptr(img), _ptr(X), _TORCH_DT[img.dtype], B, C, H, W, P, K_pad, _stream()), "gpusq_im2col_patches")
    return X


def patch_embed16(img, packed, D, act_scale=None, w_scale=None, bias=None):
    """gpusq_patch_embed16_int8 / _fp16: img [B,C,H,W] int8 or fp16 -> tokens [B*(H/16)*(W/16), D] fp16 (patches gathered by the GEMM)"""
    B, C, H, W = img.shape
    Y = torch.empty((B * (H // 16) * (W // 16), D), dtype=torch.float16, device=img.device)
    epi = EPI_BIAS if bias is not None else 0
    if img.dtype == torch.int8:
        st = lib().gpusq_patch_embed16_int8(_ptr(img), _ptr(packed), _ptr(act_scale), _ptr(w_scale), _ptr(bias), _ptr(Y), B, C, H, W, D,
                                            epi, _stream())
    else:
        st = lib().gpusq_patch_embed16_fp16(_ptr(img), _ptr(packed), _ptr(bias), _ptr(Y), B, C, H, W, D, epi, _stream())
    _check(st, "gpusq_patch_embed16")
    return Y


def spgemm_plan(dtype, M, N, K, epilogue=0, cus=0):
    """gpusq_spgemm_plan: the tile decomposition of a sparse GEMM (host-side; no GPU needed when cus > 0)."""
    out = (ctypes.c_int32 * 8)()
    _check(lib().gpusq_spgemm_plan(_TORCH_DT[dtype], M, N, K, epilogue, cus, out), "gpusq_spgemm_plan")
    keys = ("kernel", "unit_rows", "tiles_n", "full_tm", "full_chunks", "tail_tm", "tiles", "workgroups")
    return dict(zip(keys, list(out)))


def force_kernel(kernel):
    """gpusq_force_kernel (testing aid): 0 / 1 / 2 = run the sparse GEMMs on that kernel, None or -1 = size rules.
    Returns the previous setting."""
    return lib().gpusq_force_kernel(-1 if kernel is None else int(kernel))


def packed_bytes(dtype, N, K):
    return lib().gpusq_packed_bytes(_TORCH_DT[dtype], N, K)


def pack(values, meta, K):
    """gpusq_pack: canonical (values, meta) -> opaque kernel-native buffer (uint8 tensor)."""
    N = values.shape[0]
    nbytes = packed_bytes(values.dtype, N, K)
    if nbytes == 0:
        raise GpusqError(ERR_SHAPE, "gpusq_packed_bytes")
    packed = torch.empty(nbytes, dtype=torch.uint8, device=values.device)
    _check(lib().gpusq_pack(_ptr(values), _ptr(meta), _ptr(packed), _TORCH_DT[values.dtype], N, K, _stream()), "gpusq_pack")
    return packed


def prepare_weights(W, dtype, want_intermediates=False):
    """gpusq_prepare_weights: fp32 W [N,K] -> packed buffer (+ w_scale for int8) in one launch.
    With want_intermediates also returns W_pruned, W_low, values, meta."""
    N, K = W.shape
    dt = _TORCH_DT[dtype]
    packed = torch.empty(packed_bytes(dtype, N, K), dtype=torch.uint8, device=W.device)
    w_scale = torch.empty(N, dtype=torch.float32, device=W.device) if dtype == torch.int8 else None
    Wp = Wl = values = meta = None
    if want_intermediates:
        Wp = torch.empty_like(W)
        Wl = torch.empty((N, K), dtype=dtype, device=W.device)
        values = torch.empty((N, K // 2), dtype=dtype, device=W.device)
        meta = torch.empty((N, meta_row_bytes(K)), dtype=torch.uint8, device=W.device)
    _check(lib().gpusq_prepare_weights(_ptr(W), dt, _ptr(Wp), _ptr(Wl), _ptr(w_scale), _ptr(values), _ptr(meta), _ptr(packed),
                                       N, K, _stream()), "gpusq_prepare_weights")
    out = dict(packed=packed, w_scale=w_scale)
    if want_intermediates:
        out.update(W_pruned=Wp, W_low=Wl, values=values, meta=meta)
    return out


def _epi(bias, gelu):
    return (EPI_BIAS if bias is not None else 0) | (EPI_GELU if gelu else 0)


def spgemm_fp16(X, Wpacked, N, bias=None, gelu=False, out=None):
    M, K = X.shape
    Y = torch.empty((M, N), dtype=torch.float16, device=X.device) if out is None else out
    _check(lib().gpusq_spgemm_fp16(_ptr(X), _ptr(Wpacked), _ptr(bias), _ptr(Y), M, N, K, _epi(bias, gelu), _stream()),
           "gpusq_spgemm_fp16")
    return Y


def spgemm_int8(Xq, Wpacked, N, act_scale=None, w_scale=None, bias=None, gelu=False, out_dtype=torch.float16,
                out_scale=None, out=None):
    M, K = Xq.shape
    Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device) if out is None else out
    _check(lib().gpusq_spgemm_int8(_ptr(Xq), _ptr(Wpacked), _ptr(act_scale), _ptr(w_scale), _ptr(bias), _ptr(Y),
                                   _TORCH_DT[out_dtype], _ptr(out_scale), M, N, K, _epi(bias, gelu), _stream()),
           "gpusq_spgemm_int8")
    return Y


def spgemm_int8_xf16(X, Wpacked, N, act_scale, w_scale, bias=None, gelu=False, out_dtype=torch.float16, out_scale=None,
                     out=None):
    """X fp16 [M,K], quantised inside the GEMM with the static act_scale (latency kernel only: raises GpusqError with
    ERR_UNSUPPORTED for problems that spgemm_plan assigns to the tile kernel)"""
    M, K = X.shape
    Y = torch.empty((M, N), dtype=out_dtype, device=X.device) if out is None else out
    _check(lib().gpusq_spgemm_int8_xf16(_ptr(X), _ptr(Wpacked), _ptr(act_scale), _ptr(w_scale), _ptr(bias), _ptr(Y),
                                        _TORCH_DT[out_dtype], _ptr(out_scale), M, N, K, _epi(bias, gelu), _stream()),
           "gpusq_spgemm_int8_xf16")
    return Y


def gemm_fp16_dense(X, W, bias=None, gelu=False, out=None):
    M, K = X.shape
    N = W.shape[0]
    Y = torch.empty((M, N), dtype=torch.float16, device=X.device) if out is None else out
    _check(lib().gpusq_gemm_fp16_dense(_ptr(X), _ptr(W), _ptr(bias), _ptr(Y), M, N, K, _epi(bias, gelu), _stream()),
           "gpusq_gemm_fp16_dense")
    return Y


def gemm_int8_dense(Xq, Wq, act_scale=None, w_scale=None, bias=None, gelu=False, out_dtype=torch.float16, out_scale=None,
                    out=None):
    M, K = Xq.shape
    N = Wq.shape[0]
    Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device) if out is None else out
    _check(lib().gpusq_gemm_int8_dense(_ptr(Xq), _ptr(Wq), _ptr(act_scale), _ptr(w_scale), _ptr(bias), _ptr(Y),
                                       _TORCH_DT[out_dtype], _ptr(out_scale), M, N, K, _epi(bias, gelu), _stream()),
           "gpusq_gemm_int8_dense")
    return Y
