"""ctypes binding of the CPU oracle (oracle/gpusq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the CPU-baseline leg of bench.py.  The
product package never imports this module, and this module never imports the product package.
All arrays are numpy; fp16 tensors travel as uint16 bit patterns (numpy float16 arrays are viewed, not converted).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gpusq_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC"]


def build(force=False):
    """Compile the oracle with gcc (plain C, no GPU headers); a forced build also compiles its self-test driver
    (oracle/selftest.c, the program the sanitizer test runs) to check that it builds."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    if force:
        import tempfile
        with tempfile.TemporaryDirectory(prefix="oracle_build_") as tmp:
            flags = [f for f in CFLAGS if f not in ("-shared", "-fPIC")]
            subprocess.check_call(["gcc", *flags, "-o", os.path.join(tmp, "selftest"), os.path.join(_HERE, "selftest.c"), _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_f16_to_f32.restype = ctypes.c_float
        _lib.oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        _lib.oracle_f32_to_f16.restype = ctypes.c_uint16
        _lib.oracle_f32_to_f16.argtypes = [ctypes.c_float]
        _lib.oracle_f64_to_f16.restype = ctypes.c_uint16
        _lib.oracle_f64_to_f16.argtypes = [ctypes.c_double]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16 and dtype == np.uint16:
        a = a.view(np.uint16)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def _i64(x):
    return ctypes.c_int64(int(x))


def num_threads():
    return int(lib().oracle_num_threads())


def meta_row_bytes(K):
    return (K // 4 + 1) // 2


# ---------------------------------------------------------------- fp16 helpers
def f16_to_f32(h):
    return float(lib().oracle_f16_to_f32(int(h)))


def f32_to_f16(f):
    return int(lib().oracle_f32_to_f16(float(np.float32(f))))


def f64_to_f16(d):
    return int(lib().oracle_f64_to_f16(float(d)))


# ---------------------------------------------------------------- a1 prune
def prune_2to4(W):
    """W [N,K] float32 or float16 -> (pruned W, mask bytes [N,K/4]); top-2 |w| per group of 4 along K."""
    W = np.ascontiguousarray(W)
    N, K = W.shape
    mask = np.zeros((N, K // 4), np.uint8)
    if W.dtype == np.float32:
        out = np.empty_like(W)
        r = lib().oracle_prune_2to4_f32(_p(W), _p(out), _p(mask), _i64(N), _i64(K))
    elif W.dtype == np.float16:
        out = np.empty_like(W)
        r = lib().oracle_prune_2to4_f16(_p(W), _p(out), _p(mask), _i64(N), _i64(K))
    else:
        raise TypeError(W.dtype)
    if r != 0:
        raise ValueError("K must be a multiple of 4")
    return out, mask


def prune_n_of_m(W, n, m):
    """W [N,K] float32, K % m == 0: keep the n largest magnitudes of every m contiguous elements of a row"""
    W = _c(W, np.float32)
    N, K = W.shape
    out = np.empty_like(W)
    assert lib().oracle_prune_n_of_m_f32(_p(W), _p(out), int(n), int(m), _i64(N), _i64(K)) == 0
    return out


# ---------------------------------------------------------------- a2 / a4 quantise
def quantize_rows_int8(X, scale=None):
    X = _c(X, np.float32)
    rows, cols = X.shape
    Q = np.empty((rows, cols), np.int8)
    given = scale is not None
    s = _c(scale, np.float32).copy() if given else np.empty(rows, np.float32)
    lib().oracle_quantize_rows_int8(_p(X), _p(Q), _p(s), int(given), _i64(rows), _i64(cols))
    return Q, s


def quantize_tensor_int8(X, scale=None):
    X = _c(X, np.float32)
    Q = np.empty(X.shape, np.int8)
    given = scale is not None
    s = np.array([scale if given else 0.0], np.float32)
    lib().oracle_quantize_tensor_int8(_p(X), _p(Q), _p(s), int(given), _i64(X.size))
    return Q, float(s[0])


# ---------------------------------------------------------------- INT4 pair-wise 4:8
def meta4_row_bytes(K):
    return (K // 8 + 1) // 2


def prune_4to8_pairs(W, one_per_group=False):
    """W [N,K] float32, K % 8 == 0 -> (pruned W, mask bytes [N,K/8]); two of the four 2-wide sub-chunks of every chunk
    of 8 are kept (highest |a| + |b|); one_per_group: one of them in each group of 4, which makes the row 2:4 as well."""
    W = _c(W, np.float32)
    N, K = W.shape
    out = np.empty_like(W)
    mask = np.empty((N, K // 8), np.uint8)
    assert lib().oracle_prune_4to8_pairs_f32(_p(W), _p(out), _p(mask), int(one_per_group), _i64(N), _i64(K)) == 0
    return out, mask


def int4_pairs_to_sparse_int8(values4, meta4, K):
    """INT4 pair-wise storage with one kept sub-chunk per group of 4 -> the INT8 2:4 compressed form
    (values [N,K/2] int8, meta [N,ceil(K/8)] uint8, chunks without that shape)"""
    values4, meta4 = _c(values4, np.uint8), _c(meta4, np.uint8)
    N = values4.shape[0]
    values8 = np.empty((N, K // 2), np.int8)
    meta8 = np.empty((N, meta_row_bytes(K)), np.uint8)
    bad = ctypes.c_int32(0)
    assert lib().oracle_int4_pairs_to_sparse_int8(_p(values4), _p(meta4), _p(values8), _p(meta8), ctypes.byref(bad), _i64(N),
                                                  _i64(K)) == 0
    return values8, meta8, int(bad.value)


def quantize_rows_int4(X, scale=None):
    """per-row symmetric 4-bit codes (-7..7) in int8 containers, scale = amax / 7"""
    X = _c(X, np.float32)
    rows, cols = X.shape
    Q = np.empty((rows, cols), np.int8)
    given = scale is not None
    s = _c(scale, np.float32).copy() if given else np.empty(rows, np.float32)
    lib().oracle_quantize_rows_int4(_p(X), _p(Q), _p(s), int(given), _i64(rows), _i64(cols))
    return Q, s


def compress_int4_pairs(Wq):
    """Wq [N,K] int8 holding 4-bit codes -> (values [N,K/4] uint8, meta [N,ceil(K/16)] uint8, violations)"""
    Wq = _c(Wq, np.int8)
    N, K = Wq.shape
    values = np.empty((N, K // 4), np.uint8)
    meta = np.empty((N, meta4_row_bytes(K)), np.uint8)
    viol = ctypes.c_int32(0)
    assert lib().oracle_compress_int4_pairs(_p(Wq), _p(values), _p(meta), ctypes.byref(viol), _i64(N), _i64(K)) == 0
    return values, meta, int(viol.value)


def decompress_int4_pairs(values, meta, K):
    values, meta = _c(values, np.uint8), _c(meta, np.uint8)
    N = values.shape[0]
    W = np.empty((N, K), np.int8)
    assert lib().oracle_decompress_int4_pairs(_p(values), _p(meta), _p(W), _i64(N), _i64(K)) == 0
    return W


# ---------------------------------------------------------------- a3 compress / decompress
def compress(W):
    """W [N,K] float16 or int8 -> (values [N,K/2], meta [N,ceil(K/8)] uint8, violations)."""
    W = np.ascontiguousarray(W)
    N, K = W.shape
    if K % 4:
        raise ValueError("K must be a multiple of 4")
    values = np.empty((N, K // 2), W.dtype)
    meta = np.empty((N, meta_row_bytes(K)), np.uint8)
    viol = ctypes.c_int32(0)
    if W.dtype == np.float16:
        r = lib().oracle_compress_f16(_p(W), _p(values), _p(meta), ctypes.byref(viol), _i64(N), _i64(K))
    elif W.dtype == np.int8:
        r = lib().oracle_compress_i8(_p(W), _p(values), _p(meta), ctypes.byref(viol), _i64(N), _i64(K))
    else:
        raise TypeError(W.dtype)
    assert r == 0
    return values, meta, int(viol.value)


def decompress(values, meta, K):
    values = np.ascontiguousarray(values)
    meta = _c(meta, np.uint8)
    N = values.shape[0]
    W = np.empty((N, K), values.dtype)
    if values.dtype == np.float16:
        r = lib().oracle_decompress_f16(_p(values), _p(meta), _p(W), _i64(N), _i64(K))
    elif values.dtype == np.int8:
        r = lib().oracle_decompress_i8(_p(values), _p(meta), _p(W), _i64(N), _i64(K))
    else:
        raise TypeError(values.dtype)
    assert r == 0
    return W


# ---------------------------------------------------------------- a5 GEMM
def gemm_int8_dense(X, W):
    X = _c(X, np.int8); W = _c(W, np.int8)
    M, K = X.shape; N = W.shape[0]
    assert W.shape[1] == K
    acc = np.empty((M, N), np.int32)
    lib().oracle_gemm_int8_dense(_p(X), _p(W), _p(acc), _i64(M), _i64(N), _i64(K))
    return acc


def spgemm_int8(X, values, meta):
    X = _c(X, np.int8); values = _c(values, np.int8); meta = _c(meta, np.uint8)
    M, K = X.shape; N = values.shape[0]
    assert values.shape[1] * 2 == K
    acc = np.empty((M, N), np.int32)
    r = lib().oracle_spgemm_int8(_p(X), _p(values), _p(meta), _p(acc), _i64(M), _i64(N), _i64(K))
    assert r == 0
    return acc


def gemm_fp16_dense(X, W):
    """returns (acc32 sequential-fp32, acc64)"""
    X = _c(X, np.uint16); W = _c(W, np.uint16)
    M, K = X.shape; N = W.shape[0]
    assert W.shape[1] == K
    a32 = np.empty((M, N), np.float32); a64 = np.empty((M, N), np.float64)
    lib().oracle_gemm_fp16_dense(_p(X), _p(W), _p(a32), _p(a64), _i64(M), _i64(N), _i64(K))
    return a32, a64


def spgemm_fp16(X, values, meta):
    X = _c(X, np.uint16); values = _c(values, np.uint16); meta = _c(meta, np.uint8)
    M, K = X.shape; N = values.shape[0]
    assert values.shape[1] * 2 == K
    a32 = np.empty((M, N), np.float32); a64 = np.empty((M, N), np.float64)
    r = lib().oracle_spgemm_fp16(_p(X), _p(values), _p(meta), _p(a32), _p(a64), _i64(M), _i64(N), _i64(K))
    assert r == 0
    return a32, a64


# ---------------------------------------------------------------- a6 epilogue
def epilogue_int8_f64(acc, s_a, s_w, bias=None, gelu=False, out_scale=None):
    """real-arithmetic (fp64) epilogue: returns dict(ref float64, y16 float16, q8 int8 or None)"""
    acc = _c(acc, np.int32); s_w = _c(s_w, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    M, N = acc.shape
    ref = np.empty((M, N), np.float64); y16 = np.empty((M, N), np.uint16)
    q8 = np.empty((M, N), np.int8) if out_scale is not None else None
    lib().oracle_epilogue_int8_f64(_p(acc), ctypes.c_float(s_a), _p(s_w), _p(bias), int(bool(gelu)), _p(ref), _p(y16),
                                   _p(q8), ctypes.c_float(out_scale if out_scale is not None else 1.0), _i64(M), _i64(N))
    return dict(ref=ref, y16=y16.view(np.float16), q8=q8)


def epilogue_int8_f32(acc, s_a, s_w, bias=None, gelu=False, out_scale=None):
    """the same formula in fp32 in a fixed op order: returns dict(v32, y16, q8)"""
    acc = _c(acc, np.int32); s_w = _c(s_w, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    M, N = acc.shape
    v32 = np.empty((M, N), np.float32); y16 = np.empty((M, N), np.uint16)
    q8 = np.empty((M, N), np.int8) if out_scale is not None else None
    lib().oracle_epilogue_int8_f32(_p(acc), ctypes.c_float(s_a), _p(s_w), _p(bias), int(bool(gelu)), _p(v32), _p(y16),
                                   _p(q8), ctypes.c_float(out_scale if out_scale is not None else 1.0), _i64(M), _i64(N))
    return dict(v32=v32, y16=y16.view(np.float16), q8=q8)


def epilogue_fp16_f64(acc64, bias=None, gelu=False):
    acc64 = _c(acc64, np.float64)
    bias = None if bias is None else _c(bias, np.float32)
    M, N = acc64.shape
    ref = np.empty((M, N), np.float64); y16 = np.empty((M, N), np.uint16)
    lib().oracle_epilogue_fp16_f64(_p(acc64), _p(bias), int(bool(gelu)), _p(ref), _p(y16), _i64(M), _i64(N))
    return dict(ref=ref, y16=y16.view(np.float16))


def linear_int8_sparse(X, values, meta, s_a, s_w, bias=None, gelu=False):
    """whole sparse-form INT8 linear layer in one call (used to time the oracle)."""
    X = _c(X, np.int8); values = _c(values, np.int8); meta = _c(meta, np.uint8); s_w = _c(s_w, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    M, K = X.shape; N = values.shape[0]
    y16 = np.empty((M, N), np.uint16)
    r = lib().oracle_linear_int8_sparse(_p(X), _p(values), _p(meta), ctypes.c_float(s_a), _p(s_w), _p(bias),
                                        int(bool(gelu)), _p(y16), _i64(M), _i64(N), _i64(K))
    assert r == 0
    return y16.view(np.float16)


# ---------------------------------------------------------------- patch embedding (strided convolution, Sec. 3.3)
def patch_conv_int8(img, Wc):
    """img int8 [B,C,H,W], Wc int8 [D,C,P,P] -> (acc int32 [B*(H/P)*(W/P), D], multiply-accumulates performed)"""
    img = _c(img, np.int8); Wc = _c(Wc, np.int8)
    B, C, H, W = img.shape; D, C2, P, P2 = Wc.shape
    assert C2 == C and P2 == P
    acc = np.empty((B * (H // P) * (W // P), D), np.int32)
    f = lib().oracle_patch_conv_int8
    f.restype = ctypes.c_int64
    macs = f(_p(img), _p(Wc), _p(acc), _i64(B), _i64(C), _i64(H), _i64(W), _i64(P), _i64(D))
    assert macs >= 0
    return acc, int(macs)


def patch_conv_f16(img, Wc):
    """img fp16 [B,C,H,W], Wc fp16 [D,C,P,P] -> (acc float64 [B*(H/P)*(W/P), D], multiply-accumulates performed)"""
    img = _c(img, np.uint16); Wc = _c(Wc, np.uint16)
    B, C, H, W = img.shape; D, C2, P, P2 = Wc.shape
    assert C2 == C and P2 == P
    acc = np.empty((B * (H // P) * (W // P), D), np.float64)
    f = lib().oracle_patch_conv_f16
    f.restype = ctypes.c_int64
    macs = f(_p(img), _p(Wc), _p(acc), _i64(B), _i64(C), _i64(H), _i64(W), _i64(P), _i64(D))
    assert macs >= 0
    return acc, int(macs)
