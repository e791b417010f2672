"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares, and rejects bad
arguments before touching the GPU.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "gpusq.h")
LIB = os.path.join(ROOT, "paper_2305_10727_amd", "libgpusq.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2305_10727_amd import build
        build.build()
    return ctypes.CDLL(LIB)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gpusq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    from paper_2305_10727_amd import gpusq
    assert sorted(gpusq.EXPORTS) == names


def test_status_strings_and_version(lib):
    lib.gpusq_status_string.restype = ctypes.c_char_p
    seen = {lib.gpusq_status_string(i) for i in range(7)}
    assert len(seen) == 7 and lib.gpusq_status_string(0) == b"ok" and lib.gpusq_status_string(7) == b"unknown status"
    assert lib.gpusq_version() >= 100


def test_argument_errors_are_caught_on_the_host(lib):
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    OK, ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_UNSUPPORTED = 0, 1, 2, 3, 4
    good = vp(0x10000)  # never dereferenced: every call below fails validation first
    odd = vp(0x10008)
    lib.gpusq_prune_2to4.argtypes = [vp, vp, vp, ci, i64, i64, vp]
    assert lib.gpusq_prune_2to4(None, good, None, 0, 4, 8, None) == ERR_NULL
    assert lib.gpusq_prune_2to4(good, good, None, 0, 4, 6, None) == ERR_SHAPE
    assert lib.gpusq_prune_2to4(good, good, None, 0, 0, 8, None) == ERR_SHAPE
    assert lib.gpusq_prune_2to4(good, good, None, 2, 4, 8, None) == ERR_UNSUPPORTED
    assert lib.gpusq_prune_2to4(odd, good, None, 0, 4, 8, None) == ERR_ALIGN
    lib.gpusq_compress.argtypes = [vp, vp, vp, vp, ci, i64, i64, vp]
    assert lib.gpusq_compress(good, good, None, None, 1, 4, 8, None) == ERR_NULL
    assert lib.gpusq_compress(good, good, good, None, 0, 4, 8, None) == ERR_UNSUPPORTED
    assert lib.gpusq_compress(good, good, good, None, 1, 4, 10, None) == ERR_SHAPE
    lib.gpusq_check_2to4.argtypes = [vp, ci, vp, i64, i64, vp]
    assert lib.gpusq_check_2to4(good, 0, None, 4, 8, None) == ERR_NULL          # the counter is required
    assert lib.gpusq_check_2to4(good, 3, good, 4, 8, None) == ERR_UNSUPPORTED   # int32 tensors
    assert lib.gpusq_check_2to4(good, 0, good, 4, 6, None) == ERR_SHAPE
    assert lib.gpusq_check_2to4(odd, 0, good, 4, 8, None) == ERR_ALIGN
    assert lib.gpusq_check_2to4(good, 0, vp(0x10002), 4, 8, None) == ERR_ALIGN
    lib.gpusq_quantize_int8.argtypes = [vp, ci, vp, vp, ci, ci, i64, i64, vp, vp]
    assert lib.gpusq_quantize_int8(good, 0, good, None, 0, 0, 4, 8, None, None) == ERR_NULL
    assert lib.gpusq_quantize_int8(good, 0, good, good, 1, 0, 4, 8, None, None) == ERR_NULL  # per-tensor needs workspace
    assert lib.gpusq_quantize_int8(good, 0, good, good, 7, 0, 4, 8, good, None) == ERR_UNSUPPORTED
    assert lib.gpusq_quantize_int8(good, 0, good, good, 0, 0, -1, 8, good, None) == ERR_SHAPE
    lib.gpusq_spgemm_int8.argtypes = [vp, vp, vp, vp, vp, vp, ci, vp, i64, i64, i64, ci, vp]
    assert lib.gpusq_spgemm_int8(good, good, None, None, None, good, 3, None, 8, 8, 24, 0, None) == ERR_UNSUPPORTED  # K % 16
    assert lib.gpusq_spgemm_int8(good, good, None, None, None, good, 3, None, 8, 6, 32, 0, None) == ERR_UNSUPPORTED  # N % 4
    assert lib.gpusq_spgemm_int8(good, good, None, None, None, good, 3, None, 8, 8, 30, 0, None) == ERR_SHAPE
    assert lib.gpusq_spgemm_int8(good, good, None, None, None, good, 1, None, 8, 8, 32, 0, None) == ERR_NULL  # scales
    assert lib.gpusq_spgemm_int8(good, good, good, good, None, good, 1, None, 8, 8, 32, 1, None) == ERR_NULL  # bias flag
    assert lib.gpusq_spgemm_int8(good, good, good, good, None, good, 2, None, 8, 8, 32, 0, None) == ERR_NULL  # out_scale
    assert lib.gpusq_spgemm_int8(good, good, good, good, None, good, 1, None, 8, 8, 32, 8, None) == ERR_UNSUPPORTED
    # fp16 activations quantised inside the GEMM: the same checks, and problems of the tile kernel are refused
    lib.gpusq_spgemm_int8_xf16.argtypes = [vp, vp, vp, vp, vp, vp, ci, vp, i64, i64, i64, ci, vp]
    assert lib.gpusq_spgemm_int8_xf16(good, good, None, None, None, good, 1, None, 8, 8, 32, 0, None) == ERR_NULL  # scales
    assert lib.gpusq_spgemm_int8_xf16(good, good, good, good, None, good, 2, None, 8, 8, 32, 0, None) == ERR_NULL  # out_scale
    assert lib.gpusq_spgemm_int8_xf16(good, good, good, good, None, odd, 1, None, 8, 8, 32, 0, None) == ERR_ALIGN
    assert lib.gpusq_spgemm_int8_xf16(good, good, good, good, None, good, 1, None, 12608, 3072, 768, 0, None) == ERR_UNSUPPORTED
    lib.gpusq_spgemm_fp16.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp]
    assert lib.gpusq_spgemm_fp16(good, None, None, good, 8, 8, 32, 0, None) == ERR_NULL
    assert lib.gpusq_spgemm_fp16(good, good, None, odd, 8, 8, 32, 0, None) == ERR_ALIGN
    assert lib.gpusq_spgemm_fp16(good, good, None, good, 0, 8, 32, 0, None) == ERR_SHAPE
    lib.gpusq_im2col_patches.argtypes = [vp, vp, ci, i64, i64, i64, i64, i64, i64, vp]
    assert lib.gpusq_im2col_patches(good, None, 2, 1, 3, 32, 32, 16, 768, None) == ERR_NULL
    assert lib.gpusq_im2col_patches(good, good, 2, 1, 3, 30, 32, 16, 768, None) == ERR_SHAPE   # H % P
    assert lib.gpusq_im2col_patches(good, good, 2, 1, 3, 32, 32, 16, 700, None) == ERR_SHAPE   # K_pad < C*P*P
    assert lib.gpusq_im2col_patches(good, good, 0, 1, 3, 32, 32, 16, 768, None) == ERR_UNSUPPORTED
    assert lib.gpusq_im2col_patches(odd, good, 2, 1, 3, 32, 32, 16, 768, None) == ERR_ALIGN
    lib.gpusq_patch_embed16_int8.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, ci, vp]
    assert lib.gpusq_patch_embed16_int8(good, good, None, good, None, good, 4, 3, 224, 224, 768, 0, None) == ERR_NULL
    assert lib.gpusq_patch_embed16_int8(good, good, good, good, None, good, 4, 3, 220, 224, 768, 0, None) == ERR_SHAPE
    assert lib.gpusq_patch_embed16_int8(good, good, good, good, None, good, 4, 3, 224, 224, 768, 2, None) == ERR_UNSUPPORTED  # GELU
    assert lib.gpusq_patch_embed16_int8(good, good, good, good, None, good, 1, 3, 32, 32, 64, 0, None) == ERR_UNSUPPORTED   # too small
    lib.gpusq_patch_embed16_fp16.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, ci, vp]
    assert lib.gpusq_patch_embed16_fp16(good, good, None, good, 4, 3, 224, 224, 768, 1, None) == ERR_NULL                  # bias flag
    lib.gpusq_prune_n_of_m.argtypes = [vp, vp, ci, ci, i64, i64, vp]
    assert lib.gpusq_prune_n_of_m(good, None, 1, 4, 4, 16, None) == ERR_NULL
    assert lib.gpusq_prune_n_of_m(good, good, 1, 5, 4, 20, None) == ERR_UNSUPPORTED   # m
    assert lib.gpusq_prune_n_of_m(good, good, 4, 4, 4, 16, None) == ERR_SHAPE         # n < m
    assert lib.gpusq_prune_n_of_m(good, good, 2, 16, 4, 24, None) == ERR_SHAPE        # K % m
    lib.gpusq_prune_4to8_pairs.argtypes = [vp, vp, vp, ci, i64, i64, vp]
    assert lib.gpusq_prune_4to8_pairs(good, None, None, 0, 4, 8, None) == ERR_NULL
    assert lib.gpusq_prune_4to8_pairs(good, good, None, 1, 4, 12, None) == ERR_SHAPE   # K % 8
    assert lib.gpusq_prune_4to8_pairs(odd, good, None, 0, 4, 8, None) == ERR_ALIGN
    lib.gpusq_int4_to_sparse_int8.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp]
    assert lib.gpusq_int4_to_sparse_int8(good, good, good, None, None, 4, 8, None) == ERR_NULL
    assert lib.gpusq_int4_to_sparse_int8(good, good, good, good, None, 4, 12, None) == ERR_SHAPE
    assert lib.gpusq_int4_to_sparse_int8(good, good, odd, good, None, 4, 8, None) == ERR_ALIGN
    lib.gpusq_quantize_rows_int4.argtypes = [vp, ci, vp, vp, ci, i64, i64, vp]
    assert lib.gpusq_quantize_rows_int4(good, 0, good, None, 0, 4, 8, None) == ERR_NULL
    assert lib.gpusq_quantize_rows_int4(good, 2, good, good, 0, 4, 8, None) == ERR_UNSUPPORTED
    assert lib.gpusq_quantize_rows_int4(good, 0, good, good, 0, 0, 8, None) == ERR_SHAPE
    lib.gpusq_compress_int4.argtypes = [vp, vp, vp, vp, i64, i64, vp]
    assert lib.gpusq_compress_int4(good, good, None, None, 4, 8, None) == ERR_NULL
    assert lib.gpusq_compress_int4(good, good, good, None, 4, 20, None) == ERR_SHAPE
    lib.gpusq_decompress_int4.argtypes = [vp, vp, vp, i64, i64, vp]
    assert lib.gpusq_decompress_int4(good, good, None, 4, 8, None) == ERR_NULL
    assert lib.gpusq_decompress_int4(good, odd, good, 4, 8, None) == ERR_ALIGN
    lib.gpusq_packed_bytes.restype = ctypes.c_size_t
    lib.gpusq_packed_bytes.argtypes = [ci, i64, i64]
    # tiles of 256 channels x one 128-byte K step: 16 fragments of 1024 value bytes + 16 x 64 lanes of index bytes
    assert lib.gpusq_packed_bytes(2, 768, 192) == 3 * 2 * (16384 + 4096)
    assert lib.gpusq_packed_bytes(1, 768, 192) == 3 * 3 * (16384 + 2048)
    assert lib.gpusq_packed_bytes(2, 100, 144) == 1 * 2 * (16384 + 4096)
    assert lib.gpusq_packed_bytes(0, 768, 192) == 0 and lib.gpusq_packed_bytes(2, 768, 190) == 0
    lib.gpusq_quantize_workspace_bytes.restype = ctypes.c_size_t
    lib.gpusq_quantize_workspace_bytes.argtypes = [ci, i64, i64]
    assert lib.gpusq_quantize_workspace_bytes(0, 10, 10) == 0 and lib.gpusq_quantize_workspace_bytes(1, 10, 10) >= 4


def test_binding_refuses_host_tensors():
    torch = pytest.importorskip("torch")
    from paper_2305_10727_amd import gpusq
    with pytest.raises(ValueError):
        gpusq.prune_2to4(torch.zeros(4, 8))


def _plan(lib, dt, M, N, K, epi, cus):
    out = (ctypes.c_int32 * 8)()
    lib.gpusq_spgemm_plan.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                      ctypes.POINTER(ctypes.c_int32)]
    st = lib.gpusq_spgemm_plan(dt, M, N, K, epi, cus, out)
    return st, list(out)


def test_tile_plan_covers_every_row_exactly_once(lib):
    """The host-side tile plan of the sparse GEMM: the full tiles and the tail tiles partition the rows of X, the tile
    count is consistent, no more workgroups than tiles or compute units (rounded to the 8 XCDs), and a small or ragged-K
    problem takes the small kernel."""
    I8, F16 = 2, 1
    shapes = [(12608, 3072, 768), (25216, 768, 3072), (12544, 512, 2048), (65792, 5120, 1280), (50432, 1024, 4096),
              (600, 512, 384), (1500, 388, 256), (2100, 520, 128), (12345, 264, 128), (70000, 256, 128), (257, 1024, 1024),
              (3, 100000, 256), (999999, 4, 128)]
    for cus in (256, 64, 304, 8):
        for dt in (I8, F16):
            for epi in (0, 3):
                for M, N, K in shapes:
                    st, p = _plan(lib, dt, M, N, K, epi, cus)
                    assert st == 0, (M, N, K)
                    kernel, u, tiles_n, ftm, fchunks, ttm, total, wgs = p
                    if M * N <= 256 * 1024:
                        assert kernel == 0
                        continue
                    assert kernel in (0, 2, 3)
                    if kernel == 0:  # few rows: the estimated run times favour the small kernel
                        assert p[1:] == [0] * 7 and -(-M // 64) * -(-N // 64) <= 16 * cus
                        continue
                    # kernel 2: one workgroup per CU, tiles of up to 256 rows; kernel 3: two per CU, up to 128 rows
                    max_tm, per_cu = (4, 1) if kernel == 2 else (2, 2)
                    assert u == 64 and tiles_n == -(-N // 256)
                    assert 1 <= ftm <= max_tm and 1 <= ttm <= max_tm and fchunks >= 0
                    full_rows = fchunks * u * ftm
                    assert full_rows - u * ftm < M          # no full tile lies entirely beyond M
                    rows_left = max(M - full_rows, 0)
                    tail_chunks = -(-rows_left // (u * ttm))
                    assert total == (fchunks + tail_chunks) * tiles_n
                    assert full_rows + tail_chunks * u * ttm >= M                # every row is covered
                    assert tail_chunks == 0 or full_rows + (tail_chunks - 1) * u * ttm < M  # and no tail tile is empty
                    assert wgs % 8 == 0 and wgs <= -(-per_cu * cus // 8) * 8 and wgs >= min(total, 8) and wgs - 8 < total
    # one image (M = 197) takes the small kernel, a batch of 64 the tile kernel
    for N, K in ((2304, 768), (3072, 768), (768, 3072), (768, 768)):
        assert _plan(lib, I8, 197, N, K, 0, 256)[1][0] == 0 and _plan(lib, I8, 12608, N, K, 0, 256)[1][0] in (2, 3)
        assert _plan(lib, F16, 197, N, K, 0, 256)[1][0] == 0 and _plan(lib, F16, 12608, N, K, 0, 256)[1][0] in (2, 3)
    # between the two tile kernels: wide, GELU and long-K layers stay on the one-workgroup kernel, layers with few output
    # channels, short K and no GELU take the kernel with two workgroups per CU
    assert _plan(lib, I8, 12608, 3072, 768, 3, 256)[1][0] == 2 and _plan(lib, I8, 25216, 768, 3072, 1, 256)[1][0] == 2
    assert _plan(lib, F16, 12608, 3072, 768, 3, 256)[1][0] == 2 and _plan(lib, F16, 50432, 1024, 4096, 1, 256)[1][0] == 2
    assert _plan(lib, I8, 25216, 768, 768, 1, 256)[1][0] == 3 and _plan(lib, F16, 12544, 1536, 512, 1, 256)[1][0] == 3
    assert _plan(lib, F16, 25216, 768, 768, 1, 256)[1][0] == 2  # FP16: only from 1024 output channels on
    # ragged K (not a multiple of the 128-byte K step) -> zero-filling small kernel; argument errors are reported
    assert _plan(lib, I8, 4096, 4096, 144, 0, 256) == (0, [1, 0, 0, 0, 0, 0, 0, 0])
    assert _plan(lib, F16, 4096, 4096, 64, 0, 256)[1][0] == 2 and _plan(lib, F16, 4096, 4096, 80, 0, 256)[1][0] == 1
    assert _plan(lib, I8, 0, 4096, 128, 0, 256)[0] == 2 and _plan(lib, I8, 128, 4096, 130, 0, 256)[0] == 2
    assert _plan(lib, 0, 128, 4096, 128, 0, 256)[0] == 4 and _plan(lib, I8, 128, 4098, 128, 0, 256)[0] == 4


def test_force_kernel_override_is_an_explicit_call(lib):
    """the testing override: set and cleared through the ABI (no environment lookup per launch), visible in the plan query"""
    lib.gpusq_force_kernel.argtypes = [ctypes.c_int]
    I8 = 2
    prev = lib.gpusq_force_kernel(-1)
    try:
        assert _plan(lib, I8, 12608, 3072, 768, 0, 256)[1][0] == 2
        assert lib.gpusq_force_kernel(0) == -1
        assert _plan(lib, I8, 12608, 3072, 768, 0, 256)[1][0] == 0
        assert lib.gpusq_force_kernel(2) == 0
        assert _plan(lib, I8, 197, 768, 768, 0, 256)[1][0] == 2
        assert _plan(lib, I8, 197, 768, 144, 0, 256)[1][0] != 2   # ragged K cannot run on the tile kernel: the rules decide
        assert lib.gpusq_force_kernel(3) == 2
        assert _plan(lib, I8, 12608, 3072, 768, 0, 256)[1][0] == 3
        assert lib.gpusq_force_kernel(7) == 3                      # anything else clears the override
        assert lib.gpusq_force_kernel(-1) == -1
    finally:
        lib.gpusq_force_kernel(prev)


def test_gelu_fit_stays_within_its_stated_bound_of_the_exact_function():
    """The epilogue's GELU (a polynomial fit in fp32, csrc/epilogue.h) against the oracle's erf form in fp64, over every
    finite fp16 argument and a dense fp32 grid: the difference stays below the stated 0.15 units in the last place of the
    exact value as an fp16 number.  The GPU tests build their element-wise code check on this bound."""
    np = pytest.importorskip("numpy")
    import oracle
    import gelu_fit
    h = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float32)
    x = np.concatenate([np.linspace(-14.0, 14.0, 2000001).astype(np.float32), h, -h])
    exact = oracle.epilogue_fp16_f64(x.astype(np.float64).reshape(1, -1), None, True)["ref"][0]
    err = np.abs(gelu_fit.gelu_fit_f32(x).astype(np.float64) - exact) / gelu_fit.ulp16(exact)
    assert 0.05 < err.max() <= gelu_fit.FIT_BOUND_ULP16
    # so a rounded fp16 output is within one unit of the exact value's rounding, and a re-quantised code moves only at a tie
    assert np.isfinite(gelu_fit.gelu_fit_f32(np.array([-65504.0, 65504.0, 0.0, -0.0], np.float32))).all()
