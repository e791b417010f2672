// C ABI of libgpusq: argument validation, status codes, dispatch to the kernels.  No computation happens here.
#include <atomic>

#include "common.h"

namespace gpusq {
static std::atomic<int> g_last_hip_error{0};
void set_last_hip_error(hipError_t e) { g_last_hip_error.store((int)e); }
}  // namespace gpusq

using namespace gpusq;

namespace {
constexpr int64_t kMaxElems = (int64_t)1 << 40;

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

gpusq_status check_nk(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0 || K % 4 != 0) return GPUSQ_ERR_SHAPE;
  if (N > INT32_MAX || K > INT32_MAX || N * K > kMaxElems) return GPUSQ_ERR_SHAPE;
  return GPUSQ_OK;
}

gpusq_status check_gemm(const void* X, const void* W, const float* bias, const void* Y, int64_t M, int64_t N, int64_t K,
                        int epilogue) {
  if (!X || !W || !Y) return GPUSQ_ERR_NULL;
  if ((epilogue & GPUSQ_EPI_BIAS) && !bias) return GPUSQ_ERR_NULL;
  if (M <= 0) return GPUSQ_ERR_SHAPE;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (M > INT32_MAX || M * N > kMaxElems || M * K > kMaxElems) return GPUSQ_ERR_SHAPE;
  if (!aligned16(X) || !aligned16(W) || !aligned16(Y) || (bias && !aligned16(bias))) return GPUSQ_ERR_ALIGN;
  if (epilogue & ~(GPUSQ_EPI_BIAS | GPUSQ_EPI_GELU)) return GPUSQ_ERR_UNSUPPORTED;
  if (K % 16 != 0 || N % 4 != 0) return GPUSQ_ERR_UNSUPPORTED;
  return GPUSQ_OK;
}

gpusq_status check_int8_extras(const float* act_scale, const float* w_scale, gpusq_dtype out_dt, const float* out_scale) {
  if (out_dt != GPUSQ_F16 && out_dt != GPUSQ_I32 && out_dt != GPUSQ_I8) return GPUSQ_ERR_UNSUPPORTED;
  if (out_dt != GPUSQ_I32 && (!act_scale || !w_scale)) return GPUSQ_ERR_NULL;
  if (out_dt == GPUSQ_I8 && !out_scale) return GPUSQ_ERR_NULL;
  if (w_scale && !aligned16(w_scale)) return GPUSQ_ERR_ALIGN;
  return GPUSQ_OK;
}
}  // namespace

extern "C" {

const char* gpusq_status_string(gpusq_status s) {
  switch (s) {
    case GPUSQ_OK: return "ok";
    case GPUSQ_ERR_NULL: return "a required pointer is NULL";
    case GPUSQ_ERR_SHAPE: return "invalid shape (sizes must be positive, K a multiple of 4)";
    case GPUSQ_ERR_ALIGN: return "pointer not 16-byte aligned";
    case GPUSQ_ERR_UNSUPPORTED: return "valid request that this build does not implement";
    case GPUSQ_ERR_HIP: return "HIP runtime or launch failure (see gpusq_last_hip_error)";
    case GPUSQ_ERR_NOT_2TO4: return "the tensor has a group of 4 with more than two non-zero elements";
  }
  return "unknown status";
}

int gpusq_last_hip_error(void) { return g_last_hip_error.load(); }

int gpusq_version(void) { return 100; }

gpusq_status gpusq_prune_2to4(const void* W_in, void* W_out, uint8_t* mask_out, gpusq_dtype dt, int64_t N, int64_t K,
                              void* stream) {
  if (!W_in || !W_out) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (dt != GPUSQ_F32 && dt != GPUSQ_F16) return GPUSQ_ERR_UNSUPPORTED;
  if (!aligned16(W_in) || !aligned16(W_out)) return GPUSQ_ERR_ALIGN;
  return launch_prune(W_in, W_out, mask_out, dt, N, K, (hipStream_t)stream);
}

gpusq_status gpusq_cast_f16(const float* in, void* out, int64_t n, void* stream) {
  if (!in || !out) return GPUSQ_ERR_NULL;
  if (n <= 0 || n > kMaxElems) return GPUSQ_ERR_SHAPE;
  if (!aligned16(in) || !aligned16(out)) return GPUSQ_ERR_ALIGN;
  return launch_cast_f16(in, out, n, (hipStream_t)stream);
}

size_t gpusq_quantize_workspace_bytes(int mode, int64_t rows, int64_t cols) {
  (void)rows;
  (void)cols;
  return mode == GPUSQ_PER_TENSOR ? 4096 : 0;  // per-workgroup partial maxima of the first pass
}

gpusq_status gpusq_quantize_int8(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int mode, int scale_is_input,
                                 int64_t rows, int64_t cols, void* workspace, void* stream) {
  if (!X || !Xq || !scale) return GPUSQ_ERR_NULL;
  if (rows <= 0 || cols <= 0 || rows > INT32_MAX || cols > INT32_MAX || rows * cols > kMaxElems) return GPUSQ_ERR_SHAPE;
  if (dt != GPUSQ_F32 && dt != GPUSQ_F16) return GPUSQ_ERR_UNSUPPORTED;
  if (mode != GPUSQ_PER_ROW && mode != GPUSQ_PER_TENSOR) return GPUSQ_ERR_UNSUPPORTED;
  if (mode == GPUSQ_PER_TENSOR && !scale_is_input && !workspace) return GPUSQ_ERR_NULL;
  if (!aligned16(X) || !aligned16(Xq) || (workspace && !aligned16(workspace))) return GPUSQ_ERR_ALIGN;
  return launch_quantize(X, dt, Xq, scale, mode, scale_is_input, rows, cols, workspace, (hipStream_t)stream);
}

gpusq_status gpusq_quantize_tensor_int8_noalloc(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int scale_is_input,
                                                int64_t rows, int64_t cols, void* stream) {
  if (!X || !Xq || !scale) return GPUSQ_ERR_NULL;
  // the same size limits as gpusq_quantize_int8: the library's own scratch (4 KB of partial maxima) serves any of them
  if (rows <= 0 || cols <= 0 || rows > INT32_MAX || cols > INT32_MAX || rows * cols > kMaxElems) return GPUSQ_ERR_SHAPE;
  if (dt != GPUSQ_F32 && dt != GPUSQ_F16) return GPUSQ_ERR_UNSUPPORTED;
  if (!aligned16(X) || !aligned16(Xq)) return GPUSQ_ERR_ALIGN;
  return launch_quantize_tensor_static(X, dt, Xq, scale, scale_is_input, rows, cols, (hipStream_t)stream);
}

gpusq_status gpusq_compress(const void* W, void* values, uint8_t* meta, int32_t* violations, gpusq_dtype dt, int64_t N,
                            int64_t K, void* stream) {
  if (!W || !values || !meta) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (dt != GPUSQ_F16 && dt != GPUSQ_I8) return GPUSQ_ERR_UNSUPPORTED;
  if (!aligned16(W) || !aligned16(values) || !aligned16(meta)) return GPUSQ_ERR_ALIGN;
  return launch_compress(W, values, meta, violations, dt, N, K, (hipStream_t)stream);
}

gpusq_status gpusq_check_2to4(const void* W, gpusq_dtype dt, int32_t* violations, int64_t N, int64_t K, void* stream) {
  if (!W || !violations) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (N * K / 4 > INT32_MAX) return GPUSQ_ERR_SHAPE;  // the count is an int32
  if (dt != GPUSQ_F32 && dt != GPUSQ_F16 && dt != GPUSQ_I8) return GPUSQ_ERR_UNSUPPORTED;
  if (!aligned16(W) || ((uintptr_t)violations & 3u) != 0) return GPUSQ_ERR_ALIGN;
  st = launch_count_violations(W, dt, violations, N, K, (hipStream_t)stream);
  if (st != GPUSQ_OK) return st;
  int32_t count = 0;
  hipError_t e = hipMemcpyAsync(&count, violations, sizeof count, hipMemcpyDeviceToHost, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) {
    set_last_hip_error(e);
    return GPUSQ_ERR_HIP;
  }
  return count == 0 ? GPUSQ_OK : GPUSQ_ERR_NOT_2TO4;
}

gpusq_status gpusq_decompress(const void* values, const uint8_t* meta, void* W, gpusq_dtype dt, int64_t N, int64_t K,
                              void* stream) {
  if (!W || !values || !meta) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (dt != GPUSQ_F16 && dt != GPUSQ_I8) return GPUSQ_ERR_UNSUPPORTED;
  if (!aligned16(W) || !aligned16(values) || !aligned16(meta)) return GPUSQ_ERR_ALIGN;
  return launch_decompress(values, meta, W, dt, N, K, (hipStream_t)stream);
}

gpusq_status gpusq_prune_n_of_m(const float* W_in, float* W_out, int n, int m, int64_t N, int64_t K, void* stream) {
  if (!W_in || !W_out) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (m != 4 && m != 8 && m != 16) return GPUSQ_ERR_UNSUPPORTED;
  if (n < 1 || n >= m || K % m != 0) return GPUSQ_ERR_SHAPE;
  if (!aligned16(W_in) || !aligned16(W_out)) return GPUSQ_ERR_ALIGN;
  return launch_prune_n_of_m(W_in, W_out, n, m, N, K, (hipStream_t)stream);
}

gpusq_status gpusq_prune_4to8_pairs(const float* W_in, float* W_out, uint8_t* mask_out, int one_per_group, int64_t N, int64_t K,
                                    void* stream) {
  if (!W_in || !W_out) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (K % 8 != 0) return GPUSQ_ERR_SHAPE;
  if (!aligned16(W_in) || !aligned16(W_out)) return GPUSQ_ERR_ALIGN;
  return launch_prune_pairs(W_in, W_out, mask_out, one_per_group != 0, N, K, (hipStream_t)stream);
}

gpusq_status gpusq_quantize_rows_int4(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int scale_is_input, int64_t rows,
                                      int64_t cols, void* stream) {
  if (!X || !Xq || !scale) return GPUSQ_ERR_NULL;
  if (rows <= 0 || cols <= 0 || rows > INT32_MAX || cols > INT32_MAX || rows * cols > kMaxElems) return GPUSQ_ERR_SHAPE;
  if (dt != GPUSQ_F32 && dt != GPUSQ_F16) return GPUSQ_ERR_UNSUPPORTED;
  if (!aligned16(X) || !aligned16(Xq)) return GPUSQ_ERR_ALIGN;
  return launch_quantize_rows_int4(X, dt, Xq, scale, scale_is_input, rows, cols, (hipStream_t)stream);
}

gpusq_status gpusq_compress_int4(const int8_t* W, uint8_t* values, uint8_t* meta, int32_t* violations, int64_t N, int64_t K,
                                 void* stream) {
  if (!W || !values || !meta) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (K % 8 != 0) return GPUSQ_ERR_SHAPE;
  if (!aligned16(W) || !aligned16(values) || !aligned16(meta)) return GPUSQ_ERR_ALIGN;
  return launch_compress_int4(W, values, meta, violations, N, K, (hipStream_t)stream);
}

gpusq_status gpusq_int4_to_sparse_int8(const uint8_t* values4, const uint8_t* meta4, int8_t* values8, uint8_t* meta8,
                                       int32_t* mismatches, int64_t N, int64_t K, void* stream) {
  if (!values4 || !meta4 || !values8 || !meta8) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (K % 8 != 0) return GPUSQ_ERR_SHAPE;
  if (!aligned16(values4) || !aligned16(meta4) || !aligned16(values8) || !aligned16(meta8)) return GPUSQ_ERR_ALIGN;
  return launch_int4_to_sparse_int8(values4, meta4, values8, meta8, mismatches, N, K, (hipStream_t)stream);
}

gpusq_status gpusq_decompress_int4(const uint8_t* values, const uint8_t* meta, int8_t* W, int64_t N, int64_t K, void* stream) {
  if (!W || !values || !meta) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (K % 8 != 0) return GPUSQ_ERR_SHAPE;
  if (!aligned16(W) || !aligned16(values) || !aligned16(meta)) return GPUSQ_ERR_ALIGN;
  return launch_decompress_int4(values, meta, W, N, K, (hipStream_t)stream);
}

size_t gpusq_packed_bytes(gpusq_dtype dt, int64_t N, int64_t K) {
  if (check_nk(N, K) != GPUSQ_OK || (dt != GPUSQ_F16 && dt != GPUSQ_I8)) return 0;
  const bool is_i8 = dt == GPUSQ_I8;
  const int64_t ksteps = ceil_div(K, step_elems(is_i8));
  return (size_t)(ceil_div(N, kTileRows) * ksteps * tile_bytes(is_i8));
}

gpusq_status gpusq_pack(const void* values, const uint8_t* meta, void* packed, gpusq_dtype dt, int64_t N, int64_t K,
                        void* stream) {
  if (!values || !meta || !packed) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (dt != GPUSQ_F16 && dt != GPUSQ_I8) return GPUSQ_ERR_UNSUPPORTED;
  if (!aligned16(values) || !aligned16(meta) || !aligned16(packed)) return GPUSQ_ERR_ALIGN;
  return launch_pack(values, meta, packed, dt, N, K, (hipStream_t)stream);
}

gpusq_status gpusq_prepare_weights(const float* W, gpusq_dtype dt, float* W_pruned, void* W_low, float* w_scale, void* values,
                                   uint8_t* meta, void* packed, int64_t N, int64_t K, void* stream) {
  if (!W || !packed) return GPUSQ_ERR_NULL;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (dt != GPUSQ_F16 && dt != GPUSQ_I8) return GPUSQ_ERR_UNSUPPORTED;
  if (dt == GPUSQ_I8 && !w_scale) return GPUSQ_ERR_NULL;
  if (K * (int64_t)sizeof(float) > 64 * 1024) return GPUSQ_ERR_UNSUPPORTED;  // one fp32 row is staged in LDS
  if (!aligned16(W) || !aligned16(packed) || (W_pruned && !aligned16(W_pruned)) || (W_low && !aligned16(W_low)) ||
      (values && !aligned16(values)) || (meta && !aligned16(meta)))
    return GPUSQ_ERR_ALIGN;
  return launch_prepare_weights(W, dt, W_pruned, W_low, w_scale, values, meta, packed, N, K, (hipStream_t)stream);
}

gpusq_status gpusq_im2col_patches(const void* img, void* X, gpusq_dtype dt, int64_t B, int64_t C, int64_t H, int64_t W,
                                  int64_t P, int64_t K_pad, void* stream) {
  if (!img || !X) return GPUSQ_ERR_NULL;
  if (B <= 0 || C <= 0 || H <= 0 || W <= 0 || P <= 0 || H % P != 0 || W % P != 0) return GPUSQ_ERR_SHAPE;
  if (C > 65536 || P > 4096 || H > (1 << 20) || W > (1 << 20)) return GPUSQ_ERR_SHAPE;
  if (C * P * P > INT32_MAX || K_pad < C * P * P || K_pad > INT32_MAX) return GPUSQ_ERR_SHAPE;
  if (B * C * H * W > kMaxElems || B * (H / P) * (W / P) * K_pad > kMaxElems) return GPUSQ_ERR_SHAPE;
  if (dt != GPUSQ_F16 && dt != GPUSQ_I8) return GPUSQ_ERR_UNSUPPORTED;
  if (!aligned16(img) || !aligned16(X)) return GPUSQ_ERR_ALIGN;
  return launch_im2col_patches(img, X, dt, B, C, H, W, P, K_pad, (hipStream_t)stream);
}

static gpusq_status patch_embed16(bool is_i8, const void* img, const void* Wpacked, const float* act_scale, const float* w_scale,
                                  const float* bias, void* Y, int64_t B, int64_t C, int64_t H, int64_t W, int64_t D, int epilogue,
                                  void* stream) {
  if (is_i8 && (!act_scale || !w_scale)) return GPUSQ_ERR_NULL;
  if (B <= 0 || C <= 0 || H <= 0 || W <= 0 || H % 16 != 0 || W % 16 != 0) return GPUSQ_ERR_SHAPE;
  if (C > 65536 || H > (1 << 20) || W > (1 << 20)) return GPUSQ_ERR_SHAPE;
  const int64_t M = B * (H / 16) * (W / 16), K = C * 256;
  gpusq_status st = check_gemm(img, Wpacked, bias, Y, M, D, K, epilogue);
  if (st != GPUSQ_OK) return st;
  if (B * C * H * W * (is_i8 ? 1 : 2) >= ((int64_t)1 << 32)) return GPUSQ_ERR_SHAPE;  // 32-bit per-lane byte offsets
  if (epilogue & GPUSQ_EPI_GELU) return GPUSQ_ERR_UNSUPPORTED;
  GemmArgs a{img, Wpacked, act_scale, w_scale, bias, nullptr, Y, (int)M, (int)D, (int)K, epilogue, (int)GPUSQ_F16};
  a.patch_P = 16;
  a.patch_C = (int)C;
  a.patch_H = (int)H;
  a.patch_W = (int)W;
  return launch_spgemm(is_i8, a, (hipStream_t)stream);
}

gpusq_status gpusq_patch_embed16_int8(const int8_t* img, const void* Wpacked, const float* act_scale, const float* w_scale,
                                      const float* bias, void* Y, int64_t B, int64_t C, int64_t H, int64_t W, int64_t D,
                                      int epilogue, void* stream) {
  return patch_embed16(true, img, Wpacked, act_scale, w_scale, bias, Y, B, C, H, W, D, epilogue, stream);
}

gpusq_status gpusq_patch_embed16_fp16(const void* img, const void* Wpacked, const float* bias, void* Y, int64_t B, int64_t C,
                                      int64_t H, int64_t W, int64_t D, int epilogue, void* stream) {
  return patch_embed16(false, img, Wpacked, nullptr, nullptr, bias, Y, B, C, H, W, D, epilogue, stream);
}

gpusq_status gpusq_spgemm_plan(gpusq_dtype dt, int64_t M, int64_t N, int64_t K, int epilogue, int cus, int32_t out[8]) {
  if (!out) return GPUSQ_ERR_NULL;
  if (M <= 0) return GPUSQ_ERR_SHAPE;
  gpusq_status st = check_nk(N, K);
  if (st != GPUSQ_OK) return st;
  if (M > INT32_MAX || M * N > kMaxElems || M * K > kMaxElems) return GPUSQ_ERR_SHAPE;
  if (dt != GPUSQ_F16 && dt != GPUSQ_I8) return GPUSQ_ERR_UNSUPPORTED;
  if (epilogue & ~(GPUSQ_EPI_BIAS | GPUSQ_EPI_GELU)) return GPUSQ_ERR_UNSUPPORTED;
  if (K % 16 != 0 || N % 4 != 0) return GPUSQ_ERR_UNSUPPORTED;
  return plan_spgemm(dt == GPUSQ_I8, M, N, K, epilogue, cus, out);
}

int gpusq_force_kernel(int kernel) { return set_forced_kernel(kernel); }

gpusq_status gpusq_spgemm_fp16(const void* X, const void* Wpacked, const float* bias, void* Y, int64_t M, int64_t N,
                               int64_t K, int epilogue, void* stream) {
  gpusq_status st = check_gemm(X, Wpacked, bias, Y, M, N, K, epilogue);
  if (st != GPUSQ_OK) return st;
  GemmArgs a{X, Wpacked, nullptr, nullptr, bias, nullptr, Y, (int)M, (int)N, (int)K, epilogue, (int)GPUSQ_F16};
  return launch_spgemm(false, a, (hipStream_t)stream);
}

gpusq_status gpusq_spgemm_int8(const int8_t* Xq, const void* Wpacked, const float* act_scale, const float* w_scale,
                               const float* bias, void* Y, gpusq_dtype out_dt, const float* out_scale, int64_t M,
                               int64_t N, int64_t K, int epilogue, void* stream) {
  gpusq_status st = check_gemm(Xq, Wpacked, bias, Y, M, N, K, epilogue);
  if (st != GPUSQ_OK) return st;
  st = check_int8_extras(act_scale, w_scale, out_dt, out_scale);
  if (st != GPUSQ_OK) return st;
  GemmArgs a{Xq, Wpacked, act_scale, w_scale, bias, out_scale, Y, (int)M, (int)N, (int)K, epilogue, (int)out_dt};
  return launch_spgemm(true, a, (hipStream_t)stream);
}

gpusq_status gpusq_spgemm_int8_xf16(const void* X, const void* Wpacked, const float* act_scale, const float* w_scale,
                                    const float* bias, void* Y, gpusq_dtype out_dt, const float* out_scale, int64_t M,
                                    int64_t N, int64_t K, int epilogue, void* stream) {
  gpusq_status st = check_gemm(X, Wpacked, bias, Y, M, N, K, epilogue);
  if (st != GPUSQ_OK) return st;
  st = check_int8_extras(act_scale, w_scale, out_dt, out_scale);
  if (st != GPUSQ_OK) return st;
  GemmArgs a{X, Wpacked, act_scale, w_scale, bias, out_scale, Y, (int)M, (int)N, (int)K, epilogue, (int)out_dt};
  a.x_f16 = 1;
  return launch_spgemm(true, a, (hipStream_t)stream);
}

gpusq_status gpusq_gemm_fp16_dense(const void* X, const void* W, const float* bias, void* Y, int64_t M, int64_t N,
                                   int64_t K, int epilogue, void* stream) {
  gpusq_status st = check_gemm(X, W, bias, Y, M, N, K, epilogue);
  if (st != GPUSQ_OK) return st;
  GemmArgs a{X, W, nullptr, nullptr, bias, nullptr, Y, (int)M, (int)N, (int)K, epilogue, (int)GPUSQ_F16};
  return launch_dense(false, a, (hipStream_t)stream);
}

gpusq_status gpusq_gemm_int8_dense(const int8_t* Xq, const int8_t* Wq, const float* act_scale, const float* w_scale,
                                   const float* bias, void* Y, gpusq_dtype out_dt, const float* out_scale, int64_t M,
                                   int64_t N, int64_t K, int epilogue, void* stream) {
  gpusq_status st = check_gemm(Xq, Wq, bias, Y, M, N, K, epilogue);
  if (st != GPUSQ_OK) return st;
  st = check_int8_extras(act_scale, w_scale, out_dt, out_scale);
  if (st != GPUSQ_OK) return st;
  GemmArgs a{Xq, Wq, act_scale, w_scale, bias, out_scale, Y, (int)M, (int)N, (int)K, epilogue, (int)out_dt};
  return launch_dense(true, a, (hipStream_t)stream);
}

}  // extern "C"
