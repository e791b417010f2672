/* Self-test driver of the CPU oracle for sanitizer builds (TEST INFRASTRUCTURE, like the oracle itself).
 *
 * Compiled together with gpusq_oracle.c under -fsanitize=address,undefined, it runs every oracle function on small
 * seeded inputs held in heap buffers of exactly the documented sizes (so that a read or write past an operand is caught),
 * over the edge shapes of the method (one group, one row, one channel, K % 8 == 4, M not a multiple of anything), and
 * checks the invariants the paper fixes: two kept positions per group of 4 [Sec. 3.1], compress then decompress is the
 * identity on 2:4 tensors, the sparse product equals the dense product on the zero-filled operand [Sec. 3.1, Fig. 1].
 * Exit status 0 = all checks passed and no sanitizer report. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_prune_2to4_f32(const float*, float*, uint8_t*, int64_t, int64_t);
int oracle_prune_2to4_f16(const uint16_t*, uint16_t*, uint8_t*, int64_t, int64_t);
int oracle_prune_n_of_m_f32(const float*, float*, int, int, int64_t, int64_t);
int oracle_quantize_rows_int8(const float*, int8_t*, float*, int, int64_t, int64_t);
int oracle_quantize_tensor_int8(const float*, int8_t*, float*, int, int64_t);
int oracle_compress_f16(const uint16_t*, uint16_t*, uint8_t*, int32_t*, int64_t, int64_t);
int oracle_compress_i8(const int8_t*, int8_t*, uint8_t*, int32_t*, int64_t, int64_t);
int oracle_decompress_f16(const uint16_t*, const uint8_t*, uint16_t*, int64_t, int64_t);
int oracle_decompress_i8(const int8_t*, const uint8_t*, int8_t*, int64_t, int64_t);
int oracle_prune_4to8_pairs_f32(const float*, float*, uint8_t*, int, int64_t, int64_t);
int oracle_quantize_rows_int4(const float*, int8_t*, float*, int, int64_t, int64_t);
int oracle_compress_int4_pairs(const int8_t*, uint8_t*, uint8_t*, int32_t*, int64_t, int64_t);
int oracle_decompress_int4_pairs(const uint8_t*, const uint8_t*, int8_t*, int64_t, int64_t);
int oracle_int4_pairs_to_sparse_int8(const uint8_t*, const uint8_t*, int8_t*, uint8_t*, int32_t*, int64_t, int64_t);
int oracle_gemm_int8_dense(const int8_t*, const int8_t*, int32_t*, int64_t, int64_t, int64_t);
int oracle_spgemm_int8(const int8_t*, const int8_t*, const uint8_t*, int32_t*, int64_t, int64_t, int64_t);
int oracle_gemm_fp16_dense(const uint16_t*, const uint16_t*, float*, double*, int64_t, int64_t, int64_t);
int oracle_spgemm_fp16(const uint16_t*, const uint16_t*, const uint8_t*, float*, double*, int64_t, int64_t, int64_t);
int oracle_epilogue_int8_f64(const int32_t*, float, const float*, const float*, int, double*, uint16_t*, int8_t*, float, int64_t, int64_t);
int oracle_epilogue_int8_f32(const int32_t*, float, const float*, const float*, int, float*, uint16_t*, int8_t*, float, int64_t, int64_t);
int oracle_epilogue_fp16_f64(const double*, const float*, int, double*, uint16_t*, int64_t, int64_t);
int64_t oracle_patch_conv_int8(const int8_t*, const int8_t*, int32_t*, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t);
int64_t oracle_patch_conv_f16(const uint16_t*, const uint16_t*, double*, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t);
int oracle_linear_int8_sparse(const int8_t*, const int8_t*, const uint8_t*, float, const float*, const float*, int, uint16_t*, int64_t, int64_t, int64_t);
uint16_t oracle_f32_to_f16(float);
float oracle_f16_to_f32(uint16_t);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) {
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(rng_state >> 33);
}
static float rndf(void) { return ((int)(rnd() % 2001) - 1000) * 1e-3f; }
static int failures = 0;
#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "selftest: check failed at line %d: %s\n", __LINE__, #cond); \
      ++failures;                                                          \
    }                                                                      \
  } while (0)
static void* xmalloc(size_t n) {
  void* p = malloc(n ? n : 1);
  if (!p) abort();
  return p;
}

static void one_shape(int64_t M, int64_t N, int64_t K) {
  const int64_t mrb = (K / 4 + 1) / 2;
  float* W = xmalloc(sizeof(float) * N * K);
  float* Wp = xmalloc(sizeof(float) * N * K);
  uint8_t* mask = xmalloc(N * (K / 4));
  for (int64_t i = 0; i < N * K; ++i) W[i] = (rnd() % 5 == 0) ? 0.0f : rndf() * 0.02f;  /* some natural zeros and ties */
  CHECK(oracle_prune_2to4_f32(W, Wp, mask, N, K) == 0);
  for (int64_t g = 0; g < N * (K / 4); ++g) {
    CHECK(__builtin_popcount(mask[g]) == 2);
    int nz = 0;
    for (int i = 0; i < 4; ++i) nz += Wp[4 * g + i] != 0.0f;
    CHECK(nz <= 2);
  }
  /* fp16 branch */
  uint16_t* Wh = xmalloc(2 * N * K);
  uint16_t* Whp = xmalloc(2 * N * K);
  uint16_t* vals16 = xmalloc(2 * N * (K / 2));
  uint8_t* meta16 = xmalloc(N * mrb);
  uint16_t* back16 = xmalloc(2 * N * K);
  int32_t viol = -1;
  for (int64_t i = 0; i < N * K; ++i) Wh[i] = oracle_f32_to_f16(Wp[i]);
  CHECK(oracle_prune_2to4_f16(Wh, Whp, NULL, N, K) == 0);
  CHECK(oracle_compress_f16(Wh, vals16, meta16, &viol, N, K) == 0 && viol == 0);
  CHECK(oracle_decompress_f16(vals16, meta16, back16, N, K) == 0);
  for (int64_t i = 0; i < N * K; ++i) CHECK((Wh[i] & 0x7FFF) == (back16[i] & 0x7FFF) && ((Wh[i] & 0x7FFF) == 0 || Wh[i] == back16[i]));
  /* int8 branch */
  int8_t* Wq = xmalloc(N * K);
  float* s_w = xmalloc(sizeof(float) * N);
  int8_t* vals8 = xmalloc(N * (K / 2));
  uint8_t* meta8 = xmalloc(N * mrb);
  int8_t* back8 = xmalloc(N * K);
  CHECK(oracle_quantize_rows_int8(Wp, Wq, s_w, 0, N, K) == 0);
  for (int64_t i = 0; i < N * K; ++i) CHECK(Wq[i] >= -127);
  CHECK(oracle_compress_i8(Wq, vals8, meta8, &viol, N, K) == 0 && viol == 0);
  CHECK(oracle_decompress_i8(vals8, meta8, back8, N, K) == 0 && memcmp(Wq, back8, N * K) == 0);
  /* activations and products */
  float* X = xmalloc(sizeof(float) * M * K);
  int8_t* Xq = xmalloc(M * K);
  uint16_t* Xh = xmalloc(2 * M * K);
  float s_a = 0.0f;
  for (int64_t i = 0; i < M * K; ++i) {
    X[i] = rndf() * 3.0f;
    Xh[i] = oracle_f32_to_f16(X[i]);
  }
  CHECK(oracle_quantize_tensor_int8(X, Xq, &s_a, 0, M * K) == 0 && s_a > 0.0f);
  int32_t* accd = xmalloc(4 * M * N);
  int32_t* accs = xmalloc(4 * M * N);
  CHECK(oracle_gemm_int8_dense(Xq, Wq, accd, M, N, K) == 0 && oracle_spgemm_int8(Xq, vals8, meta8, accs, M, N, K) == 0);
  CHECK(memcmp(accd, accs, 4 * M * N) == 0);
  float* a32d = xmalloc(4 * M * N);
  float* a32s = xmalloc(4 * M * N);
  double* a64d = xmalloc(8 * M * N);
  double* a64s = xmalloc(8 * M * N);
  CHECK(oracle_gemm_fp16_dense(Xh, Wh, a32d, a64d, M, N, K) == 0 && oracle_spgemm_fp16(Xh, vals16, meta16, a32s, a64s, M, N, K) == 0);
  for (int64_t i = 0; i < M * N; ++i) CHECK(fabs(a64d[i] - a64s[i]) <= 1e-12 * (1.0 + fabs(a64d[i])));
  /* epilogues: every optional output present, then absent */
  float* bias = xmalloc(sizeof(float) * N);
  for (int64_t n = 0; n < N; ++n) bias[n] = rndf() * 0.01f;
  double* ref = xmalloc(8 * M * N);
  float* v32 = xmalloc(4 * M * N);
  uint16_t* y16 = xmalloc(2 * M * N);
  uint16_t* y16b = xmalloc(2 * M * N);
  int8_t* q8 = xmalloc(M * N);
  for (int gelu = 0; gelu < 2; ++gelu) {
    CHECK(oracle_epilogue_int8_f64(accs, s_a, s_w, bias, gelu, ref, y16, q8, 0.01f, M, N) == 0);
    CHECK(oracle_epilogue_int8_f64(accs, s_a, s_w, NULL, gelu, NULL, y16, NULL, 1.0f, M, N) == 0);
    CHECK(oracle_epilogue_int8_f32(accs, s_a, s_w, bias, gelu, v32, y16b, q8, 0.01f, M, N) == 0);
    CHECK(oracle_epilogue_int8_f32(accs, s_a, s_w, NULL, gelu, NULL, NULL, NULL, 1.0f, M, N) == 0);
    CHECK(oracle_epilogue_fp16_f64(a64s, bias, gelu, ref, y16, M, N) == 0 && oracle_epilogue_fp16_f64(a64s, NULL, gelu, NULL, y16, M, N) == 0);
    CHECK(oracle_linear_int8_sparse(Xq, vals8, meta8, s_a, s_w, bias, gelu, y16, M, N, K) == 0);
  }
  /* other patterns and the INT4 pair-wise format (K % 8 == 0 only) */
  if (K % 16 == 0) CHECK(oracle_prune_n_of_m_f32(W, Wp, 2, 16, N, K) == 0);
  CHECK(oracle_prune_n_of_m_f32(W, Wp, 1, 4, N, K) == 0);
  if (K % 8 == 0) {
    const int64_t mrb4 = (K / 8 + 1) / 2;
    uint8_t* m4 = xmalloc(N * (K / 8));
    int8_t* Q4 = xmalloc(N * K);
    float* s4 = xmalloc(sizeof(float) * N);
    uint8_t* v4 = xmalloc(N * (K / 4));
    uint8_t* me4 = xmalloc(N * mrb4);
    int8_t* D4 = xmalloc(N * K);
    for (int opg = 0; opg < 2; ++opg) {
      CHECK(oracle_prune_4to8_pairs_f32(W, Wp, m4, opg, N, K) == 0);
      CHECK(oracle_quantize_rows_int4(Wp, Q4, s4, 0, N, K) == 0);
      CHECK(oracle_compress_int4_pairs(Q4, v4, me4, &viol, N, K) == 0 && viol == 0);
      CHECK(oracle_decompress_int4_pairs(v4, me4, D4, N, K) == 0 && memcmp(Q4, D4, N * K) == 0);
      if (opg) {
        int32_t mism = -1;
        CHECK(oracle_int4_pairs_to_sparse_int8(v4, me4, vals8, meta8, &mism, N, K) == 0 && mism == 0);
        CHECK(oracle_decompress_i8(vals8, meta8, back8, N, K) == 0 && memcmp(Q4, back8, N * K) == 0);
      }
    }
    free(m4); free(Q4); free(s4); free(v4); free(me4); free(D4);
  }
  free(W); free(Wp); free(mask); free(Wh); free(Whp); free(vals16); free(meta16); free(back16); free(Wq); free(s_w); free(vals8);
  free(meta8); free(back8); free(X); free(Xq); free(Xh); free(accd); free(accs); free(a32d); free(a32s); free(a64d); free(a64s);
  free(bias); free(ref); free(v32); free(y16); free(y16b); free(q8);
}

static void patch_shapes(void) {
  const int64_t B = 2, C = 3, H = 8, Wd = 12, P = 4, D = 5;
  int8_t* img = xmalloc(B * C * H * Wd);
  int8_t* Wc = xmalloc(D * C * P * P);
  uint16_t* img16 = xmalloc(2 * B * C * H * Wd);
  uint16_t* Wc16 = xmalloc(2 * D * C * P * P);
  for (int64_t i = 0; i < B * C * H * Wd; ++i) { img[i] = (int8_t)(rnd() % 255 - 127); img16[i] = oracle_f32_to_f16(rndf()); }
  for (int64_t i = 0; i < D * C * P * P; ++i) { Wc[i] = (int8_t)(rnd() % 255 - 127); Wc16[i] = oracle_f32_to_f16(rndf()); }
  const int64_t T = B * (H / P) * (Wd / P);
  int32_t* acc = xmalloc(4 * T * D);
  double* acc64 = xmalloc(8 * T * D);
  CHECK(oracle_patch_conv_int8(img, Wc, acc, B, C, H, Wd, P, D) == B * C * H * Wd * D);
  CHECK(oracle_patch_conv_f16(img16, Wc16, acc64, B, C, H, Wd, P, D) == B * C * H * Wd * D);
  CHECK(oracle_patch_conv_int8(img, Wc, acc, B, C, H, Wd, 5, D) == -1);
  free(img); free(Wc); free(img16); free(Wc16); free(acc); free(acc64);
}

int main(void) {
  static const int64_t shapes[][3] = {{1, 1, 4}, {1, 4, 8}, {3, 5, 12}, {7, 9, 20}, {5, 16, 64}, {33, 17, 144}, {2, 3, 16}, {64, 48, 192}};
  for (unsigned i = 0; i < sizeof(shapes) / sizeof(shapes[0]); ++i) one_shape(shapes[i][0], shapes[i][1], shapes[i][2]);
  patch_shapes();
  /* conversions over every fp16 bit pattern: round trip */
  for (uint32_t h = 0; h < 0x10000u; ++h) {
    const float f = oracle_f16_to_f32((uint16_t)h);
    if (f == f) CHECK(oracle_f32_to_f16(f) == (uint16_t)h);
  }
  if (failures) {
    fprintf(stderr, "selftest: %d checks failed\n", failures);
    return 1;
  }
  printf("selftest ok\n");
  return 0;
}
