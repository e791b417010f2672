/*
 * gpusq_oracle.c -- plain CPU oracle for the 2:4 structured-sparse linear-layer path.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the GPU library; the product never calls it.  Only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg may load it.  It shares no code, header, table or
 * helper with the HIP sources.
 *
 * What it implements, straight from the definitions (paper sections in brackets):
 *   - the 2:4 fine-grained structured sparse pattern: in every 4 contiguous elements along a row of the sparse
 *     operand, two are zero [Sec. 1; Sec. 3.1; Fig. 1];
 *   - the compressed storage: the kept values (rows x K/2) plus 2 bits of metadata per kept value giving its
 *     position inside its group of 4 [Sec. 3.1, Fig. 2 caption];
 *   - the sparse GEMM, which must give the same C as the dense GEMM on the zero-filled operand [Sec. 3.1];
 *   - symmetric INT8 quantisation with a scale factor [Sec. 2.2; Sec. 3.4], order "prune first, then quantise"
 *     [Sec. 3.1, last sentence of the storage-format paragraph];
 *   - the pair-wise 4:8 pattern of INT4 operands and its storage (4 kept 4-bit values + two 2-bit indices per chunk
 *     of 8) [Sec. 3.1, paragraph on the INT4 instruction], decoded to INT8 for the multiply-accumulate.
 * The paper does not state the pruning criterion, tie-break, rounding mode or scale granularity; the readings
 * taken here (magnitude top-2, ties to the lower index, scale = amax/127, round-half-even, per-output-channel
 * weights, per-tensor activations) are listed in the design notes of the repository.
 *
 * Naming: the paper's sparse matrix "A" (M x K) is the weight matrix; here it is W [N][K] (nn.Linear layout, K
 * contiguous), the dense operand is X [M][K] (tokens x features) and the result is Y [M][N] = X * W^T.
 *
 * Parity pins (tests/test_oracle_pins.py): exactly-2-of-4 invariant, brute force over the 6 index pairs,
 * exhaustive small-integer grids, compress/decompress round trip, the storage-saving closed forms printed in
 * Sec. 3.1 (43.75 % / 37.5 %), sparse GEMM == dense GEMM on masked weights, numpy int64 / float64 matmul,
 * quantiser error bound, GELU closed-form values; the patch-embedding convolution against the reshape-and-matmul
 * form computed by numpy and against the operation count printed in Sec. 3.3; the INT4 pair-wise format against a brute
 * force over the 6 choices of two sub-chunks, the worked example of Sec. 3.1 (w, x, y, z), the 37.5 % saving printed there,
 * round trips and numpy's quantiser formula.  No function here is "parity unpinned".
 *
 * Loops are the definitions written out; the only parallelism is an OpenMP "for" over independent output rows.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------ fp16 <-> fp32 (IEEE binary16, RNE) */

float oracle_f16_to_f32(uint16_t h) {
  uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  uint32_t exp = (h >> 10) & 0x1Fu;
  uint32_t man = h & 0x3FFu;
  uint32_t bits;
  if (exp == 0) {
    if (man == 0) {
      bits = sign;
    } else { /* subnormal: value = man * 2^-24 */
      float f = (float)man * 5.9604644775390625e-8f; /* exact */
      memcpy(&bits, &f, 4);
      bits |= sign;
    }
  } else if (exp == 31) {
    bits = sign | 0x7F800000u | (man << 13);
  } else {
    bits = sign | ((exp + 112u) << 23) | (man << 13);
  }
  float out;
  memcpy(&out, &bits, 4);
  return out;
}

/* round-to-nearest-even from a double (so that a value computed in fp64 is rounded once) */
uint16_t oracle_f64_to_f16(double d) {
  uint16_t sign = signbit(d) ? 0x8000u : 0;
  double a = fabs(d);
  if (isnan(d)) return (uint16_t)(sign | 0x7E00u);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7C00u); /* rounds to inf (65520 is the midpoint, ties to even = inf) */
  if (a < 6.103515625e-05) {                            /* below the smallest normal: multiples of 2^-24 */
    double q = nearbyint(a * 16777216.0);               /* RNE in the default rounding mode; exact scaling */
    return (uint16_t)(sign | (uint16_t)q);              /* q == 1024 lands exactly on the smallest normal */
  }
  int e;
  double m = frexp(a, &e); /* a = m * 2^e, m in [0.5,1) */
  /* significand with 11 bits: m * 2^11 in [1024, 2048) */
  double q = nearbyint(m * 2048.0);
  if (q == 2048.0) { q = 1024.0; e += 1; }
  int be = e - 1 + 15; /* biased exponent of 1.xxx * 2^(e-1) */
  if (be >= 31) return (uint16_t)(sign | 0x7C00u);
  return (uint16_t)(sign | (uint16_t)(be << 10) | ((uint16_t)q & 0x3FFu));
}

uint16_t oracle_f32_to_f16(float f) { return oracle_f64_to_f16((double)f); }

/* ------------------------------------------------------------------ a1: prune 2:4 */

/* Top-2 by magnitude inside one group of 4.  key[i] is a totally ordered magnitude (sign-cleared bit pattern or
 * |integer|); ties go to the lower index.  Returns the two kept positions with *p0 < *p1. */
static void top2_of_4(const uint32_t key[4], int* p0, int* p1) {
  int first = 0;
  for (int i = 1; i < 4; ++i)
    if (key[i] > key[first]) first = i;
  int second = -1;
  for (int i = 0; i < 4; ++i) {
    if (i == first) continue;
    if (second < 0 || key[i] > key[second]) second = i;
  }
  if (first < second) { *p0 = first; *p1 = second; } else { *p0 = second; *p1 = first; }
}

/* W, Wout: [N][K] fp32 (may alias).  mask (optional): N*K/4 bytes, bit i of byte g = element 4g+i kept. */
int oracle_prune_2to4_f32(const float* W, float* Wout, uint8_t* mask, int64_t N, int64_t K) {
  if (K % 4) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t g = 0; g < K / 4; ++g) {
      const float* w = W + n * K + 4 * g;
      uint32_t key[4];
      float v[4];
      for (int i = 0; i < 4; ++i) {
        v[i] = w[i];
        uint32_t b;
        memcpy(&b, &v[i], 4);
        key[i] = b & 0x7FFFFFFFu;
      }
      int p0, p1;
      top2_of_4(key, &p0, &p1);
      for (int i = 0; i < 4; ++i) Wout[n * K + 4 * g + i] = (i == p0 || i == p1) ? v[i] : 0.0f;
      if (mask) mask[n * (K / 4) + g] = (uint8_t)((1u << p0) | (1u << p1));
    }
  }
  return 0;
}

int oracle_prune_2to4_f16(const uint16_t* W, uint16_t* Wout, uint8_t* mask, int64_t N, int64_t K) {
  if (K % 4) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t g = 0; g < K / 4; ++g) {
      const uint16_t* w = W + n * K + 4 * g;
      uint32_t key[4];
      uint16_t v[4];
      for (int i = 0; i < 4; ++i) { v[i] = w[i]; key[i] = v[i] & 0x7FFFu; }
      int p0, p1;
      top2_of_4(key, &p0, &p1);
      for (int i = 0; i < 4; ++i) Wout[n * K + 4 * g + i] = (i == p0 || i == p1) ? v[i] : (uint16_t)0;
      if (mask) mask[n * (K / 4) + g] = (uint8_t)((1u << p0) | (1u << p1));
    }
  }
  return 0;
}

/* Other n:m patterns [Sec. 5, the limitation paragraph names 1:4 and 2:16 as patterns a later hardware generation might
 * support]: the n largest magnitudes of every m contiguous elements of a row are kept (ties: the lower index), the
 * others become +0.  n = 2, m = 4 is oracle_prune_2to4_f32.  1:4 and 2:16 tensors are 2:4 tensors as well. */
int oracle_prune_n_of_m_f32(const float* W, float* Wout, int n_keep, int m, int64_t N, int64_t K) {
  if (m < 2 || m > 64 || n_keep < 1 || n_keep >= m || K % m) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < N; ++r)
    for (int64_t g = 0; g < K / m; ++g) {
      float v[64];
      uint32_t key[64];
      int kept[64];
      for (int i = 0; i < m; ++i) {
        v[i] = W[r * K + g * m + i];
        uint32_t b;
        memcpy(&b, &v[i], 4);
        key[i] = b & 0x7FFFFFFFu;
        kept[i] = 0;
      }
      for (int round = 0; round < n_keep; ++round) { /* pick the largest remaining, lowest index first among equals */
        int best = -1;
        for (int i = 0; i < m; ++i)
          if (!kept[i] && (best < 0 || key[i] > key[best])) best = i;
        kept[best] = 1;
      }
      for (int i = 0; i < m; ++i) Wout[r * K + g * m + i] = kept[i] ? v[i] : 0.0f;
    }
  return 0;
}

/* ------------------------------------------------------------------ a2 / a4: symmetric INT8 quantisation */

static int8_t quantize_one(float x, float s) {
  float r = rintf(x / s); /* IEEE fp32 division, round-half-even (default rounding mode) */
  if (r > 127.0f) r = 127.0f;
  if (r < -127.0f) r = -127.0f;
  if (r != r) r = 0.0f; /* NaN input: deterministic 0 */
  return (int8_t)r;
}

/* per-row (= per-output-channel) scales: scale[r] = max_c |X[r][c]| / 127 (1.0f for an all-zero row) unless
 * scale_is_input; q = clamp(rint(x / scale)). */
int oracle_quantize_rows_int8(const float* X, int8_t* Q, float* scale, int scale_is_input, int64_t rows, int64_t cols) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    float s;
    if (scale_is_input) {
      s = scale[r];
    } else {
      float amax = 0.0f;
      for (int64_t c = 0; c < cols; ++c) {
        float a = fabsf(X[r * cols + c]);
        if (a > amax) amax = a;
      }
      s = (amax == 0.0f) ? 1.0f : amax / 127.0f;
      scale[r] = s;
    }
    for (int64_t c = 0; c < cols; ++c) Q[r * cols + c] = quantize_one(X[r * cols + c], s);
  }
  return 0;
}

/* per-tensor scale: scale[0] = max |X| / 127 over all n elements (1.0f when all zero) unless scale_is_input */
int oracle_quantize_tensor_int8(const float* X, int8_t* Q, float* scale, int scale_is_input, int64_t n) {
  float s;
  if (scale_is_input) {
    s = scale[0];
  } else {
    float amax = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
      float a = fabsf(X[i]);
      if (a > amax) amax = a;
    }
    s = (amax == 0.0f) ? 1.0f : amax / 127.0f;
    scale[0] = s;
  }
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) Q[i] = quantize_one(X[i], s);
  return 0;
}

/* ------------------------------------------------------------------ a3: compress / decompress */

/* meta: [N][ceil(K/8)] bytes; byte b of a row: group 2b in bits 0..3, group 2b+1 in bits 4..7; in a nibble,
 * bits 0..1 = position of the first kept value, bits 2..3 = position of the second (first < second). */
static int64_t meta_row_bytes(int64_t K) { return (K / 4 + 1) / 2; }

int oracle_compress_f16(const uint16_t* W, uint16_t* values, uint8_t* meta, int32_t* violations, int64_t N, int64_t K) {
  if (K % 4) return -1;
  int64_t mrb = meta_row_bytes(K);
  int32_t viol = 0;
  memset(meta, 0, (size_t)(N * mrb));
#pragma omp parallel for schedule(static) reduction(+ : viol)
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t g = 0; g < K / 4; ++g) {
      const uint16_t* w = W + n * K + 4 * g;
      uint32_t key[4];
      for (int i = 0; i < 4; ++i) key[i] = w[i] & 0x7FFFu;
      int p0, p1;
      top2_of_4(key, &p0, &p1);
      values[n * (K / 2) + 2 * g + 0] = w[p0];
      values[n * (K / 2) + 2 * g + 1] = w[p1];
      uint8_t nib = (uint8_t)(p0 | (p1 << 2));
      meta[n * mrb + g / 2] |= (uint8_t)((g & 1) ? (nib << 4) : nib);
      int dropped_nonzero = 0;
      for (int i = 0; i < 4; ++i)
        if (i != p0 && i != p1 && key[i] != 0) dropped_nonzero = 1;
      viol += dropped_nonzero;
    }
  }
  if (violations) *violations = viol;
  return 0;
}

int oracle_compress_i8(const int8_t* W, int8_t* values, uint8_t* meta, int32_t* violations, int64_t N, int64_t K) {
  if (K % 4) return -1;
  int64_t mrb = meta_row_bytes(K);
  int32_t viol = 0;
  memset(meta, 0, (size_t)(N * mrb));
#pragma omp parallel for schedule(static) reduction(+ : viol)
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t g = 0; g < K / 4; ++g) {
      const int8_t* w = W + n * K + 4 * g;
      uint32_t key[4];
      for (int i = 0; i < 4; ++i) key[i] = (uint32_t)abs((int)w[i]);
      int p0, p1;
      top2_of_4(key, &p0, &p1);
      values[n * (K / 2) + 2 * g + 0] = w[p0];
      values[n * (K / 2) + 2 * g + 1] = w[p1];
      uint8_t nib = (uint8_t)(p0 | (p1 << 2));
      meta[n * mrb + g / 2] |= (uint8_t)((g & 1) ? (nib << 4) : nib);
      int dropped_nonzero = 0;
      for (int i = 0; i < 4; ++i)
        if (i != p0 && i != p1 && key[i] != 0) dropped_nonzero = 1;
      viol += dropped_nonzero;
    }
  }
  if (violations) *violations = viol;
  return 0;
}

static void nibble_positions(const uint8_t* meta, int64_t mrb, int64_t n, int64_t g, int* p0, int* p1) {
  uint8_t byte = meta[n * mrb + g / 2];
  uint8_t nib = (g & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 0xF);
  *p0 = nib & 3;
  *p1 = (nib >> 2) & 3;
}

int oracle_decompress_f16(const uint16_t* values, const uint8_t* meta, uint16_t* W, int64_t N, int64_t K) {
  if (K % 4) return -1;
  int64_t mrb = meta_row_bytes(K);
  memset(W, 0, (size_t)(N * K) * 2);
  for (int64_t n = 0; n < N; ++n)
    for (int64_t g = 0; g < K / 4; ++g) {
      int p0, p1;
      nibble_positions(meta, mrb, n, g, &p0, &p1);
      W[n * K + 4 * g + p0] = values[n * (K / 2) + 2 * g];
      W[n * K + 4 * g + p1] = values[n * (K / 2) + 2 * g + 1];
    }
  return 0;
}

int oracle_decompress_i8(const int8_t* values, const uint8_t* meta, int8_t* W, int64_t N, int64_t K) {
  if (K % 4) return -1;
  int64_t mrb = meta_row_bytes(K);
  memset(W, 0, (size_t)(N * K));
  for (int64_t n = 0; n < N; ++n)
    for (int64_t g = 0; g < K / 4; ++g) {
      int p0, p1;
      nibble_positions(meta, mrb, n, g, &p0, &p1);
      W[n * K + 4 * g + p0] = values[n * (K / 2) + 2 * g];
      W[n * K + 4 * g + p1] = values[n * (K / 2) + 2 * g + 1];
    }
  return 0;
}

/* ------------------------------------------------------------------ INT4: pair-wise 4:8 pattern and its storage */

/* The pattern the paper describes for INT4 operands [Sec. 3.1, paragraph on the INT4 instruction]: a row is cut into
 * chunks of 8 adjacent elements, a chunk into 4 sub-chunks of 2; every sub-chunk is all zero or all non-zero and
 * exactly two of the four are kept.  The compressed row stores the 4 kept values of a chunk and two 2-bit indices
 * with the positions of the two kept sub-chunks.
 * The paper gives no selection rule; as for 2:4, magnitude decides: a sub-chunk's score is |a| + |b| (one fp32
 * addition; an integer sum for integer operands), the two highest scores are kept, ties go to the lower index.
 * Scores are compared as totally ordered keys (the sign-cleared bit pattern of the fp32 sum). */
static void top2_pairs_f32(const float* w, int* p0, int* p1) {
  uint32_t key[4];
  for (int p = 0; p < 4; ++p) {
    float sum = fabsf(w[2 * p]) + fabsf(w[2 * p + 1]);
    uint32_t b;
    memcpy(&b, &sum, 4);
    key[p] = b & 0x7FFFFFFFu;
  }
  top2_of_4(key, p0, p1);
}

static void top2_pairs_i8(const int8_t* w, int* p0, int* p1) {
  uint32_t key[4];
  for (int p = 0; p < 4; ++p) key[p] = (uint32_t)(abs((int)w[2 * p]) + abs((int)w[2 * p + 1]));
  top2_of_4(key, p0, p1);
}

/* The same pattern with one more constraint, chosen for hardware whose sparse matrix instructions know 2:4 only: of the
 * two kept sub-chunks one lies in the first group of 4 and one in the second (4 of the 6 choices), so that the tensor
 * obeys the pair-wise 4:8 pattern and the 2:4 pattern at once.  In each group of 4 the sub-chunk with the higher score
 * is kept (ties: the lower index). */
static void one_pair_per_group_f32(const float* w, int* p0, int* p1) {
  int keep[2];
  for (int h = 0; h < 2; ++h) {
    uint32_t key[2];
    for (int p = 0; p < 2; ++p) {
      float sum = fabsf(w[4 * h + 2 * p]) + fabsf(w[4 * h + 2 * p + 1]);
      uint32_t b;
      memcpy(&b, &sum, 4);
      key[p] = b & 0x7FFFFFFFu;
    }
    keep[h] = 2 * h + (key[1] > key[0] ? 1 : 0);
  }
  *p0 = keep[0];
  *p1 = keep[1];
}

/* W, Wout: [N][K] fp32 (may alias), K % 8 == 0.  mask (optional): N*K/8 bytes, bit p of byte c = sub-chunk p of chunk c kept.
 * one_per_group != 0: the constrained choice above. */
int oracle_prune_4to8_pairs_f32(const float* W, float* Wout, uint8_t* mask, int one_per_group, int64_t N, int64_t K) {
  if (K % 8) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t c = 0; c < K / 8; ++c) {
      float v[8];
      for (int i = 0; i < 8; ++i) v[i] = W[n * K + 8 * c + i];
      int p0, p1;
      if (one_per_group)
        one_pair_per_group_f32(v, &p0, &p1);
      else
        top2_pairs_f32(v, &p0, &p1);
      for (int i = 0; i < 8; ++i) Wout[n * K + 8 * c + i] = (i / 2 == p0 || i / 2 == p1) ? v[i] : 0.0f;
      if (mask) mask[n * (K / 8) + c] = (uint8_t)((1u << p0) | (1u << p1));
    }
  return 0;
}

/* symmetric INT4 codes in int8 containers: q = clamp(rint(x / s), -7, 7), s = max|row| / 7 (1 for an all-zero row)
 * unless scale_is_input: the INT8 quantiser of Sec. 2.2 / 3.4 with the 4-bit range. */
int oracle_quantize_rows_int4(const float* X, int8_t* Q, float* scale, int scale_is_input, int64_t rows, int64_t cols) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    float s;
    if (scale_is_input) {
      s = scale[r];
    } else {
      float amax = 0.0f;
      for (int64_t c = 0; c < cols; ++c) {
        float a = fabsf(X[r * cols + c]);
        if (a > amax) amax = a;
      }
      s = (amax == 0.0f) ? 1.0f : amax / 7.0f;
      scale[r] = s;
    }
    for (int64_t c = 0; c < cols; ++c) {
      float q = rintf(X[r * cols + c] / s);
      if (q > 7.0f) q = 7.0f;
      if (q < -7.0f) q = -7.0f;
      if (q != q) q = 0.0f;
      Q[r * cols + c] = (int8_t)q;
    }
  }
  return 0;
}

/* W [N][K] int8 holding INT4 codes (-8..7), K % 8 == 0.
 * values: [N][K/4] bytes; the 4 kept codes of chunk c, in ascending position, as two's-complement nibbles: kept code j
 *         in byte 2c + j/2, low nibble for even j.
 * meta:   [N][ceil(K/16)] bytes; chunk c in the low (c even) or high (c odd) nibble of byte c/2; in the nibble,
 *         bits 0..1 = first kept sub-chunk, bits 2..3 = second (first < second).
 * violations (optional): chunks in which a dropped element was non-zero or a code was outside -8..7. */
static int64_t meta4_row_bytes(int64_t K) { return (K / 8 + 1) / 2; }

int oracle_compress_int4_pairs(const int8_t* W, uint8_t* values, uint8_t* meta, int32_t* violations, int64_t N, int64_t K) {
  if (K % 8) return -1;
  int64_t mrb = meta4_row_bytes(K);
  int32_t viol = 0;
  memset(meta, 0, (size_t)(N * mrb));
#pragma omp parallel for schedule(static) reduction(+ : viol)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t c = 0; c < K / 8; ++c) {
      const int8_t* w = W + n * K + 8 * c;
      int p0, p1;
      top2_pairs_i8(w, &p0, &p1);
      const int8_t kept[4] = {w[2 * p0], w[2 * p0 + 1], w[2 * p1], w[2 * p1 + 1]};
      for (int j = 0; j < 4; j += 2)
        values[n * (K / 4) + 2 * c + j / 2] = (uint8_t)((kept[j] & 0xF) | ((kept[j + 1] & 0xF) << 4));
      uint8_t nib = (uint8_t)(p0 | (p1 << 2));
      meta[n * mrb + c / 2] |= (uint8_t)((c & 1) ? (nib << 4) : nib);
      int bad = 0;
      for (int i = 0; i < 8; ++i) {
        if (i / 2 != p0 && i / 2 != p1 && w[i] != 0) bad = 1;
        if (w[i] < -8 || w[i] > 7) bad = 1;
      }
      viol += bad;
    }
  if (violations) *violations = viol;
  return 0;
}

/* inverse: the dense INT8 operand [N][K] (zero-filled, codes sign-extended): what the multiply-accumulate consumes */
int oracle_decompress_int4_pairs(const uint8_t* values, const uint8_t* meta, int8_t* W, int64_t N, int64_t K) {
  if (K % 8) return -1;
  int64_t mrb = meta4_row_bytes(K);
  memset(W, 0, (size_t)(N * K));
  for (int64_t n = 0; n < N; ++n)
    for (int64_t c = 0; c < K / 8; ++c) {
      uint8_t byte = meta[n * mrb + c / 2];
      uint8_t nib = (c & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 0xF);
      int p[2] = {nib & 3, (nib >> 2) & 3};
      for (int j = 0; j < 4; ++j) {
        uint8_t b = values[n * (K / 4) + 2 * c + j / 2];
        int code = (j & 1) ? (b >> 4) : (b & 0xF);
        if (code >= 8) code -= 16;
        W[n * K + 8 * c + 2 * p[j / 2] + (j & 1)] = (int8_t)code;
      }
    }
  return 0;
}

/* A pair-wise 4:8 row in which no group of 4 holds two non-zero sub-chunks is also a 2:4 row: its INT8 compressed form
 * (values [N][K/2] = the codes of the group's non-zero sub-chunk, sign-extended; metadata nibble per group of 4 = the
 * two positions of that sub-chunk; a group without non-zeros takes its first sub-chunk) follows from the INT4 form
 * chunk by chunk.  mismatches = groups of 4 with two non-zero sub-chunks (they keep the second one only). */
int oracle_int4_pairs_to_sparse_int8(const uint8_t* values4, const uint8_t* meta4, int8_t* values8, uint8_t* meta8,
                                     int32_t* mismatches, int64_t N, int64_t K) {
  if (K % 8) return -1;
  int64_t mrb4 = meta4_row_bytes(K), mrb8 = meta_row_bytes(K);
  int32_t bad = 0;
  memset(meta8, 0, (size_t)(N * mrb8));
  for (int64_t n = 0; n < N; ++n)
    for (int64_t c = 0; c < K / 8; ++c) {
      uint8_t byte = meta4[n * mrb4 + c / 2];
      uint8_t nib = (c & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 0xF);
      int p[2] = {nib & 3, (nib >> 2) & 3};
      int8_t dense[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      for (int j = 0; j < 4; ++j) {
        uint8_t b = values4[n * (K / 4) + 2 * c + j / 2];
        int code = (j & 1) ? (b >> 4) : (b & 0xF);
        if (code >= 8) code -= 16;
        dense[2 * p[j / 2] + (j & 1)] = (int8_t)code;
      }
      for (int h = 0; h < 2; ++h) {
        int64_t g = 2 * c + h;
        int nz0 = dense[4 * h] != 0 || dense[4 * h + 1] != 0;
        int nz1 = dense[4 * h + 2] != 0 || dense[4 * h + 3] != 0;
        bad += nz0 && nz1;
        int local = nz1 ? 1 : 0;
        uint8_t nib8 = (uint8_t)((2 * local) | ((2 * local + 1) << 2));
        meta8[n * mrb8 + g / 2] |= (uint8_t)((g & 1) ? (nib8 << 4) : nib8);
        values8[n * (K / 2) + 2 * g] = dense[4 * h + 2 * local];
        values8[n * (K / 2) + 2 * g + 1] = dense[4 * h + 2 * local + 1];
      }
    }
  if (mismatches) *mismatches = bad;
  return 0;
}

/* ------------------------------------------------------------------ a5: GEMM, INT8 with INT32 accumulation */

/* dense definition: acc[m][n] = sum_k X[m][k] * W[n][k] */
int oracle_gemm_int8_dense(const int8_t* X, const int8_t* W, int32_t* acc, int64_t M, int64_t N, int64_t K) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      int32_t s = 0;
      for (int64_t k = 0; k < K; ++k) s += (int32_t)X[m * K + k] * (int32_t)W[n * K + k];
      acc[m * N + n] = s;
    }
  return 0;
}

/* sparse form: only the kept values, each multiplied by the X element its metadata points at */
int oracle_spgemm_int8(const int8_t* X, const int8_t* values, const uint8_t* meta, int32_t* acc,
                       int64_t M, int64_t N, int64_t K) {
  if (K % 4) return -1;
  int64_t mrb = meta_row_bytes(K);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      int32_t s = 0;
      for (int64_t g = 0; g < K / 4; ++g) {
        int p0, p1;
        nibble_positions(meta, mrb, n, g, &p0, &p1);
        s += (int32_t)values[n * (K / 2) + 2 * g] * (int32_t)X[m * K + 4 * g + p0];
        s += (int32_t)values[n * (K / 2) + 2 * g + 1] * (int32_t)X[m * K + 4 * g + p1];
      }
      acc[m * N + n] = s;
    }
  return 0;
}

/* ------------------------------------------------------------------ a5: GEMM, FP16 operands */

/* dense definition.  Each product of two fp16 numbers is exact in fp32 and in fp64.  acc32: sequential fp32
 * accumulation in k order (optional).  acc64: fp64 accumulation (optional) -- the reference value. */
int oracle_gemm_fp16_dense(const uint16_t* X, const uint16_t* W, float* acc32, double* acc64,
                           int64_t M, int64_t N, int64_t K) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      float s32 = 0.0f;
      double s64 = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        float x = oracle_f16_to_f32(X[m * K + k]), w = oracle_f16_to_f32(W[n * K + k]);
        float p = x * w; /* exact: 11-bit x 11-bit significands */
        s32 = s32 + p;
        s64 = s64 + (double)x * (double)w;
      }
      if (acc32) acc32[m * N + n] = s32;
      if (acc64) acc64[m * N + n] = s64;
    }
  return 0;
}

int oracle_spgemm_fp16(const uint16_t* X, const uint16_t* values, const uint8_t* meta, float* acc32, double* acc64,
                       int64_t M, int64_t N, int64_t K) {
  if (K % 4) return -1;
  int64_t mrb = meta_row_bytes(K);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      float s32 = 0.0f;
      double s64 = 0.0;
      for (int64_t g = 0; g < K / 4; ++g) {
        int p[2];
        nibble_positions(meta, mrb, n, g, &p[0], &p[1]);
        for (int j = 0; j < 2; ++j) {
          float w = oracle_f16_to_f32(values[n * (K / 2) + 2 * g + j]);
          float x = oracle_f16_to_f32(X[m * K + 4 * g + p[j]]);
          s32 = s32 + x * w;
          s64 = s64 + (double)x * (double)w;
        }
      }
      if (acc32) acc32[m * N + n] = s32;
      if (acc64) acc64[m * N + n] = s64;
    }
  return 0;
}

/* ------------------------------------------------------------------ a6: epilogue */

static double gelu_exact(double v) { return 0.5 * v * (1.0 + erf(v * 0.70710678118654752440)); }

/* INT8 path, real-arithmetic reference in fp64:  v = acc * s_a * s_w[n] + bias[n]; optional exact-erf GELU.
 * ref (optional): v as a double before any output rounding.  Y16 (optional): v rounded once to fp16.
 * Q8 (optional, needs out_scale): clamp(rint(v / out_scale), -127, 127) computed in fp64. */
int oracle_epilogue_int8_f64(const int32_t* acc, float s_a, const float* s_w, const float* bias, int gelu,
                             double* ref, uint16_t* Y16, int8_t* Q8, float out_scale, int64_t M, int64_t N) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double v = (double)acc[m * N + n] * (double)s_a * (double)s_w[n];
      if (bias) v += (double)bias[n];
      if (gelu) v = gelu_exact(v);
      if (ref) ref[m * N + n] = v;
      if (Y16) Y16[m * N + n] = oracle_f64_to_f16(v);
      if (Q8) {
        double r = nearbyint(v / (double)out_scale);
        if (r > 127.0) r = 127.0;
        if (r < -127.0) r = -127.0;
        Q8[m * N + n] = (int8_t)r;
      }
    }
  return 0;
}

/* INT8 path, the same formula evaluated in fp32 in a fixed operation order, for the outputs where a rounding
 * decides an integer code or where bit-exact agreement is wanted:
 *   c = s_a * s_w[n] (one fp32 multiply);  v = fma((float)acc, c, bias[n])  (no bias: v = (float)acc * c);
 *   optional GELU evaluated in fp64 on v and rounded once to fp32;  Y16 = fp16(v) RNE;
 *   Q8 = clamp(rintf(v / out_scale), -127, 127) with an fp32 division. */
int oracle_epilogue_int8_f32(const int32_t* acc, float s_a, const float* s_w, const float* bias, int gelu,
                             float* V32, uint16_t* Y16, int8_t* Q8, float out_scale, int64_t M, int64_t N) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      float c = s_a * s_w[n];
      float a = (float)acc[m * N + n];
      float v = bias ? fmaf(a, c, bias[n]) : a * c;
      if (gelu) v = (float)gelu_exact((double)v);
      if (V32) V32[m * N + n] = v;
      if (Y16) Y16[m * N + n] = oracle_f32_to_f16(v);
      if (Q8) Q8[m * N + n] = quantize_one(v, out_scale);
    }
  return 0;
}

/* FP16 path: v = acc + bias[n] in fp64 from the fp64 accumulator; optional GELU; ref = v; Y16 = fp16(v). */
int oracle_epilogue_fp16_f64(const double* acc64, const float* bias, int gelu, double* ref, uint16_t* Y16,
                             int64_t M, int64_t N) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double v = acc64[m * N + n];
      if (bias) v += (double)bias[n];
      if (gelu) v = gelu_exact(v);
      if (ref) ref[m * N + n] = v;
      if (Y16) Y16[m * N + n] = oracle_f64_to_f16(v);
    }
  return 0;
}

/* ------------------------------------------------------------------ patch embedding as a strided convolution */

/* The patch-embedding layer [Sec. 3.3]: a convolution with C input channels, D output channels, kernel size and
 * stride both P, on images [B][C][H][W]; every P x P patch becomes one token.  Written out as the convolution it
 * is (no im2col, no GEMM):
 *   acc[b][py][px][d] = sum_{c, i, j} img[b][c][py*P + i][px*P + j] * Wc[d][c][i][j]
 * H and W must be multiples of P.  Returns the number of multiply-accumulates performed (counted in the loops), so
 * that the operation count the paper prints, 2 * B * C * H * W * D, can be checked against the loops themselves;
 * -1 on a shape error. */
int64_t oracle_patch_conv_int8(const int8_t* img, const int8_t* Wc, int32_t* acc, int64_t B, int64_t C, int64_t H,
                               int64_t W, int64_t P, int64_t D) {
  if (P <= 0 || H % P || W % P) return -1;
  const int64_t py_n = H / P, px_n = W / P;
  int64_t macs = 0;
#pragma omp parallel for schedule(static) reduction(+ : macs)
  for (int64_t t = 0; t < B * py_n * px_n; ++t) {
    const int64_t b = t / (py_n * px_n), py = (t / px_n) % py_n, px = t % px_n;
    for (int64_t d = 0; d < D; ++d) {
      int32_t s = 0;
      for (int64_t c = 0; c < C; ++c)
        for (int64_t i = 0; i < P; ++i)
          for (int64_t j = 0; j < P; ++j) {
            s += (int32_t)img[((b * C + c) * H + py * P + i) * W + px * P + j] * (int32_t)Wc[((d * C + c) * P + i) * P + j];
            ++macs;
          }
      acc[t * D + d] = s;
    }
  }
  return macs;
}

/* The same for fp16 operands, accumulated in fp64 (each product of two fp16 numbers is exact in fp64). */
int64_t oracle_patch_conv_f16(const uint16_t* img, const uint16_t* Wc, double* acc64, int64_t B, int64_t C, int64_t H,
                              int64_t W, int64_t P, int64_t D) {
  if (P <= 0 || H % P || W % P) return -1;
  const int64_t py_n = H / P, px_n = W / P;
  int64_t macs = 0;
#pragma omp parallel for schedule(static) reduction(+ : macs)
  for (int64_t t = 0; t < B * py_n * px_n; ++t) {
    const int64_t b = t / (py_n * px_n), py = (t / px_n) % py_n, px = t % px_n;
    for (int64_t d = 0; d < D; ++d) {
      double s = 0.0;
      for (int64_t c = 0; c < C; ++c)
        for (int64_t i = 0; i < P; ++i)
          for (int64_t j = 0; j < P; ++j) {
            s += (double)oracle_f16_to_f32(img[((b * C + c) * H + py * P + i) * W + px * P + j]) *
                 (double)oracle_f16_to_f32(Wc[((d * C + c) * P + i) * P + j]);
            ++macs;
          }
      acc64[t * D + d] = s;
    }
  }
  return macs;
}

/* ------------------------------------------------------------------ whole linear layer, sparse form (CPU baseline) */

/* Y16[m][n] = fp16( epilogue( sum over kept values ) ), INT8 path, one pass; used for timing the oracle. */
int oracle_linear_int8_sparse(const int8_t* X, const int8_t* values, const uint8_t* meta, float s_a, const float* s_w,
                              const float* bias, int gelu, uint16_t* Y16, int64_t M, int64_t N, int64_t K) {
  int32_t* acc = (int32_t*)malloc((size_t)(M * N) * sizeof(int32_t));
  if (!acc) return -2;
  int r = oracle_spgemm_int8(X, values, meta, acc, M, N, K);
  if (r == 0) r = oracle_epilogue_int8_f64(acc, s_a, s_w, bias, gelu, NULL, Y16, NULL, 1.0f, M, N);
  free(acc);
  return r;
}
