// Internal declarations shared by the HIP translation units of libgpusq (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/gpusq.h"

namespace gpusq {

// ---- geometry of the kernel-native packed weight format (written by pack.hip, read by the GEMM kernels) ----------
// K advances in steps of 128 bytes of the dense activation row (128 int8 or 64 fp16 elements), the K extent of one
// gfx950 sparse matrix instruction (v_smfmac_i32_16x16x128_i8 / v_smfmac_f32_16x16x64_f16).  Output channels are
// grouped in tiles of 256 = 4 blocks of 64 = 16 fragments of 16 rows.  The packed buffer is an array of tiles
// [ceil(N/256)][ksteps]; one tile holds, for its 256 channels and one K step,
//     16 fragments x 1024 bytes of kept values   (fragment f, lane l: 16 bytes at f*1024 + l*16)
//   + 16 fragments x 64 lanes of index bits      (4 bytes per lane for int8, 2 for fp16), starting at byte 16384
//     (see index_offset),
// so that a workgroup fetches a tile with whole 1 KB wavefront-wide copies and a wavefront reads a fragment with one
// 16-byte and one 4-byte (2-byte) access per lane.
constexpr int kRowBlock = 64;          // output channels whose fragments interleave (see packed_row_to_channel)
constexpr int kTileRows = 256;         // output channels per packed tile
constexpr int kStepBytes = 128;        // bytes of a dense activation row consumed per K step
constexpr int kFragValueBytes = 1024;  // 64 lanes x 16 bytes of kept values
constexpr int kTileValueBytes = 16 * kFragValueBytes;

__host__ __device__ constexpr int step_elems(bool is_i8) { return is_i8 ? 128 : 64; }
// index bytes of one fragment: 2 bits per kept value; 16 int8 values (32 bits) or 8 fp16 values (16 bits) per lane
__host__ __device__ constexpr int frag_index_bytes(bool is_i8) { return is_i8 ? 256 : 128; }
__host__ __device__ constexpr int tile_bytes(bool is_i8) { return kTileValueBytes + 16 * frag_index_bytes(is_i8); }
// Byte offset, inside a tile, of the index word of lane l of fragment f.  The index words are grouped per half tile
// (fragments 0..7 / 8..15 = the 128 channels one wavefront of the large-tile kernel owns) and, inside a half, per
// lane: a lane finds the index words of its 8 fragments in 32 (int8) or 16 (fp16) consecutive bytes and fetches them
// with two (one) 16-byte LDS reads instead of eight small ones.
__host__ __device__ constexpr int index_offset(bool is_i8, int f, int l) {
  const int ib = is_i8 ? 4 : 2;
  return kTileValueBytes + (f >> 3) * (64 * 8 * ib) + l * (8 * ib) + (f & 7) * ib;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Row r (0..15) of fragment t (0..3) inside a 64-row block holds output channel
//   n = 64*blk + 32*(t/2) + 8*(r/4) + 4*(t%2) + (r%4).
// The accumulator of a 16x16 matrix instruction gives lane l the rows 4*(l/16)..4*(l/16)+3 of its column, so with
// this permutation a lane ends up, over fragments 0 and 1, with the 8 consecutive channels 8*(l/16)..+7 of one
// activation row (16 bytes of fp16 output) and the four lane groups of a wavefront write 64 contiguous bytes of that
// row in one store; fragments 2 and 3 give the next 32 channels the same way.
__host__ __device__ inline int packed_row_to_channel(int t, int r) { return 32 * (t >> 1) + 8 * (r >> 2) + 4 * (t & 1) + (r & 3); }

// Integer code of x under the scale s: clamp(rint(x / s), -127, 127) with the IEEE fp32 division of the definition
// (not a reciprocal multiply) and round-half-even, NaN -> 0, so that the code is decided exactly as a plain CPU
// evaluation of the formula decides it -- but without paying for a division per element.  r = fl(1 / s) (correctly
// rounded, computed once per scale).  t = x * r carries two roundings, |t - x/s| <= |x/s| (2^-23 + 2^-48), and the
// correctly rounded quotient is within 2^-24 |x/s| of x/s, so the quotient lies within 0.38 |t| 2^-21 of t.  rint()
// of the two can differ only if a half-integer lies between them or on one of them, which is excluded when t is at
// least |t| 2^-21 away from every half-integer (t - floor(t) is exact in fp32).  Only the rare element inside that
// band (about 1 in 10^5 for |t| near 100) pays for the division; |t| >= 2^20, where the test always fails, is clamped
// either way.  +-inf and tiny or zero t take the multiply path and give the same code as the division.
__device__ __forceinline__ int finish_code(float x, float q, float qmax = 127.0f) {
  q = rintf(q);
  q = fminf(fmaxf(q, -qmax), qmax);  // NaN -> -qmax -> handled below
  return (x != x) ? 0 : (int)q;
}
// N values at once: the band test of all N values of all lanes is folded into one wavefront-uniform branch, so the
// common case executes no division at all (a per-element conditional is turned into a select by the compiler, which
// then evaluates the division for every element).
template <int N>
__device__ __forceinline__ void quantize_codes(const float (&x)[N], float s, float r, int (&q)[N], float qmax = 127.0f) {
  float t[N];
  bool near_half = false;
#pragma unroll
  for (int j = 0; j < N; ++j) {
    t[j] = x[j] * r;
    near_half |= fabsf(__builtin_amdgcn_fractf(t[j]) - 0.5f) < fabsf(t[j]) * 0x1p-21f;
  }
  if (__builtin_amdgcn_ballot_w64(near_half) != 0) {  // some element of some lane sits next to a rounding boundary
#pragma unroll
    for (int j = 0; j < N; ++j) t[j] = __fdiv_rn(x[j], s);
  }
#pragma unroll
  for (int j = 0; j < N; ++j) q[j] = finish_code(x[j], t[j]);
}
// The codes of 8 values as bytes, packed into two words (value 0 in the low byte of `lo`): the same codes as
// quantize_codes, with less arithmetic in the common case, for epilogues that are bound by the vector ALU.
//   * band test |fract(t) - 0.5| < 2^-14 instead of |t| 2^-21: for |t| < 128 it is the wider of the two, and for
//     |t| >= 128 the quotient exceeds 127.5 whenever t does, so both clamp to the same code; written as "not >=", it
//     also sends every NaN to the exact path;
//   * otherwise clamp first (for finite t, rint and the clamp to whole numbers commute), then add 1.5 * 2^23: the sum is
//     rounded to a whole number half-to-even by the addition itself, and the low byte of its bit pattern is the
//     two's-complement code.
__device__ __forceinline__ void quantize_bytes8(const float (&x)[8], float s, float r, unsigned& lo, unsigned& hi) {
  float t[8];
  bool exact_path = false;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    t[j] = x[j] * r;
    exact_path |= !(fabsf(__builtin_amdgcn_fractf(t[j]) - 0.5f) >= 0x1p-14f);
  }
  unsigned b[8];
  if (__builtin_amdgcn_ballot_w64(exact_path) != 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) b[j] = (unsigned)finish_code(x[j], __fdiv_rn(x[j], s));
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) b[j] = __float_as_uint(__builtin_amdgcn_fmed3f(t[j], -127.0f, 127.0f) + 12582912.0f);
  }
  // v_perm_b32: selector bytes 0..3 take bytes of the second operand, 4..7 of the first, 0x0c gives zero
  const unsigned p01 = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u), p23 = __builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u);
  const unsigned p45 = __builtin_amdgcn_perm(b[5], b[4], 0x0c0c0400u), p67 = __builtin_amdgcn_perm(b[7], b[6], 0x0c0c0400u);
  lo = p01 | (p23 << 16);
  hi = p45 | (p67 << 16);
}
__device__ __forceinline__ int quantize_code(float x, float s, float r, float qmax = 127.0f) {
  const float xs[1] = {x};
  int q[1];
  quantize_codes<1>(xs, s, r, q, qmax);
  return q[0];
}
__device__ __forceinline__ float scale_reciprocal(float s) { return __fdiv_rn(1.0f, s); }

// Selection rule inside one group of 4 [Sec. 3.1: two of every four contiguous elements are zero; the rule is this
// library's reading]: element i is kept iff fewer than two elements beat it, where j beats i when |w_j| > |w_i|, or
// |w_j| == |w_i| and j < i.  Magnitudes are compared as sign-cleared bit patterns (a total order).
// Returns the 4-bit keep mask (exactly two bits set).
__device__ __forceinline__ unsigned keep_mask_of_4(unsigned k0, unsigned k1, unsigned k2, unsigned k3) {
  const unsigned r0 = (k1 > k0) + (k2 > k0) + (k3 > k0);
  const unsigned r1 = (k0 >= k1) + (k2 > k1) + (k3 > k1);
  const unsigned r2 = (k0 >= k2) + (k1 >= k2) + (k3 > k2);
  const unsigned r3 = (k0 >= k3) + (k1 >= k3) + (k2 >= k3);
  return (r0 < 2u) | ((r1 < 2u) << 1) | ((r2 < 2u) << 2) | ((r3 < 2u) << 3);
}

// positions of the two set bits of a keep mask, packed as the metadata nibble p0 | p1 << 2 (p0 < p1)
__device__ __forceinline__ unsigned nibble_of_mask(unsigned m) {
  const unsigned p0 = __builtin_ctz(m);
  const unsigned p1 = 31u - __builtin_clz(m);
  return p0 | (p1 << 2);
}

void set_last_hip_error(hipError_t e);

struct GemmArgs {
  const void* X;
  const void* W;  // packed (sparse) or dense [N][K]
  const float* act_scale;
  const float* w_scale;
  const float* bias;
  const float* out_scale;
  void* Y;
  int M, N, K;
  int epilogue;
  int out_dt;
  // Patch-embedding mode (patch_P != 0): X is an image batch [B][C][H][W] and row m = (b, py, px) of the X operand is
  // patch (py, px) of image b, column (c*P + i)*P + j its pixel (py*P + i, px*P + j) of channel c; M = B*(H/P)*(W/P),
  // K = C*P*P.  The tile kernel then fetches its X slabs from the image directly (no flattened-patch buffer).
  int patch_P = 0, patch_C = 0, patch_H = 0, patch_W = 0;
  // INT8 path, small kernel only: X holds fp16 activations, quantised inside the kernel with the static act_scale
  int x_f16 = 0;
};

gpusq_status launch_spgemm(bool is_i8, const GemmArgs& a, hipStream_t s);
gpusq_status launch_dense(bool is_i8, const GemmArgs& a, hipStream_t s);
int forced_kernel();                // -1 when none is forced
int set_forced_kernel(int kernel);  // testing aid, see gpusq_force_kernel; returns the previous value
gpusq_status plan_spgemm(bool is_i8, int64_t M, int64_t N, int64_t K, int epilogue, int cus, int32_t* out);

gpusq_status launch_prune(const void* Win, void* Wout, uint8_t* mask, gpusq_dtype dt, int64_t N, int64_t K, hipStream_t s);
gpusq_status launch_prune_n_of_m(const float* Win, float* Wout, int n_keep, int m, int64_t N, int64_t K, hipStream_t s);
gpusq_status launch_cast_f16(const float* in, void* out, int64_t n, hipStream_t s);
gpusq_status launch_im2col_patches(const void* img, void* X, gpusq_dtype dt, int64_t B, int64_t C, int64_t H, int64_t W, int64_t P,
                                   int64_t K_pad, hipStream_t s);
gpusq_status launch_quantize(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int mode, int scale_is_input,
                             int64_t rows, int64_t cols, void* workspace, hipStream_t s);
gpusq_status launch_quantize_tensor_static(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int scale_is_input,
                                           int64_t rows, int64_t cols, hipStream_t s);
gpusq_status launch_quantize_rows_int4(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int scale_is_input, int64_t rows,
                                       int64_t cols, hipStream_t s);
gpusq_status launch_prune_pairs(const float* Win, float* Wout, uint8_t* mask, int one_per_group, int64_t N, int64_t K, hipStream_t s);
gpusq_status launch_int4_to_sparse_int8(const uint8_t* values4, const uint8_t* meta4, int8_t* values8, uint8_t* meta8,
                                        int32_t* mismatches, int64_t N, int64_t K, hipStream_t s);
gpusq_status launch_compress_int4(const int8_t* W, uint8_t* values, uint8_t* meta, int32_t* violations, int64_t N, int64_t K,
                                  hipStream_t s);
gpusq_status launch_decompress_int4(const uint8_t* values, const uint8_t* meta, int8_t* W, int64_t N, int64_t K, hipStream_t s);
gpusq_status launch_count_violations(const void* W, gpusq_dtype dt, int32_t* violations, int64_t N, int64_t K, hipStream_t s);
gpusq_status launch_compress(const void* W, void* values, uint8_t* meta, int32_t* violations, gpusq_dtype dt,
                             int64_t N, int64_t K, hipStream_t s);
gpusq_status launch_decompress(const void* values, const uint8_t* meta, void* W, gpusq_dtype dt, int64_t N, int64_t K,
                               hipStream_t s);
gpusq_status launch_pack(const void* values, const uint8_t* meta, void* packed, gpusq_dtype dt, int64_t N, int64_t K,
                         hipStream_t s);

gpusq_status launch_prepare_weights(const float* W, gpusq_dtype dt, float* Wp, void* Wlow, float* w_scale, void* values,
                                    uint8_t* meta, void* packed, int64_t N, int64_t K, hipStream_t s);

inline gpusq_status check_launch() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_last_hip_error(e);
    return GPUSQ_ERR_HIP;
  }
  return GPUSQ_OK;
}

}  // namespace gpusq
