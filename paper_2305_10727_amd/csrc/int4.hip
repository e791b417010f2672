// INT4 operands in the pair-wise 4:8 pattern [Sec. 3.1, paragraph on the INT4 instruction]: pruning, compressed storage
// (4 kept 4-bit values + two 2-bit indices per chunk of 8) and the decode to INT8 that feeds the multiply-accumulate.
// gfx950 has no 4-bit integer matrix instruction and the pattern is not a 2:4 pattern (both kept sub-chunks of a chunk may
// lie in the same group of 4), so the product itself runs on the dense INT8 kernel over the decoded operand; what the
// format buys on this hardware is the storage: 2.5 bits per weight in HBM and on disk.
// All kernels stream their operands once (HBM-bound); one thread handles two chunks (16 dense elements).
#include "common.h"

namespace gpusq {

// ---------------------------------------------------------------------------------------------------------- prune
// Score of a sub-chunk (a, b): |a| + |b| in fp32, compared as a sign-cleared bit pattern (a total order); the two highest
// scores are kept, ties to the lower index: the rule of the 2:4 pattern applied to the four sub-chunks.
__device__ __forceinline__ unsigned pair_key(float a, float b) { return __float_as_uint(fabsf(a) + fabsf(b)) & 0x7FFFFFFFu; }

// one_per_group: of the two kept sub-chunks one lies in each group of 4 (the better of its two; ties: the lower index),
// which makes the row a 2:4 row as well: the form that the sparse matrix instructions of this hardware can consume.
__global__ void __launch_bounds__(256) prune_pairs_f32_kernel(const float4* __restrict__ in, float4* __restrict__ out,
                                                              uint8_t* __restrict__ mask, int one_per_group, int64_t chunks) {
  const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= chunks) return;
  const float4 lo = in[2 * c], hi = in[2 * c + 1];
  const unsigned k0 = pair_key(lo.x, lo.y), k1 = pair_key(lo.z, lo.w), k2 = pair_key(hi.x, hi.y), k3 = pair_key(hi.z, hi.w);
  const unsigned m = one_per_group ? ((k1 > k0 ? 2u : 1u) | (k3 > k2 ? 8u : 4u)) : keep_mask_of_4(k0, k1, k2, k3);
  float4 o0, o1;
  o0.x = (m & 1u) ? lo.x : 0.0f; o0.y = (m & 1u) ? lo.y : 0.0f;
  o0.z = (m & 2u) ? lo.z : 0.0f; o0.w = (m & 2u) ? lo.w : 0.0f;
  o1.x = (m & 4u) ? hi.x : 0.0f; o1.y = (m & 4u) ? hi.y : 0.0f;
  o1.z = (m & 8u) ? hi.z : 0.0f; o1.w = (m & 8u) ? hi.w : 0.0f;
  out[2 * c] = o0;
  out[2 * c + 1] = o1;
  if (mask) mask[c] = (uint8_t)m;
}

gpusq_status launch_prune_pairs(const float* Win, float* Wout, uint8_t* mask, int one_per_group, int64_t N, int64_t K, hipStream_t s) {
  const int64_t chunks = N * (K / 8);
  prune_pairs_f32_kernel<<<(unsigned)ceil_div(chunks, 256), 256, 0, s>>>((const float4*)Win, (float4*)Wout, mask, one_per_group, chunks);
  return check_launch();
}

// ---------------------------------------------------------------------------------------------------------- compress
// One chunk: 8 codes in two words (little endian) -> 16 bits of values (kept code j in nibble j) + the index nibble.
__device__ __forceinline__ void compress_chunk(unsigned w0, unsigned w1, unsigned& vals16, unsigned& nib, int& bad) {
  int c[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    c[i] = (int)(int8_t)(w0 >> (8 * i));
    c[4 + i] = (int)(int8_t)(w1 >> (8 * i));
  }
  unsigned key[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) key[p] = (unsigned)(abs(c[2 * p]) + abs(c[2 * p + 1]));
  const unsigned m = keep_mask_of_4(key[0], key[1], key[2], key[3]);
  nib = nibble_of_mask(m);
  const unsigned p0 = nib & 3u, p1 = nib >> 2;
  // the two codes of sub-chunk p are bytes 2p, 2p+1 of the 64-bit chunk
  const uint64_t chunk = ((uint64_t)w1 << 32) | w0;
  const unsigned a = (unsigned)(chunk >> (16 * p0)) & 0xFFFFu, b = (unsigned)(chunk >> (16 * p1)) & 0xFFFFu;
  vals16 = (a & 0xFu) | ((a >> 4) & 0xF0u) | ((b & 0xFu) << 8) | (((b >> 8) & 0xFu) << 12);
  int out_of_range = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) out_of_range |= (c[i] < -8) | (c[i] > 7);
  bad += (int)(((m & 1u) == 0 && key[0] != 0) || ((m & 2u) == 0 && key[1] != 0) || ((m & 4u) == 0 && key[2] != 0) ||
               ((m & 8u) == 0 && key[3] != 0) || out_of_range);
}

__global__ void __launch_bounds__(256) compress_int4_kernel(const int8_t* __restrict__ W, uint8_t* __restrict__ values,
                                                            uint8_t* __restrict__ meta, int32_t* __restrict__ violations,
                                                            int64_t N, int64_t K) {
  const int64_t chunks_per_row = K / 8;
  const int64_t mrb = (chunks_per_row + 1) / 2;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int bad = 0;
  if (id < N * mrb) {
    const int64_t n = id / mrb, b = id % mrb;
    unsigned byte = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int64_t c = 2 * b + h;
      if (c < chunks_per_row) {
        const uint2 w = *(const uint2*)(W + n * K + 8 * c);  // rows and chunks are 8-byte aligned (K % 8 == 0)
        unsigned vals16, nib;
        compress_chunk(w.x, w.y, vals16, nib, bad);
        *(uint16_t*)(values + n * (K / 4) + 2 * c) = (uint16_t)vals16;
        byte |= nib << (4 * h);
      }
    }
    meta[n * mrb + b] = (uint8_t)byte;
  }
  if (violations) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) bad += __shfl_xor(bad, o, 64);
    if ((threadIdx.x & 63) == 0 && bad) atomicAdd(violations, bad);
  }
}

__global__ void clear_i32_kernel(int32_t* p) { *p = 0; }

gpusq_status launch_compress_int4(const int8_t* W, uint8_t* values, uint8_t* meta, int32_t* violations, int64_t N, int64_t K,
                                  hipStream_t s) {
  const int64_t mrb = (K / 8 + 1) / 2;
  if (violations) clear_i32_kernel<<<1, 1, 0, s>>>(violations);
  compress_int4_kernel<<<(unsigned)ceil_div(N * mrb, 256), 256, 0, s>>>(W, values, meta, violations, N, K);
  return check_launch();
}

// ---------------------------------------------------------------------------------------------------------- decode
__global__ void __launch_bounds__(256) decompress_int4_kernel(const uint8_t* __restrict__ values, const uint8_t* __restrict__ meta,
                                                              int8_t* __restrict__ W, int64_t N, int64_t K) {
  const int64_t chunks_per_row = K / 8;
  const int64_t mrb = (chunks_per_row + 1) / 2;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= N * mrb) return;
  const int64_t n = id / mrb, b = id % mrb;
  const unsigned byte = meta[n * mrb + b];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int64_t c = 2 * b + h;
    if (c < chunks_per_row) {
      const unsigned nib = (byte >> (4 * h)) & 0xFu;
      const unsigned p0 = nib & 3u, p1 = nib >> 2;
      const unsigned v = *(const uint16_t*)(values + n * (K / 4) + 2 * c);
      // sign-extend the four nibbles to bytes: the two codes of a kept sub-chunk as a 16-bit pair
      auto byte_of = [](unsigned nibble) { return (unsigned)((int)(nibble << 28) >> 28) & 0xFFu; };
      const uint64_t first = byte_of(v & 0xFu) | (byte_of((v >> 4) & 0xFu) << 8);
      const uint64_t second = byte_of((v >> 8) & 0xFu) | (byte_of((v >> 12) & 0xFu) << 8);
      const uint64_t chunk = (first << (16 * p0)) | (second << (16 * p1));
      *(uint2*)(W + n * K + 8 * c) = uint2{(unsigned)chunk, (unsigned)(chunk >> 32)};
    }
  }
}

// ---------------------------------------------------------------------------------------------------------- to 2:4
// INT4 storage -> the INT8 2:4 compressed form (values [N][K/2], one metadata byte per chunk = two groups of 4), for rows
// in which no group of 4 holds two non-zero sub-chunks (what pruning with one_per_group produces).  A group keeps its
// non-zero sub-chunk (the first one if it has none); a group with two non-zero sub-chunks keeps the second and is counted.
__global__ void __launch_bounds__(256) int4_to_sparse_int8_kernel(const uint8_t* __restrict__ values4, const uint8_t* __restrict__ meta4,
                                                                  int8_t* __restrict__ values8, uint8_t* __restrict__ meta8,
                                                                  int32_t* __restrict__ mismatches, int64_t N, int64_t K) {
  const int64_t chunks_per_row = K / 8;
  const int64_t mrb4 = (chunks_per_row + 1) / 2;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int bad = 0;
  if (id < N * chunks_per_row) {
    const int64_t n = id / chunks_per_row, c = id % chunks_per_row;
    const unsigned nib = (meta4[n * mrb4 + (c >> 1)] >> (4 * (c & 1))) & 0xFu;
    const unsigned p0 = nib & 3u, p1 = nib >> 2;
    const unsigned v = *(const uint16_t*)(values4 + n * (K / 4) + 2 * c);
    auto byte_of = [](unsigned nibble) { return (unsigned)((int)(nibble << 28) >> 28) & 0xFFu; };
    const uint64_t first = byte_of(v & 0xFu) | (byte_of((v >> 4) & 0xFu) << 8);
    const uint64_t second = byte_of((v >> 8) & 0xFu) | (byte_of((v >> 12) & 0xFu) << 8);
    const uint64_t chunk = (first << (16 * p0)) | (second << (16 * p1));  // the 8 dense codes, one byte each
    unsigned vals = 0, meta = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const unsigned group = (unsigned)(chunk >> (32 * h));
      const unsigned pair0 = group & 0xFFFFu, pair1 = group >> 16;
      bad += (int)(pair0 != 0 && pair1 != 0);
      const unsigned local = pair1 != 0 ? 1u : 0u;
      vals |= (local ? pair1 : pair0) << (16 * h);
      meta |= ((2 * local) | ((2 * local + 1) << 2)) << (4 * h);
    }
    *(uint32_t*)(values8 + n * (K / 2) + 4 * c) = vals;
    meta8[n * chunks_per_row + c] = (uint8_t)meta;
  }
  if (mismatches) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) bad += __shfl_xor(bad, o, 64);
    if ((threadIdx.x & 63) == 0 && bad) atomicAdd(mismatches, bad);
  }
}

gpusq_status launch_int4_to_sparse_int8(const uint8_t* values4, const uint8_t* meta4, int8_t* values8, uint8_t* meta8,
                                        int32_t* mismatches, int64_t N, int64_t K, hipStream_t s) {
  if (mismatches) clear_i32_kernel<<<1, 1, 0, s>>>(mismatches);
  int4_to_sparse_int8_kernel<<<(unsigned)ceil_div(N * (K / 8), 256), 256, 0, s>>>(values4, meta4, values8, meta8, mismatches, N, K);
  return check_launch();
}

gpusq_status launch_decompress_int4(const uint8_t* values, const uint8_t* meta, int8_t* W, int64_t N, int64_t K, hipStream_t s) {
  const int64_t mrb = (K / 8 + 1) / 2;
  decompress_int4_kernel<<<(unsigned)ceil_div(N * mrb, 256), 256, 0, s>>>(values, meta, W, N, K);
  return check_launch();
}

}  // namespace gpusq
