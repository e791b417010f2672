// Pieces shared by the tile kernels of the sparse GEMM and of its dense twin: vector types, the matrix-instruction
// wrappers, the tile list of a launch, direct global->LDS copies, and the epilogues that turn a wavefront's accumulators
// (128 channels x 16*TM rows) into rows of Y.
#pragma once
#include "common.h"
#include "epilogue.h"

namespace gpusq {

constexpr int kTileBN = 256;       // output channels of a tile = one packed weight tile
constexpr int kTileTN = 8;         // 16-channel fragments per wavefront: a wavefront spans 128 channels
constexpr int kTileUnitRows = 64;  // tile heights are multiples of 4 wavefronts x 16 rows
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v16h __attribute__((ext_vector_type(16)));

template <bool IS_I8>
struct AccT { typedef v4f type; };
template <>
struct AccT<true> { typedef v4i type; };

template <bool IS_I8>
__device__ __forceinline__ typename AccT<IS_I8>::type smfmac(v4i a, v8i b, typename AccT<IS_I8>::type c, int idx) {
  if constexpr (IS_I8)
    return __builtin_amdgcn_smfmac_i32_16x16x128_i8(a, b, c, idx, 0, 0);
  else
    return __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v16h, b), c, idx, 0, 0);
}

// The list of tiles of one launch.  The first `full_tiles` tiles have 64*full_tm rows (n fastest); the rows behind the
// last of them are cut into tail tiles of 64*tail_tm rows.  The host picks the three numbers so that the workgroup
// with the most work finishes as early as possible (make_plan).
struct TilePlan {
  int tiles_n;      // 256-channel blocks
  int full_tm;      // 1..4
  int full_chunks;  // row chunks covered by full tiles
  int full_tiles;   // = full_chunks * tiles_n
  int tail_tm;      // 1..4
  int total;        // full + tail tiles
  // ceil(2^32 / tiles_n), or 0 when the shortcut below does not apply (tiles_n = 1 or > 4096, or 2^20 tiles or more)
  uint32_t inv_tiles_n;
};

// idx / tiles_n without a division (a tile is decoded three times per tile, between K steps, by every wavefront, and an
// integer division is some thirty scalar instructions): for d <= 4096 and idx < 2^20, mulhi(idx, ceil(2^32 / d)) is the
// exact quotient (the error idx * e / (d * 2^32), e < d, stays below 1 / d).
__host__ __device__ __forceinline__ int div_tiles_n(const TilePlan& p, int idx) {
#if defined(__HIP_DEVICE_COMPILE__)
  return p.inv_tiles_n ? (int)__umulhi((unsigned)idx, p.inv_tiles_n) : idx / p.tiles_n;
#else
  return p.inv_tiles_n ? (int)(((uint64_t)(unsigned)idx * p.inv_tiles_n) >> 32) : idx / p.tiles_n;
#endif
}

struct Tile {
  int n_blk;
  int tm;      // 16-row slabs per wavefront (4 wavefronts along m): the tile has 64*tm rows
  int64_t m0;
};

// Item i of the list of XCD x: the XCD's share of the full tiles (a contiguous run, so tiles that share an X slab
// meet in one L2), then its share of the tail tiles.
__host__ __device__ __forceinline__ int xcd_items(const TilePlan& p, int x, int& f0, int& nf, int& t0) {
  const int tail = p.total - p.full_tiles;
  f0 = (int)((int64_t)x * p.full_tiles / 8);
  nf = (int)((int64_t)(x + 1) * p.full_tiles / 8) - f0;
  t0 = p.full_tiles + (int)((int64_t)x * tail / 8);
  return nf + (int)((int64_t)(x + 1) * tail / 8) - (int)((int64_t)x * tail / 8);
}

__device__ __forceinline__ Tile decode_tile(const TilePlan& p, int idx) {
  Tile t;
  if (idx < p.full_tiles) {
    const int chunk = div_tiles_n(p, idx);
    t.n_blk = idx - chunk * p.tiles_n;
    t.m0 = (int64_t)chunk * kTileUnitRows * p.full_tm;
    t.tm = p.full_tm;
  } else {
    const int j = idx - p.full_tiles;
    const int chunk = div_tiles_n(p, j);
    t.n_blk = j - chunk * p.tiles_n;
    t.m0 = ((int64_t)p.full_chunks * p.full_tm + (int64_t)chunk * p.tail_tm) * kTileUnitRows;
    t.tm = p.tail_tm;
  }
  return t;
}

// Direct global->LDS copies issued through inline assembly: 64 lanes x 16 (4) bytes from `gbase` (wavefront-uniform,
// scalar registers) + `voff` (per lane, unsigned 32 bits) to LDS bytes [lds, lds + 1024 (256)), lane l at lds + 16l
// (4l).  The LDS base travels in M0.  Issued this way the copies are invisible to the compiler's wait-count
// bookkeeping, so the only waits on them are the explicit s_waitcnt instructions of the kernel: the compiler would
// otherwise put a full vmcnt(0) in front of every LDS read that might alias a copy in flight.
__device__ __forceinline__ void copy16_to_lds(const void* gbase, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(gbase) : "memory", "m0");
}
// The same with the LDS address given as a scalar base plus a compile-time constant: one scalar instruction forms M0.
template <int IMM>
__device__ __forceinline__ void copy16_to_lds_at(const void* gbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(gbase), "n"(IMM)
               : "memory", "m0", "scc");
}
__device__ __forceinline__ void copy4_to_lds(const void* gbase, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds), "v"(voff), "s"(gbase) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const uint8_t*)p;
}

// Index words of fragments 4*half .. 4*half+3 of this lane (its 8 words are consecutive at `ibase`).
template <bool IS_I8>
__device__ __forceinline__ void load_index_half(int (&ai)[kTileTN], int half, const uint8_t* ibase) {
  if constexpr (IS_I8) {
    const v4i x = *(const v4i*)(ibase + half * 16);
#pragma unroll
    for (int j = 0; j < 4; ++j) ai[4 * half + j] = x[j];
  } else {
    typedef int v2i __attribute__((ext_vector_type(2)));
    const v2i x = *(const v2i*)(ibase + half * 8);  // 4 x 16 bits
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      ai[4 * half + 2 * j] = x[j] & 0xFFFF;
      ai[4 * half + 2 * j + 1] = (int)((unsigned)x[j] >> 16);
    }
  }
}

// Epilogue of one wavefront of the tile kernel for every output type and any N % 4 == 0: 128 channels x 16*tm_active rows
// of accumulators -> Y in batches of 32 channels x 16 rows (one 16-byte store per lane and batch for fp16 output); same
// lane -> output mapping as wave_epilogue, per-channel constants from the LDS array `p` (128 weight scales, then 128
// biases).
template <bool IS_I8, int GELU, int OUT, int TM>
__device__ __forceinline__ void batch_epilogue(const GemmArgs& a, const typename AccT<IS_I8>::type (&acc)[kTileTN][TM],
                                             const float* p, float s_a, int n_wave, int64_t m_wave, int lane, int tm_active) {
  constexpr bool RAW = IS_I8 && OUT == GPUSQ_I32;
  constexpr int OB = dtype_bytes(OUT);
  asm volatile("" : "+v"(lane));  // see line_epilogue
  uint8_t* yrow[TM];
  bool row_ok[TM];
#pragma unroll
  for (int mt = 0; mt < TM; ++mt) {
    const int64_t m = m_wave + mt * 16 + (lane & 15);
    row_ok[mt] = m < a.M;
    yrow[mt] = (uint8_t*)a.Y + (m * a.N + n_wave + (lane >> 4) * 8) * OB;
  }
#pragma unroll
  for (int g = 0; g < kTileTN / 2; ++g) {
    const int nb = (g >> 1) * kRowBlock + (g & 1) * 32;  // first channel of the batch relative to n_wave (lane group 0)
    const int nl = nb + (lane >> 4) * 8;                 // this lane's first channel
    float c8[8], b8[8];
    if constexpr (!RAW) {
#pragma unroll
      for (int j = 0; j < 8; j += 4) {
        const float4 bb = *(const float4*)(p + 128 + nl + j);
        b8[j] = bb.x; b8[j + 1] = bb.y; b8[j + 2] = bb.z; b8[j + 3] = bb.w;
        if constexpr (IS_I8) {
          const float4 cc = *(const float4*)(p + nl + j);
          c8[j] = s_a * cc.x; c8[j + 1] = s_a * cc.y; c8[j + 2] = s_a * cc.z; c8[j + 3] = s_a * cc.w;
        } else {
          c8[j] = c8[j + 1] = c8[j + 2] = c8[j + 3] = 1.0f;
        }
      }
    }
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      if (mt < tm_active) {
        float v[8];
        int raw[8];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int j = 4 * t + r;
            if constexpr (IS_I8) {
              raw[j] = acc[2 * g + t][mt][r];
              v[j] = RAW ? 0.0f : (float)raw[j];
            } else {
              raw[j] = 0;
              v[j] = acc[2 * g + t][mt][r] + b8[j];
            }
          }
        if constexpr (IS_I8 && !RAW) {
          pin8(v);
#pragma unroll
          for (int j = 0; j < 8; ++j) v[j] = __fmaf_rn(v[j], c8[j], b8[j]);
        }
        if constexpr (GELU != 0) gelu_f32_x8(v);
        if (row_ok[mt]) store_8_at<IS_I8, OUT, true>(a, yrow[mt] + nb * OB, n_wave + nl, v, raw);
      }
    }
  }
}

// Epilogue that writes whole 128-byte lines.  The accumulator layout gives a lane (c = lane % 16, q = lane / 16) 8
// consecutive channels of activation row c of a slab, so a plain store per lane covers 16 rows x 64 bytes (fp16; 32 for
// int8 output): partial lines, which the memory pipeline of a CU accepts at less than a third of the rate of whole
// lines (measured: 23-30 B/ns per CU against 100 B/ns).  Here every lane ends up with two 16-byte pieces, `first` and
// `second`, that lie in the same line of its row, lanes c and c+8 of a 16-lane row swap one of them through DPP
// (row_ror:8), and the first store of the pair covers rows 0..7 of the slab, the second rows 8..15, each lane writing 16
// bytes of a whole line:
//   lanes c < 8 : store 1 = own row, `first` (own)              store 2 = row c+8, `first` (from lane c+8)
//   lanes c >= 8: store 1 = row c-8, `second` (from lane c-8)   store 2 = own row, `second` (own)
// The two pieces and the line they share:
//   fp16  (N % 8 == 0):  two batches of 32 channels are paired (64 consecutive channels = 128 bytes of a row); the
//                        lane's 8 channels of the first batch and of the second.
//   int32 (N % 4 == 0):  one batch of 32 channels is a line; the lane's two accumulator fragments (4 channels each).
//   int8  (N % 16 == 0): the wavefront's 128 channels are a line, of which a lane holds 8 bytes in each of the 4
//                        batches.  Lanes q = 2j and 2j+1 exchange halves with v_permlane16_swap (the odd 16-lane rows of
//                        one register against the even rows of another): the even one then holds 16 consecutive channels
//                        of batches 0 and 1, the odd one those of batches 2 and 3.
// CHECKED = false: the wavefront's 128 channels x 64 rows all lie inside Y (the caller has checked), so the stores carry
// no per-lane tests and no branches.
// `y` is wavefront-uniform (it stays in scalar registers) and `off` the lane's 32-bit byte offset: the stores then take the
// scalar-base addressing form and no lane holds a 64-bit address.
typedef __attribute__((address_space(1))) uint8_t global_u8;
typedef __attribute__((address_space(1))) ep_v4i global_v4i;
__device__ __forceinline__ global_u8* uniform_ptr(const void* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(v >> 32)), lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
  return (global_u8*)(((uint64_t)hi << 32) | lo);  // (the builtin returns a signed int: widened directly it would sign-extend)
}
__device__ __forceinline__ void store_line_pair(const ep_v4i& first, const ep_v4i& second, global_u8* y, uint32_t off, int64_t half_bytes,
                                                bool ok1, bool ok2) {
  ep_v4i s1, s2;
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    // row_ror:8 = 0x128; bank_mask 0xC: lanes 8..15 of a row take the rotated source, 0x3: lanes 0..7
    s1[d] = __builtin_amdgcn_update_dpp(first[d], second[d], 0x128, 0xF, 0xC, false);
    s2[d] = __builtin_amdgcn_update_dpp(second[d], first[d], 0x128, 0xF, 0x3, false);
  }
  // (the empty asm keeps the widening of `off` next to the stores: hoisted out of the tile loop, the widened offset
  // would occupy a register pair and the stores would take 64-bit vector addresses)
  asm volatile("" : "+v"(off));
  if (ok1) __builtin_nontemporal_store(s1, (global_v4i*)(y + off));
  if (ok2) __builtin_nontemporal_store(s2, (global_v4i*)(y + half_bytes + off));
}

template <bool IS_I8, int GELU, int OUT, bool CHECKED, int TM>
__device__ __forceinline__ void line_epilogue(const GemmArgs& a, const typename AccT<IS_I8>::type (&acc)[kTileTN][TM],
                                              const float* p, float s_a, float so, float rso, int n_wave, int64_t m_wave, int lane,
                                              int tm_active) {
  constexpr int OB = dtype_bytes(OUT);
  // (the lane number is laundered through an empty asm: everything derived from it below is then computed here, per
  // tile, instead of once per kernel with the results held in registers, or spilled, across the K loops)
  asm volatile("" : "+v"(lane));
  const int c = lane & 15, q = lane >> 4, up = c >> 3;
  const int64_t slab_bytes = (int64_t)16 * a.N * OB, half_bytes = (int64_t)8 * a.N * OB;
  global_u8* ywave = uniform_ptr((uint8_t*)a.Y + (m_wave * a.N + n_wave) * OB);  // the wavefront's first row and channel
  const uint32_t row_off = (uint32_t)(c & 7) * (uint32_t)a.N * OB;             // row c % 8 (the host keeps 16 rows of Y below 2 GiB)
  // per-channel constants of the lane's 8 channels of batch g (32 channels): read once per batch, used for every slab
  auto batch_constants = [&](int g, float (&c8)[8], float (&b8)[8]) {
    const int nl = (g >> 1) * kRowBlock + (g & 1) * 32 + q * 8;
#pragma unroll
    for (int j = 0; j < 8; j += 4) {
      const float4 bb = *(const float4*)(p + 128 + nl + j);
      b8[j] = bb.x; b8[j + 1] = bb.y; b8[j + 2] = bb.z; b8[j + 3] = bb.w;
      if constexpr (IS_I8) {
        const float4 cc = *(const float4*)(p + nl + j);
        c8[j] = s_a * cc.x; c8[j + 1] = s_a * cc.y; c8[j + 2] = s_a * cc.z; c8[j + 3] = s_a * cc.w;
      } else {
        c8[j] = c8[j + 1] = c8[j + 2] = c8[j + 3] = 1.0f;
      }
    }
    pin8(c8);  // (keeps the products in registers: recomputing them per slab costs an instruction per output)
    pin8(b8);
  };
  // values of those channels in slab mt, dequantised / biased / activated, in fp32
  auto batch_values = [&](int g, int mt, const float (&c8)[8], const float (&b8)[8], float (&v)[8]) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int j = 4 * t + r;
        if constexpr (IS_I8)
          v[j] = (float)acc[2 * g + t][mt][r];
        else
          v[j] = acc[2 * g + t][mt][r] + b8[j];
      }
    if constexpr (IS_I8) {
      pin8(v);
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = __fmaf_rn(v[j], c8[j], b8[j]);
    }
    if constexpr (GELU != 0) gelu_f32_x8(v);
  };
  if constexpr (OUT == GPUSQ_F16) {
#pragma unroll
    for (int gp = 0; gp < kTileTN / 4; ++gp) {
      // the channels this lane stores: those of its own half of the line
      const bool n_ok = n_wave + gp * kRowBlock + up * 32 + q * 8 < a.N;
      float c8[2][8], b8[2][8];
      batch_constants(2 * gp, c8[0], b8[0]);
      batch_constants(2 * gp + 1, c8[1], b8[1]);
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) {
        if (!CHECKED || mt < tm_active) {
          ep_v4i H[2];
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            float v[8];
            batch_values(2 * gp + h, mt, c8[h], b8[h], v);
            pin8(v);  // the fp32 result is rounded to fp32 before it is rounded to fp16 (no fused fma-and-convert)
            ep_v8h hh;
#pragma unroll
            for (int j = 0; j < 8; ++j) hh[j] = (_Float16)v[j];
            H[h] = __builtin_bit_cast(ep_v4i, hh);
          }
          const int64_t row = m_wave + mt * 16 + (c & 7);
          store_line_pair(H[0], H[1], ywave + mt * slab_bytes, row_off + gp * (kRowBlock * 2) + up * 64 + q * 16, half_bytes,
                          !CHECKED || (n_ok && row < a.M), !CHECKED || (n_ok && row + 8 < a.M));
        }
      }
    }
  } else if constexpr (OUT == GPUSQ_I32) {
#pragma unroll
    for (int g = 0; g < kTileTN / 2; ++g) {
      const int nb = (g >> 1) * kRowBlock + (g & 1) * 32 + q * 8 + up * 4;  // first of the 4 channels this lane stores
      const bool n_ok = n_wave + nb < a.N;
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) {
        if (!CHECKED || mt < tm_active) {
          const int64_t row = m_wave + mt * 16 + (c & 7);
          store_line_pair(acc[2 * g][mt], acc[2 * g + 1][mt], ywave + mt * slab_bytes, row_off + nb * 4, half_bytes,
                          !CHECKED || (n_ok && row < a.M), !CHECKED || (n_ok && row + 8 < a.M));
        }
      }
    }
  } else {
    // so, rso: the output scale and its reciprocal (the same code rule as the quantiser of the activations)
    // 16-byte piece (of the 8 in a line) that this lane stores: lanes c < 8 their `first`, lanes c >= 8 the `second`
    // of lane c - 8; even q hold batches 0 (first) and 1 (second), odd q batches 2 and 3, channels 16 * (q / 2) ...
    const int piece = 4 * (q & 1) + 2 * up + (q >> 1);
    const bool n_ok = n_wave + piece * 16 < a.N;
    unsigned d[TM][4][2];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float c8[8], b8[8];
      batch_constants(g, c8, b8);
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) {
        if (!CHECKED || mt < tm_active) {
          float v[8];
          batch_values(g, mt, c8, b8, v);
          quantize_bytes8(v, so, rso, d[mt][g][0], d[mt][g][1]);
        }
      }
    }
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      if (!CHECKED || mt < tm_active) {
        ep_v4i first, second;
#pragma unroll
        for (int w = 0; w < 2; ++w) {
          // result 0: even q keep their own register, odd q receive the second register of lane q - 1;
          // result 1: even q receive the first register of lane q + 1, odd q keep their own second register
          const ep_v2u x = __builtin_amdgcn_permlane16_swap(d[mt][0][w], d[mt][2][w], false, false);
          const ep_v2u y = __builtin_amdgcn_permlane16_swap(d[mt][1][w], d[mt][3][w], false, false);
          first[w] = (int)x[0]; first[2 + w] = (int)x[1];
          second[w] = (int)y[0]; second[2 + w] = (int)y[1];
        }
        const int64_t row = m_wave + mt * 16 + (c & 7);
        store_line_pair(first, second, ywave + mt * slab_bytes, row_off + piece * 16, half_bytes, !CHECKED || (n_ok && row < a.M),
                        !CHECKED || (n_ok && row + 8 < a.M));
      }
    }
  }
}


// ---- the tile kernel with two resident workgroups per CU (tile2.hip), sparse and dense
TilePlan make_tile2_plan(int M, int N, int resident, int ksteps, bool gelu, bool dense);
int tile2_grid_of(const TilePlan& p, int resident);
bool tile2_supports(bool is_i8, bool dense, const GemmArgs& a);
gpusq_status launch_tile2(bool is_i8, bool dense, const GemmArgs& a, const TilePlan& plan, int grid, hipStream_t s);

}  // namespace gpusq
