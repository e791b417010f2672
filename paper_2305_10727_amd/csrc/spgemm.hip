// 2:4 structured-sparse GEMM with fused epilogue on the gfx950 sparse matrix instructions.
//
// Computes Y[m][n] = act( sum over the kept values of W[n][:] times the X[m][k] their metadata selects ) -- the
// sparse x dense -> dense product of Sec. 3.1 / Fig. 1, which equals the dense product on the zero-filled operand.
// The weights are the sparse "A" operand of v_smfmac_* (rows = output channels n), a 16 x 128-byte slab of
// activations is the dense "B" operand (columns = tokens m), so an accumulator tile is 16 n x 16 m and a lane owns
// 4 consecutive n of one m; with the packed row permutation (common.h) a lane owns 16 consecutive n per 64-row block.
//
// Register semantics of the instructions as measured on MI355X with one-hot operands (int8 16x16x128; fp16
// 16x16x64 is the same with "byte" read as "2-byte element pair"):
//   A (4 VGPRs): lane l, byte e -> row l%16, kept value e of the dense K range [32*(l/16), 32*(l/16)+32);
//   idx (1 VGPR): bits 2e..2e+1 of the lane's own register = position of kept value e inside its group of 4
//                 (fp16: 16 bits, the half selected by ABID);
//   B (8 VGPRs): lane l, byte i -> column l%16, K index 64*(i/16) + 16*(l/16) + i%16 (two half-K operands back to back);
//   D (4 VGPRs): lane l, register r -> row 4*(l/16)+r, column l%16.
//
// Two kernels:
//   spgemm_team_kernel  256 n x 128 m tiles, operands brought into LDS by direct global->LDS copies (no staging
//                       registers), one workgroup of two 4-wavefront teams per CU: one team runs the K loop of a tile
//                       while the other runs the epilogue of the previous one.  Needs K*elemsize % 128 == 0.
//   spgemm_small_kernel 64 x 64 / 128 x 128 tiles through registers; any K % 16 == 0; used for small or ragged-K problems.
#include "common.h"
#include "epilogue.h"

namespace gpusq {

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

// XCD-aware tile order: consecutive workgroup ids land on different XCDs (8 of them, each with its own L2), so give
// every XCD one contiguous run of tiles; tiles that share an X slab (same m block) then share an L2.
__device__ __forceinline__ int xcd_tile(int tiles_total) {
  const int per_xcd = (tiles_total + 7) / 8;
  return (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
}

// Epilogue of one wavefront: TN fragments x TM column tiles of accumulators -> Y.
// Lane (q = lane/16, c = lane%16) holds, for 64-row block b and tile mt, the 16 channels
// n = n_wave + 64*b + 16*q + 4*t + r (t = fragment in block, r = register) of activation row m = m_wave + 16*mt + c.
// cs/bs: the workgroup's per-channel constants in LDS, indexed by channel - n_tile (see ChannelParams).
// GELU / OUT: compile-time epilogue choice, or -1 to read it from the arguments.
template <bool IS_I8, int TN, int TM, int GELU = -1, int OUT = -1>
__device__ __forceinline__ void wave_epilogue(const GemmArgs& a, const typename AccT<IS_I8>::type (&acc)[TN][TM],
                                              const float* cs, const float* bs, int n_tile, int n_wave, int64_t m_wave,
                                              int lane, int tm_active = TM) {
  const bool use_gelu = GELU >= 0 ? (GELU != 0) : ((a.epilogue & GPUSQ_EPI_GELU) != 0);
#pragma unroll
  for (int g = 0; g < TN / 2; ++g) {  // pairs of fragments = 32 channels; this lane holds 8 of them
    const int n = n_wave + (g >> 1) * kRowBlock + (g & 1) * 32 + (lane >> 4) * 8;
    float c8[8], b8[8];
#pragma unroll
    for (int j = 0; j < 8; j += 4) {
      const float4 cc = *(const float4*)(cs + (n - n_tile) + j), bb = *(const float4*)(bs + (n - n_tile) + j);
      c8[j] = cc.x; c8[j + 1] = cc.y; c8[j + 2] = cc.z; c8[j + 3] = cc.w;
      b8[j] = bb.x; b8[j + 1] = bb.y; b8[j + 2] = bb.z; b8[j + 3] = bb.w;
    }
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      if (mt >= tm_active) break;
      const int64_t m = m_wave + mt * 16 + (lane & 15);
      float v[8];
      int raw[8];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int j = 4 * t + r;
          if constexpr (IS_I8) {
            raw[j] = acc[2 * g + t][mt][r];
            v[j] = epilogue_value<true>(raw[j], 0.0f, c8[j], b8[j], use_gelu);
          } else {
            raw[j] = 0;
            v[j] = epilogue_value<false>(0, acc[2 * g + t][mt][r], c8[j], b8[j], use_gelu);
          }
        }
      if (m < a.M) store_8<IS_I8, OUT>(a, m, n, v, raw);
    }
  }
}

// ------------------------------------------------------------------------------------------------ large-tile kernel
constexpr int kBigBN = 256, kBigBM = 128, kBigTN = 8, kBigTM = 4;
constexpr int kXStageBytes = kBigBM * kStepBytes;  // 16 KB: 128 rows x 128 bytes, 16-byte chunks XOR-swizzled per row

// The list of tiles of one launch.  The first `full_tiles` tiles are 256 channels x 128 rows (n fastest); the rows that
// are left over after the last whole round of tiles over the resident workgroups are cut into shorter tiles of
// 32*tail_tm rows, so that the last round costs a fraction of a full round instead of a whole one.
struct TilePlan {
  int tiles_n;      // 256-channel blocks
  int full_tiles;   // = full_chunks * tiles_n
  int full_chunks;  // 128-row chunks covered by full tiles
  int tail_tm;      // 1..4: a tail tile has 32*tail_tm rows (slabs per wavefront)
  int total;        // full + tail tiles
};

struct Tile {
  int n_blk;
  int tm;      // 16-row slabs per wavefront (2 wavefronts along m): the tile has 32*tm rows
  int64_t m0;
};

// Item i of the list of XCD x: the XCD's share of the full tiles (a contiguous run, so tiles that share an X slab
// meet in one L2), then its share of the tail tiles.
__device__ __forceinline__ int xcd_items(const TilePlan& p, int x, int& f0, int& nf, int& t0) {
  const int tail = p.total - p.full_tiles;
  f0 = (int)((int64_t)x * p.full_tiles / 8);
  nf = (int)((int64_t)(x + 1) * p.full_tiles / 8) - f0;
  t0 = p.full_tiles + (int)((int64_t)x * tail / 8);
  return nf + (int)((int64_t)(x + 1) * tail / 8) - (int)((int64_t)x * tail / 8);
}

__device__ __forceinline__ Tile decode_tile(const TilePlan& p, int idx) {
  Tile t;
  if (idx < p.full_tiles) {
    t.n_blk = idx % p.tiles_n;
    t.m0 = (int64_t)(idx / p.tiles_n) * kBigBM;
    t.tm = kBigTM;
  } else {
    const int j = idx - p.full_tiles;
    t.n_blk = j % p.tiles_n;
    t.m0 = (int64_t)p.full_chunks * kBigBM + (int64_t)(j / p.tiles_n) * 32 * p.tail_tm;
    t.tm = p.tail_tm;
  }
  return t;
}

// Per-lane byte offsets, relative to the tile's first row, of the four X blocks this wavefront copies per K step:
// block j = wave + 4i holds rows 8j..8j+7; lane l fetches row 8j + l/8, chunk (l%8) ^ ((row >> 1) & 7).  Rows past the
// end of X re-read the last row (their results are never stored).
__device__ __forceinline__ void tile_x_offsets(uint32_t (&xoff)[4], const Tile& t, int M, int64_t k_bytes, int wave, int lane) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 8 * (wave + i * 4) + (lane >> 3);
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    const int64_t last = (int64_t)M - 1 - t.m0;  // >= 0: a tile starts inside X
    const int64_t rr = r < last ? r : last;
    xoff[i] = (uint32_t)(rr * k_bytes + c * 16);
  }
}

// ------------------------------------------------------------------------------------------------ two-team kernel
// Direct global->LDS copies issued through inline assembly: 64 lanes x 16 (4) bytes from `gbase` (wavefront-uniform,
// scalar registers) + `voff` (per lane, unsigned 32 bits) to LDS bytes [lds, lds + 1024 (256)), lane l at lds + 16l
// (4l).  The LDS base travels in M0.  Issued this way the copies are invisible to the compiler's wait-count
// bookkeeping, so the only waits on them are the explicit s_waitcnt instructions of the kernel: the compiler would
// otherwise put a full vmcnt(0) in front of every LDS read that might alias a copy in flight.
__device__ __forceinline__ void copy16_to_lds(const void* gbase, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(gbase) : "memory", "m0");
}
__device__ __forceinline__ void copy4_to_lds(const void* gbase, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds), "v"(voff), "s"(gbase) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const uint8_t*)p;
}

constexpr int kRing = 4;            // LDS stages: the K step being read plus three requested ahead
constexpr int kCopiesPerStep = 9;   // copy instructions every wavefront of the computing team issues per K step

// Copy i (0..8) of one wavefront's share (a quarter) of the copies that bring one K step of a tile into the LDS
// stage at `stage_lds`: i = 0..3 are 1 KB blocks of the X slab (block j = w + 4i holds rows 8j..8j+7), i = 4..7
// fragments of kept values, i = 8 1 KB of index words.  Each copy moves 64 lanes x 16 bytes from a wavefront-uniform
// 64-bit base (scalar registers, advanced per K step by scalar adds) plus a 32-bit per-lane offset to 1 KB of
// consecutive LDS, so a K step costs no vector ALU work for addressing.  The X slab is stored row-major with the
// 16-byte chunk c of row r at chunk position c ^ ((r >> 1) & 7), so that the 16 rows a quarter-wavefront reads at the
// same K offset fall in 16 different 16-byte bank groups; the swizzle is applied by choosing which global chunk each
// lane fetches (tile_x_offsets).  Always
// exactly kCopiesPerStep instructions per step, whatever the tile: a short tail tile copies rows it does not use, and
// on the fp16 path (2 KB of index words) wavefronts 2 and 3 repeat the copies of wavefronts 0 and 1, so that the
// waits can count instructions.
template <bool IS_I8>
__device__ __forceinline__ void issue_step_copy(int i, uint32_t stage_lds, const uint8_t* Xks, const uint8_t* Wks,
                                                const uint32_t (&xoff)[4], int w, uint32_t loff) {
  if (i < 4) {
    copy16_to_lds(Xks, xoff[i], stage_lds + (uint32_t)(w + 4 * i) * 1024u);
  } else if (i < 8) {
    const int f = w + 4 * (i - 4);
    copy16_to_lds(Wks + f * kFragValueBytes, loff, stage_lds + kXStageBytes + (uint32_t)f * kFragValueBytes);
  } else {
    const int iw = IS_I8 ? w : (w & 1);
    copy16_to_lds(Wks + kTileValueBytes + iw * 1024, loff, stage_lds + kXStageBytes + kTileValueBytes + (uint32_t)iw * 1024u);
  }
}

// s_waitcnt immediates (gfx9 encoding: vmcnt [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8])
constexpr int kWaitVm0 = 0x0F70;         // vmcnt(0)
constexpr int kWaitVm0Lgkm0 = 0x0070;    // vmcnt(0) lgkmcnt(0)
constexpr int kWaitVm9Lgkm0 = 0x0079;    // vmcnt(kCopiesPerStep) lgkmcnt(0)
static_assert(kCopiesPerStep == 9, "kWaitVm9Lgkm0 encodes one K step of copies");

// Workgroup-wide barrier preceded by a scheduling barrier (the compiler must not move it above the matrix
// instructions of the K step) and followed by a compiler-level memory barrier (no LDS read moves above it).
#define GPUSQ_TEAM_BARRIER()              \
  do {                                    \
    __builtin_amdgcn_sched_barrier(0);    \
    __builtin_amdgcn_s_barrier();         \
    asm volatile("" ::: "memory");        \
  } while (0)

// Per-lane byte offsets of the B operand inside an X slab: lane l reads row wm*16*tm + 16*mt + l%16, the 16-byte
// chunks l/16 and 4 + l/16 of it (at their swizzled positions).
struct BOffsets {
  uint32_t lo, hi;
};
__device__ __forceinline__ BOffsets b_offsets(int wm, int tm, int lane) {
  const int sw = (lane & 15) >> 1, q = lane >> 4;
  const uint32_t row = (uint32_t)(wm * tm * 16 + (lane & 15)) * kStepBytes;
  return BOffsets{row + (uint32_t)((q ^ sw) * 16), row + (uint32_t)(((4 + q) ^ sw) * 16)};
}

// The four B slabs of one K step, from the X slab at `xslab`, into registers.
__device__ __forceinline__ void load_b_slabs(v8i (&b)[kBigTM], const uint8_t* xslab, const BOffsets& o) {
#pragma unroll
  for (int mt = 0; mt < kBigTM; ++mt) {
    const v4i lo = *(const v4i*)(xslab + o.lo + mt * 16 * kStepBytes), hi = *(const v4i*)(xslab + o.hi + mt * 16 * kStepBytes);
    b[mt] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  }
}

// Index words of fragments 4*half .. 4*half+3 of this lane (its 8 words are consecutive at `ibase`).
template <bool IS_I8>
__device__ __forceinline__ void load_index_half(int (&ai)[kBigTN], int half, const uint8_t* ibase) {
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

// What a computing wavefront holds in registers when a K step begins: the four B slabs of the step, its A fragments
// 0..2 (fragment f lives in av[f % 4]) and the index words of fragments 0..3.
template <bool IS_I8>
__device__ __forceinline__ void load_step_head(v8i (&b)[kBigTM], v4i (&av)[4], int (&ai)[kBigTN], const uint8_t* stage,
                                               const BOffsets& bo, uint32_t a_off, uint32_t i_off) {
  load_b_slabs(b, stage, bo);
  load_index_half<IS_I8>(ai, 0, stage + kXStageBytes + i_off);
#pragma unroll
  for (int f = 0; f < 3; ++f) av[f] = *(const v4i*)(stage + kXStageBytes + a_off + f * kFragValueBytes);
}

// One K step of a computing wavefront (128 n x 64 m), software-pipelined by hand across steps.  When the step
// begins its B operand (`b`), its A fragments 0..2 and the index words of fragments 0..3 are already in registers.
// Per fragment the step issues: the LDS read of the fragment three ahead -- which for the last three fragments is
// fragment 0..2 of the NEXT step, read from `next` --, one 16-byte piece of the next step's B operand (`bn`), the
// index words it will need four fragments later, and then the four matrix instructions of the fragment.  So the
// matrix pipe never waits for a step to "start": LDS latency is always covered by 12 matrix instructions, also across
// the barrier between two steps.  (`next` = the stage of the next step of the same tile; after the last step of a
// tile the reads ahead go to `stage` again and are discarded.)
// The wavefront's kCopiesPerStep copy requests are spread over the step, one per fragment.
template <bool IS_I8>
__device__ __forceinline__ void team_step(const uint8_t* stage, const uint8_t* next, const BOffsets& bo,
                                          typename AccT<IS_I8>::type (&acc)[kBigTN][kBigTM], const v8i (&b)[kBigTM],
                                          v8i (&bn)[kBigTM], v4i (&av)[4], int (&ai)[kBigTN], uint32_t a_off, uint32_t i_off,
                                          bool requested, uint32_t req_lds, const uint8_t* req_x, const uint8_t* req_w,
                                          const uint32_t (&xoff)[4], int w, uint32_t loff) {
  const uint8_t* abase = stage + kXStageBytes + a_off;
  const uint8_t* ibase = stage + kXStageBytes + i_off;
  const uint8_t* abase_n = next + kXStageBytes + a_off;
  const uint8_t* ibase_n = next + kXStageBytes + i_off;
  // One matrix instruction per slot; in front of each, at most one LDS read and one copy request, so that every other
  // instruction is issued in the shadow of a matrix instruction (a wavefront issues in order: a clump of reads and
  // copies between two groups of matrix instructions would leave the matrix pipe idle for its whole length).
#pragma unroll
  for (int tn = 0; tn < kBigTN; ++tn) {
#pragma unroll
    for (int mt = 0; mt < kBigTM; ++mt) {
      if (mt == 0) {
        const int f = tn + 3;
        av[f & 3] = f < kBigTN ? *(const v4i*)(abase + f * kFragValueBytes) : *(const v4i*)(abase_n + (f - kBigTN) * kFragValueBytes);
      }
      if (mt == 1) {
        const v4i piece = *(const v4i*)(next + ((tn & 1) ? bo.hi : bo.lo) + (tn >> 1) * 16 * kStepBytes);
#pragma unroll
        for (int j = 0; j < 4; ++j) bn[tn >> 1][4 * (tn & 1) + j] = piece[j];
      }
      if (mt == 2 && tn == 0) load_index_half<IS_I8>(ai, 1, ibase);
      if (mt == 2 && tn == 4) load_index_half<IS_I8>(ai, 0, ibase_n);
      if (requested) {
        if (mt == 3) issue_step_copy<IS_I8>(tn, req_lds, req_x, req_w, xoff, w, loff);
        if (mt == 2 && tn == kBigTN - 1) issue_step_copy<IS_I8>(kBigTN, req_lds, req_x, req_w, xoff, w, loff);
      }
      __builtin_amdgcn_sched_barrier(0);
      acc[tn][mt] = smfmac<IS_I8>(av[tn & 3], b[mt], acc[tn][mt], ai[tn]);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
}

// Epilogue of one wavefront of the team that is not computing: same lane -> output mapping as wave_epilogue, with
//  * the per-channel constants read from the wavefront's own LDS array `p` (128 weight scales, then 128 biases),
//  * `ksteps` workgroup barriers spread evenly over the 16 batches of 8 outputs per lane, so that this team stays in
//    step with the K steps of the team that is computing (both execute the same number of barriers per phase),
//  * a wait for the wavefront's own outstanding copies (requested for the other team's tile) after the first batch of
//    arithmetic and before the first store and the first barrier: from then on this wavefront has stores in flight
//    and never waits on the vector-memory counter again until its next compute phase,
//  * `before_last_barrier()` called once, after the last batch and before the last barrier of the phase: the caller
//    sets up the wavefront's next tile there (the accumulators are free by then).
template <bool IS_I8, int GELU, int OUT, class Hook>
__device__ __forceinline__ void team_epilogue(const GemmArgs& a, const typename AccT<IS_I8>::type (&acc)[kBigTN][kBigTM],
                                              const float* p, float s_a, int n_wave, int64_t m_wave, int lane, int tm_active,
                                              int ksteps, Hook&& before_last_barrier) {
  constexpr bool RAW = IS_I8 && OUT == GPUSQ_I32;
  constexpr int OB = dtype_bytes(OUT);
  // address of this lane's first 8 channels in each of its 4 rows, computed once: a batch then only adds a constant
  uint8_t* yrow[kBigTM];
  bool row_ok[kBigTM];
#pragma unroll
  for (int mt = 0; mt < kBigTM; ++mt) {
    const int64_t m = m_wave + mt * 16 + (lane & 15);
    row_ok[mt] = m < a.M;
    yrow[mt] = (uint8_t*)a.Y + (m * a.N + n_wave + (lane >> 4) * 8) * OB;
  }
  int done = 0;
#pragma unroll
  for (int g = 0; g < kBigTN / 2; ++g) {
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
    for (int mt = 0; mt < kBigTM; ++mt) {
      const int batch = g * kBigTM + mt;
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
        if (batch == 0) {
          __builtin_amdgcn_sched_barrier(0);
          __builtin_amdgcn_s_waitcnt(kWaitVm0);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (row_ok[mt]) store_8_at<IS_I8, OUT, true>(a, yrow[mt] + nb * OB, n_wave + nl, v, raw);
      }
      const int target = ((batch + 1) * ksteps) >> 4;
      while (done < target) {
        // the phase's last barrier always falls after the last batch: (15 * ksteps) >> 4 < ksteps
        if (batch == 4 * kBigTM - 1 && done == ksteps - 1) before_last_barrier();
        GPUSQ_TEAM_BARRIER();
        ++done;
      }
    }
  }
}

// Workgroup = 8 wavefronts = two teams of 4 (2 along n x 2 along m, 128 channels x 64 rows and 128 accumulator
// registers each), one workgroup per CU (the LDS footprint, 4 stages of 36 KB, allows no more); wavefronts 0-3 and 4-7 land on the four SIMDs once each, so every SIMD hosts one
// wavefront of each team.  The workgroup walks over its tiles; team (i mod 2) computes tile i.  Time is cut into
// phases of `ksteps` workgroup barriers: in phase i one team runs the K loop of tile i (matrix instructions, LDS
// reads, copy requests) while the other runs the epilogue of tile i-1 (vector ALU, stores), then they swap.  The
// epilogue's arithmetic and the output stores therefore always overlap matrix work on the same SIMD, the computing
// team has all four LDS stages (copies run three K steps ahead, across tile boundaries), and because loads and stores
// are issued by different wavefronts in any phase, waiting for copies never means waiting for stores.
//
// Copy protocol.  K steps are numbered g = 0, 1, ... over the whole sequence of tiles; step g lives in stage g mod 4.
// The wavefronts of the team that computes step g request step g+3 during step g (stage (g+3) mod 4 was last read in
// step g-1, which every wavefront left through a barrier after its LDS reads had returned), then wait until at most
// the copies just requested are outstanding (vmcnt counts instructions, and every wavefront issues kCopiesPerStep
// per step), then meet at the barrier.  Invariant: at the barrier that ends step g the data of all steps <= g+2 has
// landed -- step g+2 was requested during step g-1, either by this team (covered by its wait) or, when g is the
// first step of a tile, by the other team, which waits for all its copies before the first barrier of its epilogue
// phase (see team_epilogue).  When nothing is requested in a step (the end of the sequence) the wait is for all
// copies.  So during step g a wavefront may read stage g and stage g+1 (what it reads ahead for the next step), and a
// wavefront of the epilogue team may read the stage of the first step of its next tile before the last barrier of
// its phase (set_up_tile).
// Every wavefront executes exactly 1 + (tiles + 1) * ksteps barriers.
template <bool IS_I8, int GELU, int OUT>
__global__ void __launch_bounds__(512, 1) spgemm_team_kernel(const GemmArgs a, const TilePlan plan) {
  typedef typename AccT<IS_I8>::type acc_t;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int STAGE = kXStageBytes + tile_bytes(IS_I8);
  constexpr bool RAW = IS_I8 && OUT == GPUSQ_I32;
  __shared__ __attribute__((aligned(1024))) uint8_t ring[kRing * STAGE];
  __shared__ __attribute__((aligned(1024))) float prm[8][256];  // per wavefront: 128 weight scales, 128 biases

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int team = wave >> 2, w = wave & 3, wn = w & 1, wm = w >> 1;
  const int64_t k_bytes = (int64_t)a.K * ES;
  const int ksteps = (int)(k_bytes / kStepBytes);
  const uint8_t* Xg = (const uint8_t*)a.X;
  const uint8_t* Wg = (const uint8_t*)a.W;
  const int64_t w_col_bytes = (int64_t)ksteps * tile_bytes(IS_I8);
  const int xcd = (int)(blockIdx.x & 7), wgs_per_xcd = (int)(gridDim.x >> 3), wl = (int)(blockIdx.x >> 3);
  int f0, nf, t0;
  const int items = xcd_items(plan, xcd, f0, nf, t0);
  const int my_items = wl < items ? (items - wl + wgs_per_xcd - 1) / wgs_per_xcd : 0;
  if (my_items == 0) return;  // the whole workgroup leaves before any barrier
  auto tile_of = [&](int i) {
    const int it = wl + i * wgs_per_xcd;
    return decode_tile(plan, it < nf ? f0 + it : t0 + it - nf);
  };
  const bool has_bias = !RAW && (a.epilogue & GPUSQ_EPI_BIAS) != 0;
  const float s_a = (IS_I8 && !RAW) ? a.act_scale[0] : 1.0f;
  float* my_prm = prm[wave];
  if (!has_bias) {  // the bias half stays zero for the whole launch
    my_prm[128 + lane] = 0.0f;
    my_prm[192 + lane] = 0.0f;
  }
  const uint32_t ring_lds = lds_address(ring), prm_lds = lds_address(my_prm);
  const uint32_t loff = (uint32_t)lane * 16u;
  const uint32_t a_off = (uint32_t)(wn * kBigTN * kFragValueBytes + lane * 16);
  const uint32_t i_off = (uint32_t)index_offset(IS_I8, wn * kBigTN, lane);

  // cursor of the copy requests: the next K step to request, as (tile, step), with its source addresses
  int pf_item = 0, pf_ks = 0;
  const uint8_t *pf_x = Xg, *pf_w = Wg;
  uint32_t pf_xoff[4] = {0, 0, 0, 0};
  auto seek = [&](int item, int ks) {
    while (ks >= ksteps) {
      ks -= ksteps;
      ++item;
    }
    pf_item = item;
    pf_ks = ks;
    if (item < my_items) {
      const Tile t = tile_of(item);
      tile_x_offsets(pf_xoff, t, a.M, k_bytes, w, lane);
      pf_x = Xg + t.m0 * k_bytes + (int64_t)ks * kStepBytes;
      pf_w = Wg + t.n_blk * w_col_bytes + (int64_t)ks * tile_bytes(IS_I8);
    }
  };
  auto advance = [&]() {
    ++pf_ks;
    pf_x += kStepBytes;
    pf_w += tile_bytes(IS_I8);
    if (pf_ks == ksteps) seek(pf_item + 1, 0);
  };

  // state of a wavefront across its compute and epilogue phases
  acc_t acc[kBigTN][kBigTM];
  v8i b0[kBigTM], b1[kBigTM];  // B operands of the current and the next K step (roles alternate)
  v4i av[4];                   // A fragments in flight
  int ai[kBigTN];              // index words
  Tile t = tile_of(0);
  BOffsets bo = b_offsets(wm, t.tm, lane);
  // Everything a wavefront can do for its tile `item` before the phase in which it computes it: called after the
  // barrier that ends the second-to-last step of the previous phase (the tile's first stage has landed by then) and
  // before the last barrier of that phase.
  auto set_up_tile = [&](int item) {
    t = tile_of(item);
    bo = b_offsets(wm, t.tm, lane);
#pragma unroll
    for (int i = 0; i < kBigTN; ++i)
#pragma unroll
      for (int j = 0; j < kBigTM; ++j) acc[i][j] = acc_t{0, 0, 0, 0};
    seek(item, kRing - 1);
    if constexpr (!RAW) {  // this wavefront's 128 channels of epilogue constants, into its own LDS array
      const int n0 = t.n_blk * kBigBN + wn * (kBigTN * 16);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        int n = n0 + i * 64 + lane;
        n = n < a.N ? n : a.N - 1;  // channels past the end are never stored
        if constexpr (IS_I8) copy4_to_lds(a.w_scale, (uint32_t)n * 4u, prm_lds + (uint32_t)i * 256u);
        if (has_bias) copy4_to_lds(a.bias, (uint32_t)n * 4u, prm_lds + 512u + (uint32_t)i * 256u);
      }
    }
    load_step_head<IS_I8>(b0, av, ai, ring + (size_t)((item * ksteps) & (kRing - 1)) * STAGE, bo, a_off, i_off);
  };

  if (team == 0) {  // the first three K steps of the sequence
    seek(0, 0);
    int n_req = 0;
    for (int g = 0; g < kRing - 1; ++g) {
      if (pf_item < my_items) {
#pragma unroll
        for (int i = 0; i < kCopiesPerStep; ++i)
          issue_step_copy<IS_I8>(i, ring_lds + (uint32_t)g * STAGE, pf_x, pf_w, pf_xoff, w, loff);
        advance();
        ++n_req;
      }
    }
    if (n_req == kRing - 1)
      __builtin_amdgcn_s_waitcnt(kWaitVm9Lgkm0);  // steps 0 and 1 have landed
    else
      __builtin_amdgcn_s_waitcnt(kWaitVm0Lgkm0);
  }
  GPUSQ_TEAM_BARRIER();

  int ph = 0;
  if (team == 0) {
    set_up_tile(0);
  } else {  // phase 0: the second team only gets ready for its first tile
    for (int k = 0; k < ksteps; ++k) {
      if (k == ksteps - 1 && my_items > 1) set_up_tile(1);
      GPUSQ_TEAM_BARRIER();
    }
    ph = 1;
  }
  while (ph <= my_items) {
    // ---- compute phase ph --------------------------------------------------------------------------------------
    if (ph >= my_items) {  // one phase after the last tile: only the other team's last epilogue runs
      for (int k = 0; k < ksteps; ++k) GPUSQ_TEAM_BARRIER();
      break;
    }
    const int g0 = ph * ksteps;
    auto step = [&](int ks, const v8i (&b)[kBigTM], v8i (&bn)[kBigTM]) {
      const int g = g0 + ks;
      const bool requested = pf_item < my_items;
      const uint8_t* stage = ring + (size_t)(g & (kRing - 1)) * STAGE;
      const uint8_t* next = ks + 1 < ksteps ? ring + (size_t)((g + 1) & (kRing - 1)) * STAGE : stage;
      team_step<IS_I8>(stage, next, bo, acc, b, bn, av, ai, a_off, i_off, requested,
                       ring_lds + (uint32_t)((g + kRing - 1) & (kRing - 1)) * STAGE, pf_x, pf_w, pf_xoff, w, loff);
      __builtin_amdgcn_sched_barrier(0);
      if (requested) {
        __builtin_amdgcn_s_waitcnt(kWaitVm9Lgkm0);
        advance();
      } else {
        __builtin_amdgcn_s_waitcnt(kWaitVm0Lgkm0);
      }
      GPUSQ_TEAM_BARRIER();
    };
    for (int ks = 0; ks < ksteps; ks += 2) {
      step(ks, b0, b1);
      if (ks + 1 < ksteps) step(ks + 1, b1, b0);
    }
    ++ph;
    // ---- epilogue phase ph: tile ph-1; at its end, get ready for tile ph+1 -------------------------------------------
    const int next_item = ph + 1;
    team_epilogue<IS_I8, GELU, OUT>(a, acc, my_prm, s_a, t.n_blk * kBigBN + wn * (kBigTN * 16), t.m0 + wm * t.tm * 16, lane, t.tm,
                                    ksteps, [&]() {
                                      if (next_item < my_items) set_up_tile(next_item);
                                    });
    ++ph;
  }
}

// ------------------------------------------------------------------------------------------------ small / generic kernel
constexpr int kLdsRow = kStepBytes + 16;  // 144-byte row pitch: 16 rows x 16-byte reads hit 16 distinct bank groups

// Workgroup = 4 wavefronts arranged WN (along n) x WM (along m); a wavefront owns TN x TM accumulator tiles.
// Workgroup tile: BN = WN*TN*16 output channels x BM = WM*TM*16 activation rows.  X goes global -> registers -> LDS
// (zero-filled past the row end and past M), the weight fragments go straight from global memory to registers.
template <bool IS_I8, int TN, int TM, int WN, int WM>
__global__ void __launch_bounds__(256) spgemm_small_kernel(const GemmArgs a, const int tiles_n, const int tiles_total) {
  static_assert(WN * WM == 4 && TN % 4 == 0, "4 wavefronts; a wavefront spans whole 64-row blocks");
  typedef typename AccT<IS_I8>::type acc_t;
  constexpr int BN = WN * TN * 16, BM = WM * TM * 16;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int XCH = BM / 32;  // 16-byte chunks of the X slab each thread moves per K step

  __shared__ __attribute__((aligned(16))) uint8_t Xs[2][BM * kLdsRow];
  __shared__ __attribute__((aligned(16))) float cs[BN];
  __shared__ __attribute__((aligned(16))) float bs[BN];

  const int tile = xcd_tile(tiles_total);
  if (tile >= tiles_total) return;
  const int n_blk = tile % tiles_n, m_blk = tile / tiles_n;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % WN, wm = wave / WN;
  const int M = a.M, N = a.N;
  if (tid < BN) {
    ChannelParams prm;
    prm.fetch<IS_I8>(a, n_blk * BN + tid);
    prm.publish(cs, bs, tid);  // made visible by the barriers of the main loop
  }
  const int64_t k_bytes = (int64_t)a.K * ES;
  const int ksteps = (int)((k_bytes + kStepBytes - 1) / kStepBytes);
  const int row_blocks = ((N + kTileRows - 1) / kTileRows) * 4;  // the packed buffer is padded to whole 256-row tiles
  const int rb0 = (n_blk * BN + wn * TN * 16) / kRowBlock;
  const uint8_t* Xg = (const uint8_t*)a.X;
  const uint8_t* Wg = (const uint8_t*)a.W;

  acc_t acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j) acc[i][j] = acc_t{0, 0, 0, 0};

  v4i xr[XCH];
  v4i av[2][TN];
  int ai[2][TN];

  auto load_x = [&](int ks) {
#pragma unroll
    for (int j = 0; j < XCH; ++j) {
      const int c = tid + 256 * j;
      const int row = c >> 3, cc = c & 7;
      const int64_t m = (int64_t)m_blk * BM + row;
      const int64_t off = (int64_t)ks * kStepBytes + cc * 16;
      xr[j] = (m < M && off < k_bytes) ? *(const v4i*)(Xg + m * k_bytes + off) : v4i{0, 0, 0, 0};
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int j = 0; j < XCH; ++j) {
      const int c = tid + 256 * j;
      *(v4i*)(&Xs[buf][(c >> 3) * kLdsRow + (c & 7) * 16]) = xr[j];
    }
  };
  auto load_a = [&](int ks, int slot) {
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
      const int rb = rb0 + tn / 4;
      if (rb < row_blocks) {
        const uint8_t* t = Wg + ((int64_t)(rb >> 2) * ksteps + ks) * tile_bytes(IS_I8);
        const int f = (rb & 3) * 4 + (tn & 3);
        av[slot][tn] = *(const v4i*)(t + f * kFragValueBytes + lane * 16);
        if constexpr (IS_I8)
          ai[slot][tn] = *(const int*)(t + index_offset(true, f, lane));
        else
          ai[slot][tn] = (int)*(const uint16_t*)(t + index_offset(false, f, lane));
      } else {
        av[slot][tn] = v4i{0, 0, 0, 0};
        ai[slot][tn] = 0;
      }
    }
  };

  load_x(0);
  load_a(0, 0);
  store_x(0);
  __syncthreads();

  const int b_row = wm * TM * 16 + (lane & 15);
  const int b_col = (lane >> 4) * 16;
  for (int ks = 0; ks < ksteps; ++ks) {
    const int cur = ks & 1;
    const bool more = ks + 1 < ksteps;
    if (more) {
      load_x(ks + 1);
      load_a(ks + 1, cur ^ 1);
    }
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      const uint8_t* p = &Xs[cur][(b_row + mt * 16) * kLdsRow + b_col];
      const v4i lo = *(const v4i*)p, hi = *(const v4i*)(p + 64);
      const v8i b = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) acc[tn][mt] = smfmac<IS_I8>(av[cur][tn], b, acc[tn][mt], ai[cur][tn]);
    }
    if (more) store_x(cur ^ 1);
    __syncthreads();
  }
  wave_epilogue<IS_I8, TN, TM>(a, acc, cs, bs, n_blk * BN, n_blk * BN + wn * TN * 16, (int64_t)m_blk * BM + wm * TM * 16, lane);
}

template <bool IS_I8, int TN, int TM, int WN, int WM>
static gpusq_status launch_small(const GemmArgs& a, hipStream_t s) {
  constexpr int BN = WN * TN * 16, BM = WM * TM * 16;
  const int tiles_n = (int)ceil_div(a.N, BN), tiles_m = (int)ceil_div(a.M, BM);
  const int total = tiles_n * tiles_m;
  const int grid = (int)ceil_div(total, 8) * 8;  // whole rounds over the 8 XCDs; surplus workgroups exit at once
  spgemm_small_kernel<IS_I8, TN, TM, WN, WM><<<grid, 256, 0, s>>>(a, tiles_n, total);
  return check_launch();
}

static int num_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cus = n;
  }
  return cus;
}

// Full 128-row tiles for as many whole rounds over the resident workgroups as the problem has; the remaining rows in
// shorter tiles, as tall as still fits them in one more round.
static TilePlan make_plan(int M, int N, int resident) {
  TilePlan p;
  p.tiles_n = (int)ceil_div(N, kBigBN);
  const int chunks = (int)ceil_div(M, kBigBM);
  const int all_tiles = chunks * p.tiles_n;
  int full_chunks = chunks;
  if (all_tiles > resident && all_tiles % resident != 0) full_chunks = (all_tiles / resident) * resident / p.tiles_n;
  p.full_chunks = full_chunks;
  p.full_tiles = full_chunks * p.tiles_n;
  const int64_t rows_left = (int64_t)M - (int64_t)full_chunks * kBigBM;
  p.tail_tm = kBigTM;
  int tail_tiles = 0;
  if (rows_left > 0) {
    for (int tm = kBigTM; tm >= 1; --tm) {
      p.tail_tm = tm;
      tail_tiles = (int)ceil_div(rows_left, 32 * tm) * p.tiles_n;
      if (tm > 1 && (int)ceil_div(rows_left, 32 * (tm - 1)) * p.tiles_n > resident) break;  // a shorter tile would need a second round
    }
  }
  p.total = p.full_tiles + tail_tiles;
  return p;
}

template <bool IS_I8>
static gpusq_status launch_typed(const GemmArgs& a, hipStream_t s) {
  const int64_t work = (int64_t)a.M * a.N;
  const int64_t k_bytes = (int64_t)a.K * (IS_I8 ? 1 : 2);
  if (work <= (int64_t)256 * 1024) return launch_small<IS_I8, 4, 1, 1, 4>(a, s);  // 64 x 64 tiles: latency-bound sizes
  if (k_bytes % kStepBytes != 0) return launch_small<IS_I8, 4, 4, 2, 2>(a, s);    // ragged K: zero-filling path
  const bool gelu = (a.epilogue & GPUSQ_EPI_GELU) != 0;
  {
    // persistent grid: one workgroup of two teams per CU, never more workgroups than tiles
    const int resident = num_cus();
    const TilePlan plan = make_plan(a.M, a.N, resident);
    const dim3 grid((unsigned)(ceil_div(plan.total < resident ? plan.total : resident, 8) * 8));
    if ((ceil_div(plan.total, grid.x) + 2) * (k_bytes / kStepBytes) >= ((int64_t)1 << 30)) return GPUSQ_ERR_UNSUPPORTED;
    if constexpr (IS_I8) {
      if (a.out_dt == GPUSQ_I32)
        spgemm_team_kernel<true, 0, GPUSQ_I32><<<grid, 512, 0, s>>>(a, plan);
      else if (a.out_dt == GPUSQ_I8 && gelu)
        spgemm_team_kernel<true, 1, GPUSQ_I8><<<grid, 512, 0, s>>>(a, plan);
      else if (a.out_dt == GPUSQ_I8)
        spgemm_team_kernel<true, 0, GPUSQ_I8><<<grid, 512, 0, s>>>(a, plan);
      else if (gelu)
        spgemm_team_kernel<true, 1, GPUSQ_F16><<<grid, 512, 0, s>>>(a, plan);
      else
        spgemm_team_kernel<true, 0, GPUSQ_F16><<<grid, 512, 0, s>>>(a, plan);
    } else {
      if (gelu)
        spgemm_team_kernel<false, 1, GPUSQ_F16><<<grid, 512, 0, s>>>(a, plan);
      else
        spgemm_team_kernel<false, 0, GPUSQ_F16><<<grid, 512, 0, s>>>(a, plan);
    }
    return check_launch();
  }
}

gpusq_status launch_spgemm(bool is_i8, const GemmArgs& a, hipStream_t s) {
  return is_i8 ? launch_typed<true>(a, s) : launch_typed<false>(a, s);
}

}  // namespace gpusq
