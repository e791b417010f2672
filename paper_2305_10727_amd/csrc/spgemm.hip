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
//   spgemm_tile_kernel  256 n x 128 m workgroup tile, operands brought into LDS by direct global->LDS copies
//                       (no staging registers), two LDS stages, two workgroups per CU so that one workgroup's
//                       epilogue (VALU + stores) overlaps the other's matrix instructions.  Needs K*elemsize % 128 == 0.
//   spgemm_small_kernel 64 x 64 / 128 x 128 tiles through registers; any K % 16 == 0; used for small or ragged-K problems.
#include <stdlib.h>

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
#define GPUSQ_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define GPUSQ_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

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

// One wavefront's share of the copies that bring K step `ks` of a tile into an LDS stage: the X slab (up to 16 KB),
// 16 fragments of kept values and 4 KB (fp16: 2 KB) of index words are moved in 1 KB pieces dealt round-robin to the
// 4 wavefronts.  Each copy instruction moves 64 lanes x 16 bytes from per-lane global addresses to 1 KB of
// consecutive LDS.  The X slab is stored row-major with the 16-byte chunk c of row r at chunk position
// c ^ ((r >> 1) & 7), so that the 16 rows a quarter-wavefront reads at the same K offset fall in 16 different 16-byte
// bank groups; the swizzle is applied by choosing which global chunk each lane fetches.
// Addresses are a wavefront-uniform 64-bit base (scalar registers, advanced per K step by scalar adds) plus a 32-bit
// per-lane offset fixed for the whole tile (`xoff`), so a K step costs no vector ALU work for addressing.
template <bool IS_I8>
__device__ __forceinline__ void issue_stage_copies(uint8_t* stage, const uint8_t* Xtile_ks, const uint8_t* Wtile,
                                                   const uint32_t (&xoff)[4], int tm, int wave, int lane) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int j = wave + i * 4;  // 1 KB block = 8 rows; the tile has 32*tm rows
    if (j < 4 * tm)
      __builtin_amdgcn_global_load_lds(GPUSQ_GPTR(Xtile_ks + xoff[i]), GPUSQ_LPTR(stage + j * 1024), 16, 0, 0);
  }
  const uint8_t* wsrc = Wtile + wave * kFragValueBytes;
  uint8_t* wdst = stage + kXStageBytes + wave * kFragValueBytes;
  const uint32_t loff = (uint32_t)lane * 16;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    __builtin_amdgcn_global_load_lds(GPUSQ_GPTR(wsrc + i * 4 * kFragValueBytes + loff), GPUSQ_LPTR(wdst + i * 4 * kFragValueBytes),
                                     16, 0, 0);
  if (wave < (IS_I8 ? 4 : 2))
    __builtin_amdgcn_global_load_lds(GPUSQ_GPTR(wsrc + kTileValueBytes + loff), GPUSQ_LPTR(wdst + kTileValueBytes), 16, 0, 0);
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

// All matrix instructions of one K step for one wavefront (128 n x 16*tm m): 8 fragments of A, tm slabs of B.
template <bool IS_I8>
__device__ __forceinline__ void compute_stage(const uint8_t* stage, typename AccT<IS_I8>::type (&acc)[kBigTN][kBigTM], int wn,
                                              int wm, int tm, int lane) {
  const uint8_t* Ws = stage + kXStageBytes;
  const int sw = (lane & 15) >> 1;  // (row >> 1) & 7: slab and wavefront offsets are multiples of 16 rows
  const int q = lane >> 4;
  const uint8_t* xrow = stage + (wm * tm * 16 + (lane & 15)) * kStepBytes;
  const uint8_t* xlo = xrow + (q ^ sw) * 16;
  const uint8_t* xhi = xrow + ((4 + q) ^ sw) * 16;
  const uint8_t* abase = Ws + wn * kBigTN * kFragValueBytes + lane * 16;
  const uint8_t* ibase = Ws + index_offset(IS_I8, wn * kBigTN, lane);  // this lane's 8 index words, consecutive
  // B slabs first, then the A fragments in the order they are consumed: LDS returns data in request order, so the
  // matrix instructions of fragment 0 can start while the remaining fragments stream in
  // (a short tail tile still runs all four slabs: the surplus slabs read stale rows of the stage and their
  // accumulators are never stored; the matrix pipe is not what limits a K step)
  v8i b[kBigTM];
#pragma unroll
  for (int mt = 0; mt < kBigTM; ++mt) {
    const v4i lo = *(const v4i*)(xlo + mt * 16 * kStepBytes), hi = *(const v4i*)(xhi + mt * 16 * kStepBytes);
    b[mt] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  }
  int ai[kBigTN];
  if constexpr (IS_I8) {
    const v4i i0 = *(const v4i*)ibase, i1 = *(const v4i*)(ibase + 16);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      ai[j] = i0[j];
      ai[4 + j] = i1[j];
    }
  } else {
    const v4i i0 = *(const v4i*)ibase;  // 8 x 16 bits
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      ai[2 * j] = i0[j] & 0xFFFF;
      ai[2 * j + 1] = (int)((unsigned)i0[j] >> 16);
    }
  }
  v4i av[kBigTN];
#pragma unroll
  for (int tn = 0; tn < kBigTN; ++tn) av[tn] = *(const v4i*)(abase + tn * kFragValueBytes);
#pragma unroll
  for (int tn = 0; tn < kBigTN; ++tn)
#pragma unroll
    for (int mt = 0; mt < kBigTM; ++mt) acc[tn][mt] = smfmac<IS_I8>(av[tn], b[mt], acc[tn][mt], ai[tn]);
  // Issue order within the K step: the 8 reads of B, the index words and the first three A fragments up front, then
  // four matrix instructions per fragment with the read of the fragment three ahead in between, so that an LDS round
  // trip is covered by 12 matrix instructions and at most 4 fragments are live.
  __builtin_amdgcn_sched_group_barrier(0x100, 8 + (IS_I8 ? 2 : 1) + 3, 0);
#pragma unroll
  for (int tn = 0; tn < kBigTN; ++tn) {
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    if (tn + 3 < kBigTN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
  }
}

// s_waitcnt vmcnt(0) lgkmcnt(0) (gfx9 encoding: vmcnt [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8]): the
// wavefront's own global->LDS copies have landed and its LDS reads of the stage it leaves have returned, so after
// the barrier that follows every stage may be read, and the stage just left may be overwritten.
// The scheduling barrier in front keeps the compiler from hoisting the wait (and the s_barrier after it) above the
// matrix instructions of the K step, which would expose the copy latency instead of hiding it behind them.
#define GPUSQ_WAIT_COPIES_AND_LDS()       \
  do {                                    \
    __builtin_amdgcn_sched_barrier(0);    \
    __builtin_amdgcn_s_waitcnt(0x0070);   \
  } while (0)

// Workgroup = 4 wavefronts (2 along n x 2 along m), 128 channels x 64 rows each, 128 accumulator registers, two
// wavefronts per SIMD = two workgroups per CU (the LDS footprint, 2 stages of 36 KB, allows no more).
//
// Persistent: the grid holds two workgroups per CU and every workgroup walks over tiles with a fixed stride, so the
// output stores of one tile drain while the next tile is being computed; the first K step of the next tile is
// requested before the epilogue of the current one starts, which hides its latency behind the epilogue.
// Tile order: workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2); XCD x takes an eighth of the
// full tiles as one contiguous run plus an eighth of the tail tiles, and its workgroups take them in order, so tiles
// that share an X slab (same rows, n fastest) are computed close in time on one L2.
template <bool IS_I8, int GELU, int OUT>
__global__ void __launch_bounds__(256, 2) spgemm_tile_kernel(const GemmArgs a, const TilePlan plan) {
  typedef typename AccT<IS_I8>::type acc_t;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int STAGE = kXStageBytes + tile_bytes(IS_I8);
  __shared__ __attribute__((aligned(1024))) uint8_t S0[STAGE];
  __shared__ __attribute__((aligned(1024))) uint8_t S1[STAGE];
  __shared__ __attribute__((aligned(16))) float cs[kBigBN];
  __shared__ __attribute__((aligned(16))) float bs[kBigBN];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps wave-derived addresses in scalar registers
  const int wn = wave & 1, wm = wave >> 1;
  const int64_t k_bytes = (int64_t)a.K * ES;
  const int ksteps = (int)(k_bytes / kStepBytes);
  const uint8_t* Xg = (const uint8_t*)a.X;
  const uint8_t* Wg = (const uint8_t*)a.W;
  const int64_t w_col_bytes = (int64_t)ksteps * tile_bytes(IS_I8);  // packed bytes of one 256-channel block
  const int xcd = (int)(blockIdx.x & 7), wgs_per_xcd = (int)(gridDim.x >> 3);
  int f0, nf, t0;
  const int items = xcd_items(plan, xcd, f0, nf, t0);
  // A workgroup first takes its tail tiles, then its full tiles, and the tail tiles go preferably to the second
  // workgroup of each CU (local ids wgs/2 .. wgs-1): the two workgroups that share a CU then run about half a tile out
  // of phase, so that one is in its store/VALU epilogue while the other is in its matrix-instruction loop.
  const int wl = (int)(blockIdx.x >> 3);
  const int nt = items - nf;
  const int tl = (wl + wgs_per_xcd - (wgs_per_xcd >> 1)) % wgs_per_xcd;  // position in the tail hand-out order
  const int my_tail = tl < nt ? (nt - tl + wgs_per_xcd - 1) / wgs_per_xcd : 0;
  const int my_full = wl < nf ? (nf - wl + wgs_per_xcd - 1) / wgs_per_xcd : 0;
  const int my_items = my_tail + my_full;
  if (my_items == 0) return;
  int it = 0;
  auto tile_of = [&](int i) { return i < my_tail ? t0 + tl + i * wgs_per_xcd : f0 + wl + (i - my_tail) * wgs_per_xcd; };
  Tile t = decode_tile(plan, tile_of(0));
  uint32_t xoff[4];
  tile_x_offsets(xoff, t, a.M, k_bytes, wave, lane);
  issue_stage_copies<IS_I8>(S0, Xg + t.m0 * k_bytes, Wg + t.n_blk * w_col_bytes, xoff, t.tm, wave, lane);
  ChannelParams prm;
  prm.fetch<IS_I8>(a, t.n_blk * kBigBN + tid);

  while (true) {
    const uint8_t* Wt = Wg + t.n_blk * w_col_bytes;
    const uint8_t* Xt = Xg + t.m0 * k_bytes;
    acc_t acc[kBigTN][kBigTM];
#pragma unroll
    for (int i = 0; i < kBigTN; ++i)
#pragma unroll
      for (int j = 0; j < kBigTM; ++j) acc[i][j] = acc_t{0, 0, 0, 0};

    GPUSQ_WAIT_COPIES_AND_LDS();  // stage 0 of this tile has landed; the previous tile's reads of cs/bs have returned
    __builtin_amdgcn_s_barrier();
    prm.publish(cs, bs, tid);     // read in the epilogue, after the barriers of the main loop
    for (int ks = 0; ks < ksteps; ks += 2) {
      // stage 1 was last read before the barrier that ended the previous trip, so it may be overwritten now
      if (ks + 1 < ksteps) issue_stage_copies<IS_I8>(S1, Xt + (int64_t)(ks + 1) * kStepBytes, Wt + (int64_t)(ks + 1) * tile_bytes(IS_I8), xoff, t.tm, wave, lane);
      compute_stage<IS_I8>(S0, acc, wn, wm, t.tm, lane);
      GPUSQ_WAIT_COPIES_AND_LDS();
      __builtin_amdgcn_s_barrier();
      if (ks + 1 < ksteps) {
        if (ks + 2 < ksteps) issue_stage_copies<IS_I8>(S0, Xt + (int64_t)(ks + 2) * kStepBytes, Wt + (int64_t)(ks + 2) * tile_bytes(IS_I8), xoff, t.tm, wave, lane);
        compute_stage<IS_I8>(S1, acc, wn, wm, t.tm, lane);
        GPUSQ_WAIT_COPIES_AND_LDS();
        __builtin_amdgcn_s_barrier();
      }
    }
    // both stages are free now (every wavefront passed the last barrier after its last reads): request the first
    // K step of the next tile before the epilogue
    const int cur_n = t.n_blk, cur_tm = t.tm;
    const int64_t cur_m0 = t.m0;
    ++it;
    const bool more = it < my_items;
    if (more) {
      t = decode_tile(plan, tile_of(it));
      tile_x_offsets(xoff, t, a.M, k_bytes, wave, lane);
      issue_stage_copies<IS_I8>(S0, Xg + t.m0 * k_bytes, Wg + t.n_blk * w_col_bytes, xoff, t.tm, wave, lane);
      prm.fetch<IS_I8>(a, t.n_blk * kBigBN + tid);
    }
    wave_epilogue<IS_I8, kBigTN, kBigTM, GELU, OUT>(a, acc, cs, bs, cur_n * kBigBN, cur_n * kBigBN + wn * kBigTN * 16,
                                                    cur_m0 + wm * cur_tm * 16, lane, cur_tm);
    if (!more) break;
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

constexpr int kRing = 4;            // LDS stages: the K step being read plus three in flight
constexpr int kCopiesPerStep = 9;   // copy instructions every wavefront of the computing team issues per K step

// One wavefront's share (a quarter) of the copies of one K step of a tile into the LDS stage at `stage_lds`: four
// 1 KB blocks of the X slab (block j = w + 4i holds rows 8j..8j+7, chunks swizzled as described above
// issue_stage_copies), four fragments of kept values and 1 KB of index words.  Always exactly kCopiesPerStep
// instructions, whatever the tile: a short tail tile copies rows it does not use, and on the fp16 path (2 KB of
// index words) wavefronts 2 and 3 repeat the copies of wavefronts 0 and 1, so that the waits can count instructions.
template <bool IS_I8>
__device__ __forceinline__ void issue_step_copies(uint32_t stage_lds, const uint8_t* Xks, const uint8_t* Wks,
                                                  const uint32_t (&xoff)[4], int w, uint32_t loff) {
#pragma unroll
  for (int i = 0; i < 4; ++i) copy16_to_lds(Xks, xoff[i], stage_lds + (uint32_t)(w + 4 * i) * 1024u);
  const uint8_t* wsrc = Wks + w * kFragValueBytes;
  const uint32_t wdst = stage_lds + kXStageBytes + (uint32_t)w * kFragValueBytes;
#pragma unroll
  for (int i = 0; i < 4; ++i) copy16_to_lds(wsrc + i * 4 * kFragValueBytes, loff, wdst + (uint32_t)i * 4 * kFragValueBytes);
  const int iw = IS_I8 ? w : (w & 1);
  copy16_to_lds(Wks + kTileValueBytes + iw * 1024, loff, stage_lds + kXStageBytes + kTileValueBytes + (uint32_t)iw * 1024u);
}

// s_waitcnt immediates (gfx9 encoding: vmcnt [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8])
constexpr int kWaitVm0 = 0x0F70;            // vmcnt(0)
constexpr int kWaitVm0Lgkm0 = 0x0070;       // vmcnt(0) lgkmcnt(0)
constexpr int kWaitVm18Lgkm0 = 0x4072;      // vmcnt(2 * kCopiesPerStep) lgkmcnt(0)
static_assert(2 * kCopiesPerStep == 18, "kWaitVm18Lgkm0 encodes two K steps of copies");

// Workgroup-wide barrier preceded by a scheduling barrier (the compiler must not move it above the matrix
// instructions of the K step) and followed by a compiler-level memory barrier (no LDS read moves above it).
#define GPUSQ_TEAM_BARRIER()              \
  do {                                    \
    __builtin_amdgcn_sched_barrier(0);    \
    __builtin_amdgcn_s_barrier();         \
    asm volatile("" ::: "memory");        \
  } while (0)

// Epilogue of one wavefront of the team that is not computing: same lane -> output mapping as wave_epilogue, with
//  * the per-channel constants read from the wavefront's own LDS array `p` (128 weight scales, then 128 biases),
//  * `ksteps` workgroup barriers spread evenly over the 16 batches of 8 outputs per lane, so that this team stays in
//    step with the K steps of the team that is computing (both execute the same number of barriers per phase),
//  * a wait for the wavefront's own outstanding copies (requested for the other team's next tile) after the first
//    batch of arithmetic and before the first store and the first barrier: from then on this wavefront has stores in
//    flight and never waits on the vector-memory counter again until its next compute phase.
template <bool IS_I8, int GELU, int OUT>
__device__ __forceinline__ void team_epilogue(const GemmArgs& a, const typename AccT<IS_I8>::type (&acc)[kBigTN][kBigTM],
                                              const float* p, float s_a, int n_wave, int64_t m_wave, int lane, int tm_active,
                                              int ksteps) {
  constexpr bool RAW = IS_I8 && OUT == GPUSQ_I32;
  int done = 0;
#pragma unroll
  for (int g = 0; g < kBigTN / 2; ++g) {
    const int nl = (g >> 1) * kRowBlock + (g & 1) * 32 + (lane >> 4) * 8;  // channel relative to n_wave
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
              v[j] = RAW ? 0.0f : __fmaf_rn((float)raw[j], c8[j], b8[j]);
            } else {
              raw[j] = 0;
              v[j] = acc[2 * g + t][mt][r] + b8[j];
            }
          }
        if constexpr (GELU != 0) gelu_f32_x8(v);
        if (batch == 0) {
          __builtin_amdgcn_sched_barrier(0);
          __builtin_amdgcn_s_waitcnt(kWaitVm0);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (m < a.M) store_8<IS_I8, OUT>(a, m, n_wave + nl, v, raw);
      }
      const int target = ((batch + 1) * ksteps) >> 4;
      while (done < target) {
        GPUSQ_TEAM_BARRIER();
        ++done;
      }
    }
  }
}

// Workgroup = 8 wavefronts = two teams of 4 (2 along n x 2 along m, 128 channels x 64 rows each, as in the kernel
// above), one workgroup per CU; wavefronts 0-3 and 4-7 land on the four SIMDs once each, so every SIMD hosts one
// wavefront of each team.  The workgroup walks over its tiles; team (i mod 2) computes tile i.  Time is cut into
// phases of `ksteps` workgroup barriers: in phase i one team runs the K loop of tile i (matrix instructions, LDS
// reads, copy requests) while the other runs the epilogue of tile i-1 (vector ALU, stores), then they swap.  The
// epilogue's arithmetic and the output stores therefore always overlap matrix work on the same SIMD, the computing
// team has all four LDS stages (copies run three K steps ahead, across tile boundaries), and because loads and stores
// are issued by different wavefronts in any phase, waiting for copies never means waiting for stores.
//
// Copy protocol.  K steps are numbered g = 0, 1, ... over the whole sequence of tiles; step g lives in stage g mod 4.
// The wavefronts of the team that computes step g request step g+3 first (stage (g+3) mod 4 was last read in step
// g-1, which every wavefront left through a barrier after its LDS reads had returned), then run step g, then wait
// until at most the copies of steps g+2 and g+3 are outstanding (vmcnt counts instructions, and every wavefront
// issues kCopiesPerStep per step), then meet at the barrier.  So when step g+1 starts, its data has landed, provided
// it was requested by this team; if it was requested by the other team (the first steps of a tile), that team has
// waited for all its copies before the first barrier of its epilogue phase (see team_epilogue), which is earlier.
// When nothing is requested in a step (the last steps of the last tile) the wait is for all copies.
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
  auto request = [&](int g) -> bool {  // requests the cursor's step into the stage of global step g, advances the cursor
    const bool any = pf_item < my_items;
    if (any) {
      issue_step_copies<IS_I8>(ring_lds + (uint32_t)(g & (kRing - 1)) * STAGE, pf_x, pf_w, pf_xoff, w, loff);
      ++pf_ks;
      pf_x += kStepBytes;
      pf_w += tile_bytes(IS_I8);
      if (pf_ks == ksteps) seek(pf_item + 1, 0);
    }
    return any;
  };

  if (team == 0) {  // the first three K steps of the sequence
    seek(0, 0);
    int n_req = 0;
    for (int g = 0; g < kRing - 1; ++g) n_req += request(g) ? 1 : 0;
    if (n_req == kRing - 1)
      __builtin_amdgcn_s_waitcnt(kWaitVm18Lgkm0);  // step 0 has landed
    else
      __builtin_amdgcn_s_waitcnt(kWaitVm0Lgkm0);
  }
  GPUSQ_TEAM_BARRIER();

  int ph = 0;
  if (team == 1) {  // phase 0: nothing to do for the second team
    for (int k = 0; k < ksteps; ++k) GPUSQ_TEAM_BARRIER();
    ph = 1;
  }
  while (ph <= my_items) {
    // ---- compute phase ph --------------------------------------------------------------------------------------
    if (ph >= my_items) {  // one phase after the last tile: only the other team's last epilogue runs
      for (int k = 0; k < ksteps; ++k) GPUSQ_TEAM_BARRIER();
      break;
    }
    const Tile t = tile_of(ph);
    acc_t acc[kBigTN][kBigTM];
#pragma unroll
    for (int i = 0; i < kBigTN; ++i)
#pragma unroll
      for (int j = 0; j < kBigTM; ++j) acc[i][j] = acc_t{0, 0, 0, 0};
    seek(ph, kRing - 1);
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
    const int g0 = ph * ksteps;
    for (int ks = 0; ks < ksteps; ++ks) {
      const int g = g0 + ks;
      const bool requested = request(g + kRing - 1);
      compute_stage<IS_I8>(ring + (size_t)(g & (kRing - 1)) * STAGE, acc, wn, wm, t.tm, lane);
      __builtin_amdgcn_sched_barrier(0);
      if (requested)
        __builtin_amdgcn_s_waitcnt(kWaitVm18Lgkm0);
      else
        __builtin_amdgcn_s_waitcnt(kWaitVm0Lgkm0);
      GPUSQ_TEAM_BARRIER();
    }
    ++ph;
    // ---- epilogue phase ph: tile ph-1 --------------------------------------------------------------------------------
    team_epilogue<IS_I8, GELU, OUT>(a, acc, my_prm, s_a, t.n_blk * kBigBN + wn * (kBigTN * 16), t.m0 + wm * t.tm * 16, lane, t.tm,
                                    ksteps);
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
  static const bool use_tile_kernel = [] { const char* e = getenv("GPUSQ_KERNEL"); return e && e[0] == 't' && e[1] == 'i'; }();
  if (!use_tile_kernel) {
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
  // persistent grid: two workgroups per CU (the LDS footprint allows no more), never more workgroups than tiles
  const int resident = 2 * num_cus();
  const TilePlan plan = make_plan(a.M, a.N, resident);
  const dim3 grid((unsigned)(ceil_div(plan.total < resident ? plan.total : resident, 8) * 8));
  if constexpr (IS_I8) {
    if (a.out_dt == GPUSQ_I32)
      spgemm_tile_kernel<true, 0, GPUSQ_I32><<<grid, 256, 0, s>>>(a, plan);
    else if (a.out_dt == GPUSQ_I8 && gelu)
      spgemm_tile_kernel<true, 1, GPUSQ_I8><<<grid, 256, 0, s>>>(a, plan);
    else if (a.out_dt == GPUSQ_I8)
      spgemm_tile_kernel<true, 0, GPUSQ_I8><<<grid, 256, 0, s>>>(a, plan);
    else if (gelu)
      spgemm_tile_kernel<true, 1, GPUSQ_F16><<<grid, 256, 0, s>>>(a, plan);
    else
      spgemm_tile_kernel<true, 0, GPUSQ_F16><<<grid, 256, 0, s>>>(a, plan);
  } else {
    if (gelu)
      spgemm_tile_kernel<false, 1, GPUSQ_F16><<<grid, 256, 0, s>>>(a, plan);
    else
      spgemm_tile_kernel<false, 0, GPUSQ_F16><<<grid, 256, 0, s>>>(a, plan);
  }
  return check_launch();
}

gpusq_status launch_spgemm(bool is_i8, const GemmArgs& a, hipStream_t s) {
  return is_i8 ? launch_typed<true>(a, s) : launch_typed<false>(a, s);
}

}  // namespace gpusq
