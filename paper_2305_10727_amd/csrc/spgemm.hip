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
//   spgemm_tile_kernel  tiles of 256 channels x up to 256 rows, operands brought into a three-stage LDS ring by direct
//                       global->LDS copies (no staging registers), one persistent workgroup of 8 wavefronts per CU.
//                       Needs K*elemsize % 128 == 0.
//   spgemm_small_kernel 64 x 64 / 128 x 128 tiles through registers; any K % 16 == 0; used for small or ragged-K problems.
#include <atomic>
#include <cstdlib>
#include <type_traits>

#include "tile_common.h"

namespace gpusq {

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

// ------------------------------------------------------------------------------------------------ tile kernel
// One persistent workgroup of 8 wavefronts per CU on tiles of 256 channels x 64*tm rows (tm <= 4): 2 wavefronts along n x
// 4 along m, 128 channels x 16*tm rows and 128 accumulator registers each.  All wavefronts run the K loop of a tile,
// then all run its epilogue.  With two wavefronts per SIMD in the same phase, a SIMD always has a second wavefront to
// issue from while one waits (for LDS data in the K loop, for a free issue slot in the epilogue: a lone wavefront issues
// a vector instruction only every 6-8 clocks), and the weight tile is brought into the CU once per 256 rows: 52 KB per K
// step through the vector-memory path, which at 48-64 bytes per clock and CU is the narrowest pipe of the K loop.
//
// LDS: a ring of three stages (X slab 32 KB, kept values 16 KB, index words 4/2 KB).  K steps are numbered g = 0, 1, ...
// over the workgroup's whole sequence of tiles; step g lives in stage g % 3.  One workgroup barrier per K step, in front
// of fragment kBarrierFrag: by then a wavefront has issued, and waits for, the last LDS read of the step's stage, and
// it waits for its own copies of step g+1 (the vector-memory counter retires in order, so "at most the copies of step
// g+2 outstanding" means step g+1 has landed).  Behind the barrier stage g+1 is complete and is read ahead (the head of
// the next step: its B operand, its first three A fragments, half of its index words), and stage g is free: the copies
// of step g+3 are requested there, two whole steps before they are needed, also across tile boundaries (the next
// tile's first steps land during the epilogue).  Every wavefront executes exactly one barrier per step of every tile
// of the workgroup, plus one at start-up.
constexpr int kTileTM = 4, kTileWM = 4, kRing = 3;
static_assert(kTileWM * 16 == kTileUnitRows, "tile heights are multiples of one slab per wavefront");
constexpr int kXSlabBytes = kTileWM * kTileTM * 16 * kStepBytes;  // 32 KB: 256 rows x 128 bytes, 16-byte chunks XOR-swizzled per row
constexpr int kBarrierFrag = 5;
constexpr int kCopies = 7;  // copy instructions per wavefront and K step: 4 X blocks, 2 fragments, 1 KB of index words

// s_waitcnt immediates (gfx9 encoding: vmcnt [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8]), all with lgkmcnt(0)
constexpr int kWaitVm0 = 0x0070;    // vmcnt(0)
constexpr int kWaitVm7 = 0x0077;    // vmcnt(kCopies)
constexpr int kWaitVm14 = 0x007E;   // vmcnt(2 * kCopies)
constexpr int kWaitVm15 = 0x007F;   // vmcnt(kCopies + 8)
constexpr int kWaitVm23 = 0x4077;   // vmcnt(kCopies + 16)
static_assert(kCopies == 7, "the wait immediates encode 7, 14, 7 + 8 and 7 + 16");
static_assert(kBarrierFrag + 3 == kTileTN, "slot plan of tile_step");

// Copy I (0..6) of one wavefront's share (an eighth) of the copies that bring one K step of a tile into an LDS stage:
// I = 0..3 are 1 KB blocks of the X slab (block j = wave + 8I holds rows 8j..8j+7), I = 4, 5 fragments of kept values,
// I = 6 1 KB of index words.  Each copy moves 64 lanes x 16 bytes from a wavefront-uniform 64-bit base in scalar
// registers plus a 32-bit per-lane offset that is fixed for the whole tile, to 1 KB of consecutive LDS at a scalar
// base plus a constant: per copy the K loop spends one scalar instruction and one wait state besides the copy itself
// (the K loop is bound by instruction issue, scalar instructions and branches first of all).
//   lds_wave = LDS address of the stage + wave * 1024, lds_idx = that of the index block this wavefront copies;
//   Xks = the X rows of the tile at this K step, Wwave = the packed tile of this K step + wave * 1024;
//   loff = lane * 16, loff8k = loff + 8192, ioff = loff + the index block's offset relative to Wwave.
// Always exactly kCopies instructions per step, whatever the tile (a short tile copies rows it does not use; there are
// only 4 KB / 2 KB of index words, so some wavefronts repeat a block), so that the waits can count instructions.
template <int I>
__device__ __forceinline__ void issue_step_copy(uint32_t lds_wave, uint32_t lds_idx, const uint8_t* Xks, const uint8_t* Wwave,
                                                const uint32_t (&xoff)[4], uint32_t loff, uint32_t loff8k, uint32_t ioff) {
  if constexpr (I < 4)
    copy16_to_lds_at<8192 * I>(Xks, xoff[I < 4 ? I : 0], lds_wave);
  else if constexpr (I == 4)
    copy16_to_lds_at<kXSlabBytes>(Wwave, loff, lds_wave);
  else if constexpr (I == 5)
    copy16_to_lds_at<kXSlabBytes + 8192>(Wwave, loff8k, lds_wave);
  else
    copy16_to_lds_at<0>(Wwave, ioff, lds_idx);
}

// Per-lane byte offsets, relative to the tile's first row, of the four X blocks a wavefront copies per K step: lane l
// fetches row 8j + l/8 of block j, chunk (l%8) ^ ((row >> 1) & 7).  The X slab is stored row-major with the 16-byte
// chunk c of row r at chunk position c ^ ((r >> 1) & 7), so that the 16 rows a quarter-wavefront reads at the same K
// offset fall in 16 different 16-byte bank groups; the swizzle is applied by choosing which global chunk each lane
// fetches.  Rows past the end of X, and rows past the end of a tile shorter than 256 rows (`rows` = its height), re-read
// the last row they may: their results are never stored, and a short tile then draws no rows from memory that it does
// not use (the number of copies stays the same, the waits count them).
__device__ __forceinline__ void tile_x_offsets(uint32_t (&xoff)[4], int64_t m0, int M, int rows, int64_t k_bytes, int wave, int lane) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 8 * (wave + i * 8) + (lane >> 3);
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    int64_t last = (int64_t)M - 1 - m0;  // >= 0: a tile starts inside X
    last = last < rows - 1 ? last : rows - 1;
    const int64_t rr = r < last ? r : last;
    xoff[i] = (uint32_t)(rr * k_bytes + c * 16);
  }
}

// The same for the patch-embedding mode with P = 16: the 16-byte chunk kc of row m = (b, py, px) of the X operand is, for
// int8, the 16 pixels of row py*16 + kc % 16 of patch column px in channel kc / 16 (for fp16, with 2 chunks per patch row:
// row (kc / 2) % 16, channel kc / 32, half kc % 2).  A K step of 8 chunks stays inside one channel, so a lane's address
// splits into a per-lane part that does not depend on the step (returned here, relative to the image batch: the patch's
// first pixel plus the lane's logical chunk inside a step) and a wavefront-uniform part per step (patch_step_offset).
template <bool IS_I8>
__device__ __forceinline__ void patch_x_offsets(uint32_t (&xoff)[4], int64_t m0, const GemmArgs& a, int wave, int lane) {
  constexpr int ES = IS_I8 ? 1 : 2;
  const int px_n = a.patch_W / 16, py_n = a.patch_H / 16;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 8 * (wave + i * 8) + (lane >> 3);
    const int ch = (lane & 7) ^ ((r >> 1) & 7);  // logical chunk of the step this lane fetches (see tile_x_offsets)
    // (32-bit unsigned arithmetic: M < 2^31, and 64-bit divisions here cost the K loop, into which the tile change is
    // inlined, scores of registers)
    uint32_t m = (uint32_t)m0 + (uint32_t)r;
    m = m < (uint32_t)a.M ? m : (uint32_t)a.M - 1u;  // rows past the end re-read the last row
    const uint32_t prow = m / (uint32_t)px_n, px = m - prow * (uint32_t)px_n;
    const uint32_t b = prow / (uint32_t)py_n, py = prow - b * (uint32_t)py_n;
    const int64_t pixel = (((int64_t)b * a.patch_C) * a.patch_H + py * 16) * a.patch_W + px * 16;  // first pixel of the patch, channel 0
    const int row_in_step = IS_I8 ? ch : (ch >> 1), half = IS_I8 ? 0 : (ch & 1);
    xoff[i] = (uint32_t)((pixel + (int64_t)row_in_step * a.patch_W) * ES + half * 16);
  }
}
// Byte offset (wavefront-uniform) that K step ks adds: channel ks / S, first patch row (ks % S) * (16 / S), where a channel
// takes S = 2 (int8) or 4 (fp16) steps.
template <bool IS_I8>
__device__ __forceinline__ int64_t patch_step_offset(const GemmArgs& a, int ks) {
  constexpr int ES = IS_I8 ? 1 : 2, S = IS_I8 ? 2 : 4;
  return ((int64_t)(ks / S) * a.patch_H * a.patch_W + (int64_t)(ks % S) * (16 / S) * a.patch_W) * ES;
}

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

// What a wavefront holds in registers when a K step begins: the four B slabs of the step, its A fragments 0..2
// (fragment f lives in av[f % 4]) and the index words of fragments 0..3; read from the stage whose X slab is at `xslab`
// and whose weight tile is at `wtile`.
template <bool IS_I8>
__device__ __forceinline__ void load_step_head(v8i (&b)[kTileTM], v4i (&av)[4], int (&ai)[kTileTN], const uint8_t* xslab,
                                               const uint8_t* wtile, const BOffsets& bo, uint32_t a_off, uint32_t i_off) {
#pragma unroll
  for (int mt = 0; mt < kTileTM; ++mt) {
    const v4i lo = *(const v4i*)(xslab + bo.lo + mt * 16 * kStepBytes), hi = *(const v4i*)(xslab + bo.hi + mt * 16 * kStepBytes);
    b[mt] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  }
  load_index_half<IS_I8>(ai, 0, wtile + i_off);
#pragma unroll
  for (int f = 0; f < 3; ++f) av[f] = *(const v4i*)(wtile + a_off + f * kFragValueBytes);
}

// One K step of a wavefront (128 n x 64 m), software-pipelined by hand across steps.  When the step begins its B
// operand `b`, its A fragments 0..2 and the index words of fragments 0..3 are in registers.  Per fragment the step
// issues the LDS read of the fragment three ahead, then the four matrix instructions of the fragment; in front of
// fragment kBarrierFrag the wait and the barrier (see the kernel); behind it, one per matrix instruction, the reads
// of the next step's head from `next` into `bn`, `av`, `ai` and the wavefront's kCopies copy requests.  So every other
// instruction is issued in the shadow of a matrix instruction.
// The step has no conditional parts: what the K loop can sustain is set by the instructions a wavefront must issue per
// step (measured: a compare-and-branch pair between two matrix instructions costs more than the matrix instruction), so
// the last step of a tile reads ahead like any other (the next tile reloads those registers) and the steps at the end of
// a workgroup's sequence request copies like any other (the cursor then stays on the last step: they land in a free
// stage and are never read).
// wait_mode (wavefront-uniform): what may stay outstanding at the barrier besides one step of copies: 1 = nothing,
// 2 = 16 output stores, 3 = 8 output stores; 0 = nothing at all may stay outstanding.
// behind_barrier(): called once, right behind the barrier and before the step's copy requests.
template <bool IS_I8, int TMA, class Hook>
__device__ __forceinline__ void tile_step(int wait_mode, const uint8_t* stage, const uint8_t* next, const BOffsets& bo,
                                          typename AccT<IS_I8>::type (&acc)[kTileTN][kTileTM], const v8i (&b)[kTileTM],
                                          v8i (&bn)[kTileTM], v4i (&av)[4], int (&ai)[kTileTN], uint32_t a_off, uint32_t i_off,
                                          uint32_t req_lds_wave, uint32_t req_lds_idx, const uint8_t* req_x, const uint8_t* req_w,
                                          const uint32_t (&xoff)[4], uint32_t loff, uint32_t loff8k, uint32_t ioff,
                                          Hook&& behind_barrier) {
  const uint8_t* abase = stage + kXSlabBytes + a_off;
  const uint8_t* ibase = stage + kXSlabBytes + i_off;
  const uint8_t* abase_n = next + kXSlabBytes + a_off;
  const uint8_t* ibase_n = next + kXSlabBytes + i_off;
  constexpr int kSlots = (kTileTN - kBarrierFrag) * TMA;  // matrix instructions behind the barrier
  static_assert(kSlots >= 2 * TMA + 1, "slot plan of tile_step");
#pragma unroll
  for (int tn = 0; tn < kTileTN; ++tn) {
#pragma unroll
    for (int mt = 0; mt < TMA; ++mt) {
      if (tn == kBarrierFrag && mt == 0) {
        __builtin_amdgcn_sched_barrier(0);  // the compiler must not move the wait above the matrix instructions before it
        if (wait_mode == 1)
          __builtin_amdgcn_s_waitcnt(kWaitVm7);
        else if (wait_mode == 2)
          __builtin_amdgcn_s_waitcnt(kWaitVm23);
        else if (wait_mode == 3)
          __builtin_amdgcn_s_waitcnt(kWaitVm15);
        else
          __builtin_amdgcn_s_waitcnt(kWaitVm0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");  // no LDS read moves above the barrier
        behind_barrier();
      }
      if (mt == 0) {
        const int f = tn + 3;  // f >= kTileTN exactly when tn >= kBarrierFrag: the next stage, behind the barrier
        if (f < kTileTN)
          av[f & 3] = *(const v4i*)(abase + f * kFragValueBytes);
        else
          av[f & 3] = *(const v4i*)(abase_n + (f - kTileTN) * kFragValueBytes);
      }
      if (tn == 0 && mt == (TMA > 2 ? 2 : TMA - 1)) load_index_half<IS_I8>(ai, 1, ibase);
      if (tn >= kBarrierFrag) {
        const int slot = (tn - kBarrierFrag) * TMA + mt;  // 0..kSlots-1
        if (slot < 2 * TMA) {
          const v4i piece = *(const v4i*)(next + ((slot & 1) ? bo.hi : bo.lo) + (slot >> 1) * 16 * kStepBytes);
#pragma unroll
          for (int j = 0; j < 4; ++j) bn[slot >> 1][4 * (slot & 1) + j] = piece[j];
        }
        if (slot == 2 * TMA) load_index_half<IS_I8>(ai, 0, ibase_n);
        // copy c goes out in slot c (12 slots) or is spread evenly over fewer slots
        auto at = [&](int c) { return slot == (kSlots >= kCopies ? c : c * kSlots / kCopies); };
        if (at(0)) issue_step_copy<0>(req_lds_wave, req_lds_idx, req_x, req_w, xoff, loff, loff8k, ioff);
        if (at(1)) issue_step_copy<1>(req_lds_wave, req_lds_idx, req_x, req_w, xoff, loff, loff8k, ioff);
        if (at(2)) issue_step_copy<2>(req_lds_wave, req_lds_idx, req_x, req_w, xoff, loff, loff8k, ioff);
        if (at(3)) issue_step_copy<3>(req_lds_wave, req_lds_idx, req_x, req_w, xoff, loff, loff8k, ioff);
        if (at(4)) issue_step_copy<4>(req_lds_wave, req_lds_idx, req_x, req_w, xoff, loff, loff8k, ioff);
        if (at(5)) issue_step_copy<5>(req_lds_wave, req_lds_idx, req_x, req_w, xoff, loff, loff8k, ioff);
        if (at(6)) issue_step_copy<6>(req_lds_wave, req_lds_idx, req_x, req_w, xoff, loff, loff8k, ioff);
      }
      __builtin_amdgcn_sched_barrier(0);
      acc[tn][mt] = smfmac<IS_I8>(av[tn & 3], b[mt], acc[tn][mt], ai[tn]);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
}

// PATCH: the X operand is gathered from an image batch (patch embedding with P = 16, see patch_x_offsets).
template <bool IS_I8, int GELU, int OUT, bool PATCH = false>
__global__ void __launch_bounds__(512, 1) spgemm_tile_kernel(const GemmArgs a, const TilePlan plan) {
  typedef typename AccT<IS_I8>::type acc_t;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int STAGE = kXSlabBytes + tile_bytes(IS_I8);
  constexpr bool RAW = IS_I8 && OUT == GPUSQ_I32;
  __shared__ __attribute__((aligned(1024))) uint8_t ring[kRing * STAGE];
  // per tile parity and 128-channel half: 128 weight scales, 128 biases (with the int8 ring: 160 KB in all, the CU's LDS)
  __shared__ __attribute__((aligned(1024))) float prm[2][2][256];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wn = wave & 1, wm = wave >> 1;
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
  const float s_out = OUT == GPUSQ_I8 ? a.out_scale[0] : 1.0f, r_out = scale_reciprocal(s_out);  // read once: a load in the epilogue would wait for the copies in flight
  if (!has_bias && wm == 0) {  // the bias halves stay zero for the whole launch (visible after the first barrier)
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      prm[par][wn][128 + lane] = 0.0f;
      prm[par][wn][192 + lane] = 0.0f;
    }
  }
  const uint32_t ring_lds = lds_address(ring), prm_lds = lds_address(prm[0][wn]);
  // The 128 channels [n0, n0 + 128) of epilogue constants of this wavefront's half of a tile, into the constants array
  // of the given parity; requested by the first wavefront of the half.  n0 < 0: nothing (there is no such tile).
  auto request_constants = [&](int n0, int parity) {
    if constexpr (!RAW) {
      if (wm == 0 && n0 >= 0) {
        const uint32_t dst = prm_lds + (uint32_t)parity * (uint32_t)sizeof(prm[0]);
        int lane_now = lane;
        asm volatile("" : "+v"(lane_now));  // computed here, per tile: nothing lane-dependent is carried (or spilled) across the K loop
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          int n = n0 + i * 64 + lane_now;
          n = n < a.N ? n : a.N - 1;  // channels past the end are never stored
          if constexpr (IS_I8) copy4_to_lds(a.w_scale, (uint32_t)n * 4u, dst + (uint32_t)i * 256u);
          if (has_bias) copy4_to_lds(a.bias, (uint32_t)n * 4u, dst + 512u + (uint32_t)i * 256u);
        }
      }
    }
  };
  const uint32_t loff = (uint32_t)lane * 16u;
  const uint32_t a_off = (uint32_t)(wn * kTileTN * kFragValueBytes + lane * 16);
  const uint32_t i_off = (uint32_t)index_offset(IS_I8, wn * kTileTN, lane);

  // lane offsets of the copies of kept values and index words, relative to the packed tile of a K step + wave * 1024
  const uint32_t loff8k = loff + 8192u;
  const int idx_block = IS_I8 ? (wave & 3) : (wave & 1);  // the 1 KB of index words this wavefront copies
  const uint32_t ioff = loff + (uint32_t)(kTileValueBytes + idx_block * 1024 - wave * 1024);
  const uint32_t wave_lds = (uint32_t)wave * 1024u, idx_lds = (uint32_t)(kXSlabBytes + kTileValueBytes + idx_block * 1024);

  // Cursor of the copy requests: the next K step to request, as (tile, step), with its source addresses (pf_w includes
  // wave * 1024).  At the end of the workgroup's sequence it stays on the last step: the requests go on (the waits
  // count a fixed number of copies per step) and re-fetch that step into a stage that nothing reads any more.
  int pf_item = 0, pf_ks = 0;
  const uint8_t *pf_x = Xg, *pf_w = Wg;
  uint32_t pf_xoff[4] = {0, 0, 0, 0};
  auto seek = [&](int item) {
    pf_item = item;
    pf_ks = 0;
    const Tile t = tile_of(item);
    int lane_now = lane;
    asm volatile("" : "+v"(lane_now));  // (computed here, per tile)
    if constexpr (PATCH) {
      patch_x_offsets<IS_I8>(pf_xoff, t.m0, a, wave, lane_now);
      pf_x = Xg;
    } else {
      tile_x_offsets(pf_xoff, t.m0, a.M, kTileUnitRows * t.tm, k_bytes, wave, lane_now);
      pf_x = Xg + t.m0 * k_bytes;
    }
    pf_w = Wg + t.n_blk * w_col_bytes + wave_lds;
  };
  auto advance = [&]() {
    if (pf_ks + 1 < ksteps) {
      ++pf_ks;
      if constexpr (PATCH)
        pf_x = Xg + patch_step_offset<IS_I8>(a, pf_ks);
      else
        pf_x += kStepBytes;
      pf_w += tile_bytes(IS_I8);
    } else if (pf_item + 1 < my_items) {
      seek(pf_item + 1);
    }
  };
  auto request_step = [&](uint32_t stage_lds) {
    issue_step_copy<0>(stage_lds + wave_lds, stage_lds + idx_lds, pf_x, pf_w, pf_xoff, loff, loff8k, ioff);
    issue_step_copy<1>(stage_lds + wave_lds, stage_lds + idx_lds, pf_x, pf_w, pf_xoff, loff, loff8k, ioff);
    issue_step_copy<2>(stage_lds + wave_lds, stage_lds + idx_lds, pf_x, pf_w, pf_xoff, loff, loff8k, ioff);
    issue_step_copy<3>(stage_lds + wave_lds, stage_lds + idx_lds, pf_x, pf_w, pf_xoff, loff, loff8k, ioff);
    issue_step_copy<4>(stage_lds + wave_lds, stage_lds + idx_lds, pf_x, pf_w, pf_xoff, loff, loff8k, ioff);
    issue_step_copy<5>(stage_lds + wave_lds, stage_lds + idx_lds, pf_x, pf_w, pf_xoff, loff, loff8k, ioff);
    issue_step_copy<6>(stage_lds + wave_lds, stage_lds + idx_lds, pf_x, pf_w, pf_xoff, loff, loff8k, ioff);
  };

  acc_t acc[kTileTN][kTileTM];
  v8i b0[kTileTM], b1[kTileTM];  // B operands of the current and the next K step (roles alternate)
  v4i av[4];                     // A fragments in flight
  int ai[kTileTN];               // index words

  // the constants of the first tile, then the first three K steps of the sequence
  request_constants(tile_of(0).n_blk * kTileBN + wn * (kTileTN * 16), 0);
  seek(0);
  for (int g = 0; g < kRing; ++g) {
    request_step(ring_lds + (uint32_t)g * STAGE);
    advance();
  }
  __builtin_amdgcn_s_waitcnt(kWaitVm14);  // the constants and step 0 have landed
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  int slot_off = 0;        // byte offset of the current K step's ring stage
  int first2_mode = 1;     // wait mode of a tile's first two steps (output stores of the previous tile still in the queue)
  for (int item = 0; item < my_items; ++item) {
    const Tile t = tile_of(item);
    int lane_now = lane;
    asm volatile("" : "+v"(lane_now));  // the offsets are computed here, per tile, not once per kernel and kept (or spilled)
    const BOffsets bo = b_offsets(wm, t.tm, lane_now);
    const int next_n0 = item + 1 < my_items ? tile_of(item + 1).n_blk * kTileBN + wn * (kTileTN * 16) : -1;
#pragma unroll
    for (int i = 0; i < kTileTN; ++i)
#pragma unroll
      for (int j = 0; j < kTileTM; ++j) acc[i][j] = acc_t{0, 0, 0, 0};
    // the stage of the tile's first step has landed: start-up barrier, or the barrier in the previous tile's last step
    load_step_head<IS_I8>(b0, av, ai, ring + slot_off, ring + slot_off + kXSlabBytes, bo, a_off, i_off);
    auto step = [&](auto tma, int ks, const v8i (&b)[kTileTM], v8i (&bn)[kTileTM]) {
      const int next_off = slot_off + STAGE == kRing * STAGE ? 0 : slot_off + STAGE;
      // Outstanding at the barrier of step g, oldest first: the copies of step g+1, then those of step g+2, which may
      // stay in flight.  In the first two steps of a tile the output stores of the previous tile's epilogue sit in the
      // queue behind the copies waited for, so they may stay in flight too: the stores drain to memory while the K loop
      // goes on.  The third barrier of a tile then waits for copies that were requested after those stores.  (Only two
      // counts are exploited, the 16 and 8 stores of a wavefront whose 128 x 64 outputs all lie inside Y; any other
      // count waits for the stores as well, which is only stricter.)
      const int wait_mode = ks < 2 ? first2_mode : 1;
      tile_step<IS_I8, decltype(tma)::value>(wait_mode, ring + slot_off, ring + next_off, bo, acc, b, bn, av, ai, a_off, i_off,
                       ring_lds + (uint32_t)slot_off + wave_lds, ring_lds + (uint32_t)slot_off + idx_lds, pf_x, pf_w, pf_xoff, loff,
                       loff8k, ioff, [&]() {
                         // The next tile's constants go into the other constants array, which was last read in the
                         // previous tile's epilogue (every wavefront has left it: it passed this tile's barriers).  They
                         // are older than this step's copy requests and than this tile's output stores, so the wait in
                         // front of the next tile's first barrier covers them and that barrier publishes them.
                         if (ks + 1 == ksteps) request_constants(next_n0, (item + 1) & 1);
                       });
      advance();
      slot_off = next_off;
    };
    // A tile of fewer than 4 slabs per wavefront runs a K loop with the matrix instructions of its own slabs only (the
    // other accumulators stay zero and are never stored); the copies stay the same, so that the waits count the same
    // in every tile.
    auto k_loop = [&](auto tma) {
      for (int ks = 0; ks < ksteps; ks += 2) {
        step(tma, ks, b0, b1);
        if (ks + 1 < ksteps) step(tma, ks + 1, b1, b0);
      }
    };
    if (t.tm == 4)
      k_loop(std::integral_constant<int, 4>{});
    else if (t.tm == 3)
      k_loop(std::integral_constant<int, 3>{});
    else if (t.tm == 2)
      k_loop(std::integral_constant<int, 2>{});
    else
      k_loop(std::integral_constant<int, 1>{});
    const int n_wave = t.n_blk * kTileBN + wn * (kTileTN * 16);
    const int64_t m_wave = t.m0 + wm * t.tm * 16;
    const int64_t rows = (int64_t)a.M - m_wave;
    const int chans = a.N - n_wave;
    // The epilogue, and the number of store instructions this wavefront issues in it (a count that is too high would let
    // the next tile's copies go unwaited, one that is too low only waits for stores as well).
    int stores_pending;
    const bool lines = OUT == GPUSQ_F16 ? (a.N & 7) == 0 : (OUT == GPUSQ_I8 ? (a.N & 15) == 0 : true);
    if (lines) {
      if (t.tm == kTileTM && rows >= kTileTM * 16 && chans >= kTileTN * 16)
        line_epilogue<IS_I8, GELU, OUT, false, kTileTM>(a, acc, prm[item & 1][wn], s_a, s_out, r_out, n_wave, m_wave, lane, kTileTM);
      else
        line_epilogue<IS_I8, GELU, OUT, true, kTileTM>(a, acc, prm[item & 1][wn], s_a, s_out, r_out, n_wave, m_wave, lane, t.tm);
      // per line of the wavefront's 128 channels with a channel inside N (fp16: 64 channels, int32: 32, int8: all 128):
      // one store per slab with a row inside M among its first 8 rows and one for its last 8 rows
      int n = 0;
      for (int mt = 0; mt < t.tm; ++mt) n += (16 * mt < rows) + (16 * mt + 8 < rows);
      const int per_line = OUT == GPUSQ_F16 ? kRowBlock : (OUT == GPUSQ_I8 ? 128 : 32);
      stores_pending = n * (chans <= 0 ? 0 : (chans >= 128 ? 128 / per_line : (chans + per_line - 1) / per_line));
    } else {
      batch_epilogue<IS_I8, GELU, OUT, kTileTM>(a, acc, prm[item & 1][wn], s_a, n_wave, m_wave, lane, t.tm);
      // one (two for 2 x 16 bytes of int32) per batch of 32 channels x 16 rows with a row inside M and a channel inside N;
      // with N % 8 != 0 the number depends on the lanes and is not used
      const int mts = rows <= 0 ? 0 : (rows >= t.tm * 16 ? t.tm : (int)((rows + 15) >> 4));
      const int gs = chans <= 0 ? 0 : (chans >= 128 ? 4 : (chans + 31) >> 5);
      stores_pending = (a.N & 7) ? 0 : mts * gs * (OUT == GPUSQ_I32 ? 2 : 1);
    }
    first2_mode = stores_pending >= 16 ? 2 : (stores_pending >= 8 ? 3 : 1);
  }
  __builtin_amdgcn_s_waitcnt(kWaitVm0);  // the copies requested past the end of the sequence land before the LDS is given up
}

// ------------------------------------------------------------------------------------------------ small / generic kernel
constexpr int kLdsRow = kStepBytes + 16;  // 144-byte row pitch: 16 rows x 16-byte reads hit 16 distinct bank groups

// Workgroup = 4 wavefronts arranged WN (along n) x WM (along m); a wavefront owns TN x TM accumulator tiles.
// Workgroup tile: BN = WN*TN*16 output channels x BM = WM*TM*16 activation rows.  X goes global -> registers -> LDS
// (zero-filled past the row end, rows past M re-read the last row), and so do the weight fragments and index words of
// the tile, a 256th of them per thread.
// XF16 (INT8 path only): X is given in fp16 and quantised on its way through the registers, with the caller's static
// activation scale and the code rule of the activation quantiser; a chunk of 16 codes is then 32 bytes in memory.
template <bool IS_I8, int TN, int TM, int WN, int WM, bool XF16 = false>
__global__ void __launch_bounds__(256) spgemm_small_kernel(const GemmArgs a, const int tiles_n, const int tiles_total) {
  static_assert(WN * WM == 4 && TN % 4 == 0, "4 wavefronts; a wavefront spans whole 64-row blocks");
  static_assert(IS_I8 || !XF16, "the fp16 path takes fp16 X as it is");
  typedef typename AccT<IS_I8>::type acc_t;
  constexpr int BN = WN * TN * 16, BM = WM * TM * 16;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int XW = XF16 ? 2 : 1;  // bytes of X in memory per byte of the X operand
  constexpr int XCH = BM / 32;      // 16-byte chunks of the X slab each thread moves per K step

  constexpr int RBW = BN / kRowBlock;  // 64-channel row blocks of the workgroup's tile (= WN: a wavefront spans one)
  constexpr int kAStep = RBW * 4 * kFragValueBytes;  // kept values of the tile per K step; 1 KB of index words per row block behind them
  static_assert(RBW == WN && (RBW == 1 || RBW == 2), "the workgroup's fragments lie in one packed tile");
  __shared__ __attribute__((aligned(16))) uint8_t Xs[2][BM * kLdsRow];
  __shared__ __attribute__((aligned(16))) uint8_t As[2][kAStep + RBW * 1024];
  __shared__ __attribute__((aligned(16))) float cs[BN];
  __shared__ __attribute__((aligned(16))) float bs[BN];

  const int tile = xcd_tile(tiles_total);
  if (tile >= tiles_total) return;
  const int n_blk = tile % tiles_n, m_blk = tile / tiles_n;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % WN, wm = wave / WN;
  const int M = a.M;
  if (tid < BN) {
    ChannelParams prm;
    prm.fetch<IS_I8>(a, n_blk * BN + tid);
    prm.publish(cs, bs, tid);  // made visible by the barriers of the main loop
  }
  const int64_t k_bytes = (int64_t)a.K * ES;
  const int ksteps = (int)((k_bytes + kStepBytes - 1) / kStepBytes);
  const uint8_t* Xg = (const uint8_t*)a.X;
  const uint8_t* Wg = (const uint8_t*)a.W;

  acc_t acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j) acc[i][j] = acc_t{0, 0, 0, 0};

  // Operands are requested D - 1 K steps ahead, each step into its own set of registers: at these sizes a K step is a
  // few matrix instructions, and what a step costs is the memory latency divided by the number of steps in flight.
  constexpr int D = TM == 1 ? (XF16 ? 4 : 6) : 3;  // (fp16 X in flight takes twice the registers per step)
  v4i xr[D][XCH][XW];
  v4i ar[D][RBW];  // this thread's 16-byte pieces of the tile's kept values (thread t: lane t % 64 of fragment t / 64 + 4j)
  v4i ir[D];       // threads below 64 * RBW: the index words of lane t % 64 for row block t / 64

  // Addresses: a wavefront-uniform base that advances by a constant per K step (scalar arithmetic) plus a 32-bit lane
  // offset fixed for the whole tile, so a K step issues its loads with next to no vector arithmetic: with one wavefront
  // per SIMD (a lone wavefront issues a vector instruction only every 6-8 clocks) address arithmetic per load is what a
  // step would otherwise cost.
  const global_u8* Xtile = uniform_ptr(Xg + (int64_t)m_blk * BM * k_bytes * XW);
  float s_x = 1.0f, r_x = 1.0f;
  if constexpr (XF16) {
    s_x = a.act_scale[0];
    r_x = scale_reciprocal(s_x);
  }
  // Rows past the end of X re-read the last row (their results are never stored), so only a K that is not a whole
  // number of steps needs a predicate, and only in the last step: a plain step is 7 loads and nothing else.
  uint32_t xoff[XCH];
  const int64_t last_row = (int64_t)M - 1 - (int64_t)m_blk * BM;  // >= 0: a tile starts inside X
#pragma unroll
  for (int j = 0; j < XCH; ++j) {
    const int c = tid + 256 * j;
    const int row = (c >> 3) < last_row ? (c >> 3) : (int)last_row;
    xoff[j] = ((uint32_t)row * (uint32_t)k_bytes + (c & 7) * 16) * XW;  // the host keeps 128 rows of X below 4 GiB
  }
  const int tail_bytes = (int)(k_bytes % kStepBytes);  // 0: K is a whole number of steps
  static_assert(TN == 4, "a wavefront's fragments are the four of one 64-channel row block");
  // The weights, like X, enter the CU once per workgroup and K step and reach the wavefronts through LDS: the
  // wavefronts along m need the same fragments, and fetched by each of them straight into registers they were what
  // bound a K step (4 x 5 KB + 8 KB of X per step is all a CU can draw from the L2).
  // (the packed buffer is padded to whole 256-channel tiles, so the tile's row blocks always exist)
  const int rbw = n_blk * RBW;
  const int f0 = (rbw & 3) * 4;
  const global_u8* Wrow = uniform_ptr(Wg + (int64_t)(rbw >> 2) * ksteps * tile_bytes(IS_I8));
  const uint32_t a_thr = (uint32_t)(f0 * kFragValueBytes + tid * 16);
  const bool idx_thr = tid < 64 * RBW;  // (whole wavefronts)
  // the index words of the 4 fragments of a row block are adjacent per lane: 16 bytes (int8) or 8 bytes (fp16)
  const uint32_t i_thr = (uint32_t)index_offset(IS_I8, f0 + 4 * ((tid >> 6) & (RBW - 1)), lane);
  auto load_x = [&](int ks, int slot) {
    const global_u8* base = Xtile + (int64_t)ks * (kStepBytes * XW);
    if (tail_bytes != 0 && ks + 1 == ksteps) {  // workgroup-uniform: the ragged last step zero-fills past the row end
#pragma unroll
      for (int j = 0; j < XCH; ++j)
#pragma unroll
        for (int h = 0; h < XW; ++h)
          xr[slot][j][h] = (int)(((tid + 256 * j) & 7) * 16) < tail_bytes
                               ? *(const __attribute__((address_space(1))) v4i*)(base + xoff[j] + 16 * h)
                               : v4i{0, 0, 0, 0};
    } else {
#pragma unroll
      for (int j = 0; j < XCH; ++j)
#pragma unroll
        for (int h = 0; h < XW; ++h) xr[slot][j][h] = *(const __attribute__((address_space(1))) v4i*)(base + xoff[j] + 16 * h);
    }
  };
  auto store_x = [&](int buf, int slot) {
#pragma unroll
    for (int j = 0; j < XCH; ++j) {
      const int c = tid + 256 * j;
      v4i codes;
      if constexpr (XF16) {
        // 16 fp16 values -> 16 int8 codes (zero-filled chunks give zero codes)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const ep_v8h x = __builtin_bit_cast(ep_v8h, xr[slot][j][h]);
          float v[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = (float)x[e];
          unsigned lo, hi;
          quantize_bytes8(v, s_x, r_x, lo, hi);
          codes[2 * h] = (int)lo;
          codes[2 * h + 1] = (int)hi;
        }
      } else {
        codes = xr[slot][j][0];
      }
      *(v4i*)(&Xs[buf][(c >> 3) * kLdsRow + (c & 7) * 16]) = codes;
    }
  };
  auto load_a = [&](int ks, int slot) {
    const global_u8* t = Wrow + (int64_t)ks * tile_bytes(IS_I8);
#pragma unroll
    for (int j = 0; j < RBW; ++j)
      ar[slot][j] = *(const __attribute__((address_space(1))) v4i*)(t + a_thr + j * (4 * kFragValueBytes));
    if (idx_thr) {
      if constexpr (IS_I8) {
        ir[slot] = *(const __attribute__((address_space(1))) v4i*)(t + i_thr);
      } else {
        const ep_v2u w = *(const __attribute__((address_space(1))) ep_v2u*)(t + i_thr);
        ir[slot] = v4i{(int)w[0], (int)w[1], 0, 0};
      }
    }
  };
  auto store_a = [&](int buf, int slot) {
#pragma unroll
    for (int j = 0; j < RBW; ++j) *(v4i*)(&As[buf][tid * 16 + j * (4 * kFragValueBytes)]) = ar[slot][j];
    if (idx_thr) *(v4i*)(&As[buf][kAStep + tid * 16]) = ir[slot];
  };

  // K steps q * D + r: q passes of D steps without any condition in them (the request D - 1 steps ahead is clamped to
  // the last step, whose data is then fetched again and not used), then the r < D remaining steps, whose operands the
  // last pass (or the preamble) has already requested, as straight-line code behind uniform forward branches.
  auto clamp_step = [&](int ks) { return ks < ksteps ? ks : ksteps - 1; };
#pragma unroll
  for (int d = 0; d < D - 1; ++d) {
    load_x(clamp_step(d), d);
    load_a(clamp_step(d), d);
  }
  const int b_row = wm * TM * 16 + (lane & 15);
  const int b_col = (lane >> 4) * 16;
  // The operands alternate between two LDS buffers, and the step is pipelined across them: step ks first writes the
  // operands of step ks + 1 into the other buffer (last read in step ks - 1, whose closing barrier every wavefront has
  // passed), then reads its own, multiplies, and closes with the barrier that publishes what it wrote.  So the LDS round
  // trip of a step's operands runs beside the previous step's reads and matrix instructions instead of in front of its
  // own.
  store_x(0, 0);
  store_a(0, 0);
  __syncthreads();
  auto compute_step = [&](int ks, int slot) {
    const int cur = ks & 1;
    if (ks + 1 < ksteps) {  // workgroup-uniform
      store_x(cur ^ 1, (slot + 1) % D);
      store_a(cur ^ 1, (slot + 1) % D);
    }
    v4i av[TN];
    int ai[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) av[tn] = *(const v4i*)(&As[cur][(wn * TN + tn) * kFragValueBytes + lane * 16]);
    const v4i iw = *(const v4i*)(&As[cur][kAStep + wn * 1024 + lane * 16]);
    if constexpr (IS_I8) {
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) ai[tn] = iw[tn];
    } else {
      ai[0] = iw[0] & 0xFFFF;
      ai[1] = (int)((unsigned)iw[0] >> 16);
      ai[2] = iw[1] & 0xFFFF;
      ai[3] = (int)((unsigned)iw[1] >> 16);
    }
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      const uint8_t* p = &Xs[cur][(b_row + mt * 16) * kLdsRow + b_col];
      const v4i lo = *(const v4i*)p, hi = *(const v4i*)(p + 64);
      const v8i b = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) acc[tn][mt] = smfmac<IS_I8>(av[tn], b, acc[tn][mt], ai[tn]);
    }
    __syncthreads();
  };
  const int passes = ksteps / D, rest = ksteps - passes * D;
  int ks = 0;
  for (int pass = 0; pass < passes; ++pass) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
      load_x(clamp_step(ks + D - 1), (j + D - 1) % D);
      load_a(clamp_step(ks + D - 1), (j + D - 1) % D);
      compute_step(ks, j);
      ++ks;
    }
  }
#pragma unroll
  for (int d = 0; d < D - 1; ++d)
    if (d < rest) compute_step(ks + d, d);  // workgroup-uniform
  __syncthreads();  // the per-channel constants written at the top are read below (also when K has no step at all)
  wave_epilogue<IS_I8, TN, TM>(a, acc, cs, bs, n_blk * BN, n_blk * BN + wn * TN * 16, (int64_t)m_blk * BM + wm * TM * 16, lane);
}

template <bool IS_I8, int TN, int TM, int WN, int WM>
static gpusq_status launch_small(const GemmArgs& a, hipStream_t s) {
  constexpr int BN = WN * TN * 16, BM = WM * TM * 16;
  const int tiles_n = (int)ceil_div(a.N, BN), tiles_m = (int)ceil_div(a.M, BM);
  const int total = tiles_n * tiles_m;
  const int grid = (int)ceil_div(total, 8) * 8;  // whole rounds over the 8 XCDs; surplus workgroups exit at once
  const int x_elem_bytes = (IS_I8 && !a.x_f16) ? 1 : 2;
  if ((int64_t)a.K * x_elem_bytes * BM >= ((int64_t)1 << 32)) return GPUSQ_ERR_UNSUPPORTED;  // 32-bit lane offsets inside a tile's rows of X
  if constexpr (IS_I8) {
    if (a.x_f16) {
      spgemm_small_kernel<true, TN, TM, WN, WM, true><<<grid, 256, 0, s>>>(a, tiles_n, total);
      return check_launch();
    }
  }
  spgemm_small_kernel<IS_I8, TN, TM, WN, WM><<<grid, 256, 0, s>>>(a, tiles_n, total);
  return check_launch();
}

// Compute units of the current device, read once per device (a racing first call reads the same value twice).
static int num_cus() {
  constexpr int kMaxDevices = 64;
  static std::atomic<int> cus[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
  int n = cus[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cus[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// Testing aid: -1 = the size rules decide, 0 / 1 / 2 = run every problem the kernel can take on that kernel.  Set by
// gpusq_force_kernel(); the environment variable GPUSQ_FORCE_KERNEL gives the initial value and is read once, when the
// library is loaded, so that no launch pays for an environment lookup.
static int initial_forced_kernel() {
  const char* f = getenv("GPUSQ_FORCE_KERNEL");
  return (f && f[0] >= '0' && f[0] <= '3' && f[1] == 0) ? f[0] - '0' : -1;
}
static std::atomic<int> g_forced_kernel{initial_forced_kernel()};
int forced_kernel() { return g_forced_kernel.load(std::memory_order_relaxed); }
int set_forced_kernel(int kernel) {
  return g_forced_kernel.exchange(kernel >= 0 && kernel <= 3 ? kernel : -1);
}

// Estimated run time (microseconds, fitted to traces and timings of the kernel on MI355X) of one tile of 64*tm rows: a
// K step costs nearly the same whatever tm (a short tile copies and reads whole operands and only leaves out the matrix
// instructions of the slabs it does not have: 1.1 us for tm = 4, about 0.075 us less per slab left out), the epilogue
// scales with the rows stored and is larger with GELU.
// `busy` is the fraction of the CUs that have a workgroup: the fewer run, the faster each one's K steps (the chip runs
// at its power limit when all of them multiply: 1.1 us per step on 256 CUs, 0.63 on 150, 0.46 on 100).
static double tile_cost(int tm, int ksteps, bool gelu, double busy) {
  double step = (0.8 + 0.075 * tm) * (0.1 + 0.9 * busy);
  if (step < 0.6) step = 0.6;  // (what a K step costs a lone workgroup: latency, not throughput)
  return ksteps * step + (gelu ? 1.6 : 1.1) * tm + 0.3;
}

// The workgroup with the most work under the kernel's assignment (XCD x takes its share of the list, its workgroup wl
// the items wl, wl + W, ...).
static double plan_makespan(const TilePlan& p, int grid, int ksteps, bool gelu, double busy) {
  const int W = grid / 8;
  const double cf = tile_cost(p.full_tm, ksteps, gelu, busy), ct = tile_cost(p.tail_tm, ksteps, gelu, busy);
  double worst = 0;
  for (int x = 0; x < 8; ++x) {
    int f0, nf, t0;
    const int items = xcd_items(p, x, f0, nf, t0);
    for (int wl = 0; wl < W && wl < items; ++wl) {
      const int mine = (items - wl + W - 1) / W;
      const int full = wl < nf ? (nf - wl + W - 1) / W : 0;
      const double c = full * cf + (mine - full) * ct;
      if (c > worst) worst = c;
    }
  }
  return worst;
}

static int grid_for(const TilePlan& p, int resident) { return (int)ceil_div(p.total < resident ? p.total : resident, 8) * 8; }

// Candidates: full tiles of 64, 128, 192 or 256 rows, either over all of M, or for as many whole rounds over the resident
// workgroups as the problem has with the remaining rows in tail tiles of 64..64*full_tm rows; the one whose busiest
// workgroup finishes first wins.
static TilePlan make_plan(int M, int N, int resident, int ksteps, bool gelu) {
  TilePlan best{};
  double best_cost = -1;
  const int tiles_n = (int)ceil_div(N, kTileBN);
  auto consider = [&](int ftm, int full_chunks, int ttm) {
    TilePlan p;
    p.tiles_n = tiles_n;
    p.full_tm = ftm;
    p.full_chunks = full_chunks;
    p.full_tiles = full_chunks * tiles_n;
    p.tail_tm = ttm;
    const int64_t rows_left = (int64_t)M - (int64_t)full_chunks * 64 * ftm;
    p.total = p.full_tiles + (rows_left > 0 ? (int)ceil_div(rows_left, 64 * ttm) * tiles_n : 0);
    p.inv_tiles_n = (tiles_n > 1 && tiles_n <= 4096 && p.total < (1 << 20)) ? (uint32_t)((((uint64_t)1 << 32) + tiles_n - 1) / tiles_n) : 0u;
    const double c = plan_makespan(p, grid_for(p, resident), ksteps, gelu, 1.0);  // (plans are compared at the full-chip step cost)
    if (best_cost < 0 || c < best_cost) {
      best_cost = c;
      best = p;
    }
  };
  for (int ftm = kTileTM; ftm >= 1; --ftm) {
    const int chunks = (int)ceil_div(M, 64 * ftm);
    consider(ftm, chunks, ftm);
    const int all_tiles = chunks * tiles_n;
    if (all_tiles > resident && all_tiles % resident != 0) {
      const int full_chunks = (all_tiles / resident) * resident / tiles_n;
      for (int ttm = ftm; ttm >= 1; --ttm) consider(ftm, full_chunks, ttm);
    }
  }
  return best;
}

// Which kernel a problem takes: 0 = small kernel with 64 x 64 tiles, 1 = small kernel with 128 x 128 tiles, 2 = tile
// kernel.  K that is not a whole number of 128-byte steps needs the zero-filling small kernel.  Otherwise the estimated
// run times decide (microseconds, fitted to graph-replayed launches on MI355X for M = 197 ... 6304): the small kernel
// keeps two workgroups per CU busy, costs about 0.7 us + 0.45 us per K step per round of 512 workgroups and never less than what
// one workgroup's chain of loads takes; the tile kernel costs its plan's makespan plus the start-up of its pipeline.
// With few rows (one image: M = 197) the tile kernel has too few tiles for the chip and the small kernel is about
// twice as fast; from a few thousand rows on the tile kernel wins.  fused_patches: the patch gather exists in the tile
// kernel only, so that mode keeps the plain size rule.
static int kernel_choice(bool is_i8, int64_t M, int64_t N, int64_t K, bool gelu, int resident, bool fused_patches = false) {
  const int64_t k_bytes = K * (is_i8 ? 1 : 2);
  const int64_t ksteps = ceil_div(k_bytes, kStepBytes);
  const int64_t wgs64 = ceil_div(M, 64) * ceil_div(N, 64);
  // Testing aid: a forced kernel overrides the choice (2 only where the tile kernel can run the problem).
  if (const int c = g_forced_kernel.load(std::memory_order_relaxed); c >= 0) {
    if (c < 2 || k_bytes % kStepBytes == 0) return c;
  }
  if (M * N <= (int64_t)256 * 1024) return 0;
  if (k_bytes % kStepBytes != 0) return wgs64 <= 2 * resident ? 0 : 1;
  if (fused_patches) return 2;
  // Between the two tile kernels the measured times decide (every linear layer of the ViT-B, Swin-B, ViT-L and ViT-H
  // workloads, FP16 and INT8, with hot and with cold buffers, the two kernels timed in turn; they are within 10 % of each
  // other almost everywhere): the kernel with two workgroups per CU is ahead, by 15-20 %, on layers with few output
  // channels, short K and no GELU (the attention projections and the QKV layer of the narrow models: few tiles per CU,
  // where its smaller tiles balance better); for FP16 only from 1024 output channels on (below that it is up to 14 %
  // behind once the activations come from HBM).  The single-workgroup kernel keeps the wide layers, the GELU layers and
  // every long-K layer, where its deeper ring hides the latency of cold activations (the other kernel is 10-25 % behind
  // there on cold buffers).
  const int tile_kernel = (N <= 1536 && K <= 1024 && !gelu && (is_i8 || N >= 1024)) ? 3 : 2;
  if (wgs64 > 16 * resident) return tile_kernel;  // far beyond the crossover with the small kernel: skip the planning
  const double per_round = 0.7 + 0.45 * ksteps, chain = 3.6 + 0.25 * ksteps;
  const double throughput = 4.0 + per_round * (double)wgs64 / (2.0 * resident);
  const double est_small = chain > throughput ? chain : throughput;
  const TilePlan p = make_plan((int)M, (int)N, resident, (int)ksteps, gelu);
  const int grid = grid_for(p, resident);
  const double est_tile = plan_makespan(p, grid, (int)ksteps, gelu, (double)(p.total < grid ? p.total : grid) / resident) + 2.8;
  return est_small < est_tile ? 0 : tile_kernel;
}

gpusq_status plan_spgemm(bool is_i8, int64_t M, int64_t N, int64_t K, int epilogue, int cus, int32_t* out) {
  const int resident = cus > 0 ? cus : num_cus();
  const int choice = kernel_choice(is_i8, M, N, K, (epilogue & GPUSQ_EPI_GELU) != 0, resident);
  for (int i = 0; i < 8; ++i) out[i] = 0;
  out[0] = choice;
  if (choice < 2) return GPUSQ_OK;
  const int ksteps = (int)(K * (is_i8 ? 1 : 2) / kStepBytes);
  const bool gelu = (epilogue & GPUSQ_EPI_GELU) != 0;
  const TilePlan p = choice == 2 ? make_plan((int)M, (int)N, resident, ksteps, gelu) : make_tile2_plan((int)M, (int)N, 2 * resident, ksteps, gelu, false);
  out[1] = 64;
  out[2] = p.tiles_n;
  out[3] = p.full_tm;
  out[4] = p.full_chunks;
  out[5] = p.tail_tm;
  out[6] = p.total;
  out[7] = choice == 2 ? grid_for(p, resident) : tile2_grid_of(p, 2 * resident);
  return GPUSQ_OK;
}

// The kernel choice and tile plan of a problem, remembered per thread for the last few distinct problems: a layer is
// launched over and over with the same sizes, and planning (a dozen candidate plans, each walked over every workgroup)
// takes the host several microseconds, which is what a launch of a 10 us GEMM is bound by when it is repeated.
struct Decision {
  bool is_i8, gelu, patches;
  int forced;  // the forced kernel when the decision was taken, -1 for none
  int64_t M, N, K;
  int resident, choice;
  TilePlan plan;  // valid when choice == 2
};
static const Decision& decide(bool is_i8, int64_t M, int64_t N, int64_t K, bool gelu, int resident, bool patches) {
  constexpr int kSlots = 16;
  thread_local Decision cache[kSlots];
  thread_local int used = 0, next = 0;
  const int forced = g_forced_kernel.load(std::memory_order_relaxed);
  for (int i = 0; i < used; ++i) {
    const Decision& d = cache[i];
    if (d.M == M && d.N == N && d.K == K && d.is_i8 == is_i8 && d.gelu == gelu && d.patches == patches && d.forced == forced &&
        d.resident == resident)
      return d;
  }
  Decision& d = cache[next];
  next = (next + 1) % kSlots;
  if (used < kSlots) ++used;
  d = Decision{is_i8, gelu, patches, forced, M, N, K, resident, kernel_choice(is_i8, M, N, K, gelu, resident, patches), TilePlan{}};
  const int64_t k_bytes = K * (is_i8 ? 1 : 2);
  if (d.choice == 2) d.plan = make_plan((int)M, (int)N, resident, (int)(k_bytes / kStepBytes), gelu);
  if (d.choice == 3) d.plan = make_tile2_plan((int)M, (int)N, 2 * resident, (int)(k_bytes / kStepBytes), gelu, false);
  return d;
}

template <bool IS_I8>
static gpusq_status launch_typed(const GemmArgs& a, hipStream_t s) {
  const int64_t k_bytes = (int64_t)a.K * (IS_I8 ? 1 : 2);
  const bool gelu = (a.epilogue & GPUSQ_EPI_GELU) != 0;
  const int resident = num_cus();
  const Decision& dec = decide(IS_I8, a.M, a.N, a.K, gelu, resident, a.patch_P != 0);
  const int choice = dec.choice;
  // the fused patch gather exists in the tile kernel only, for 16 x 16 patches, fp16 output, no GELU
  if (a.patch_P != 0 && choice == 3) return GPUSQ_ERR_UNSUPPORTED;
  if (a.patch_P != 0 && (choice != 2 || a.patch_P != 16 || a.out_dt != GPUSQ_F16 || gelu)) return GPUSQ_ERR_UNSUPPORTED;
  // quantising fp16 activations on the way in exists in the small kernel only (X passes through its registers)
  if (a.x_f16 && (!IS_I8 || choice >= 2)) return GPUSQ_ERR_UNSUPPORTED;
  if (choice == 3) {
    if (!tile2_supports(IS_I8, false, a)) return GPUSQ_ERR_UNSUPPORTED;
    return launch_tile2(IS_I8, false, a, dec.plan, tile2_grid_of(dec.plan, 2 * resident), s);
  }
  if (choice == 0) return launch_small<IS_I8, 4, 1, 1, 4>(a, s);
  if (choice == 1) return launch_small<IS_I8, 4, 4, 2, 2>(a, s);
  // persistent grid: one workgroup per CU, never more workgroups than tiles
  const int ksteps = (int)(k_bytes / kStepBytes);
  const TilePlan plan = dec.plan;
  const dim3 grid((unsigned)grid_for(plan, resident));
  if ((ceil_div(plan.total, grid.x) + 2) * ksteps >= ((int64_t)1 << 30)) return GPUSQ_ERR_UNSUPPORTED;
  if ((int64_t)a.N * 16 * 4 >= ((int64_t)1 << 31)) return GPUSQ_ERR_UNSUPPORTED;  // 32-bit lane offsets inside 16 rows of Y
  // 32-bit lane offsets inside the 256 rows of X of a tile (tile_x_offsets; the patch gather has its own limit)
  if (a.patch_P == 0 && 255 * k_bytes + kStepBytes >= ((int64_t)1 << 32)) return GPUSQ_ERR_UNSUPPORTED;
  if (a.patch_P != 0) {
    spgemm_tile_kernel<IS_I8, 0, GPUSQ_F16, true><<<grid, 512, 0, s>>>(a, plan);
    return check_launch();
  }
  if constexpr (IS_I8) {
    if (a.out_dt == GPUSQ_I32)
      spgemm_tile_kernel<true, 0, GPUSQ_I32><<<grid, 512, 0, s>>>(a, plan);
    else if (a.out_dt == GPUSQ_I8 && gelu)
      spgemm_tile_kernel<true, 1, GPUSQ_I8><<<grid, 512, 0, s>>>(a, plan);
    else if (a.out_dt == GPUSQ_I8)
      spgemm_tile_kernel<true, 0, GPUSQ_I8><<<grid, 512, 0, s>>>(a, plan);
    else if (gelu)
      spgemm_tile_kernel<true, 1, GPUSQ_F16><<<grid, 512, 0, s>>>(a, plan);
    else
      spgemm_tile_kernel<true, 0, GPUSQ_F16><<<grid, 512, 0, s>>>(a, plan);
  } else {
    if (gelu)
      spgemm_tile_kernel<false, 1, GPUSQ_F16><<<grid, 512, 0, s>>>(a, plan);
    else
      spgemm_tile_kernel<false, 0, GPUSQ_F16><<<grid, 512, 0, s>>>(a, plan);
  }
  return check_launch();
}

gpusq_status launch_spgemm(bool is_i8, const GemmArgs& a, hipStream_t s) {
  return is_i8 ? launch_typed<true>(a, s) : launch_typed<false>(a, s);
}

}  // namespace gpusq
