// Tile kernel with two resident workgroups per CU, for the 2:4 sparse GEMM (Sec. 3.1 / Fig. 1: sparse x dense -> dense over
// the kept values) and, from the same template, for its dense twin on the masked but uncompressed weights (the "T cycles"
// side of the paper's T vs T/2 comparison).
//
// Why two workgroups.  A tile has two phases that use different units of a SIMD: the K loop (matrix pipe, LDS reads,
// operand copies) and the fused epilogue (dequantise, bias, GELU, convert: vector ALU, about 13 issue slots per output,
// and the output stores).  Here a workgroup of 8 wavefronts owns a tile of 256 channels x 128 rows and needs at most 128
// registers per lane and 80 KB of LDS, so two workgroups are resident per CU (four wavefronts per SIMD) and one
// workgroup's epilogue can run beside the other's K loop.  Measured, the overlap is partial (a wavefront of vector
// instructions beside a busy matrix pipe issues at about half its rate) and is paid for with more LDS reads per matrix
// instruction (wavefront tile 128 x 32) and a ring of two stages: against the kernel with one workgroup per CU this one
// is 15-20 % ahead where there are few tiles per CU (its smaller tiles balance better), level on most shapes and behind
// on long K with cold activations; the size rule in spgemm.hip sends it the former.
//
// One template, two operand formats:
//   sparse: K step = 128 bytes of an activation row; the packed weight tile of the step (16 fragments x 1 KB of kept
//           values + index words, common.h) is copied as it lies in memory; v_smfmac_i32_16x16x128_i8 /
//           v_smfmac_f32_16x16x64_f16.
//   dense : K step = 64 bytes; the 256 weight rows of the step are gathered from W [N][K] into the same fragment order
//           (lane l of fragment f: 16 bytes of channel row l % 16 at K offset 16 * (l / 16)), so the accumulators and the
//           epilogue are the same; v_mfma_i32_16x16x64_i8 / v_mfma_f32_16x16x32_f16.  One dense step holds as many matrix
//           instructions as one sparse step and half the K extent: twice the instructions per output, the 2x of Fig. 1.
// Everything else is shared: persistent XCD-aware grid, direct global->LDS copies with explicit waits, a two-stage LDS
// ring per workgroup, whole-line non-temporal output stores.
//
// Synchronisation.  K steps are numbered over the workgroup's whole sequence of tiles; step g lives in stage g % 2.  Each
// step starts with "wait for my copies of this step, barrier": behind the barrier the step's stage is complete and the
// other stage is free (every wavefront has issued, and received, its last LDS read of the previous step), so the copies of
// the next step, possibly the next tile's first, are requested there and land while this step multiplies (and, across a
// tile boundary, during the epilogue).  A wavefront executes one barrier per step of every tile of its workgroup.
#include <type_traits>

#include "tile_common.h"

namespace gpusq {

constexpr int kT2TM = 2;  // 16-row slabs per wavefront; 4 wavefronts along m: tiles of 128 rows (64 for a short tile)

template <bool IS_I8, bool DENSE>
struct T2 {
  static constexpr int ES = IS_I8 ? 1 : 2;
  static constexpr int STEP = DENSE ? 64 : kStepBytes;                 // bytes of an activation row per K step
  static constexpr int ROWS = 4 * kT2TM * 16;                          // 128
  static constexpr int XSLAB = ROWS * STEP;                            // 16 KB / 8 KB
  static constexpr int XBLOCKS = XSLAB / 1024 / 8;                     // 1 KB copies of the X slab per wavefront and step
  static constexpr int WIDX = DENSE ? 0 : 16 * frag_index_bytes(IS_I8);
  static constexpr int STAGE = XSLAB + kTileValueBytes + WIDX;         // 36 / 34 KB (sparse), 24 KB (dense)
  static constexpr int IDX_BLOCKS = WIDX / 1024;                       // 4 / 2 / 0
  typedef typename std::conditional<DENSE, v4i, v8i>::type b_t;        // B operand of one matrix instruction
};

template <bool IS_I8>
__device__ __forceinline__ typename AccT<IS_I8>::type mfma_dense(v4i a, v4i b, typename AccT<IS_I8>::type c) {
  if constexpr (IS_I8)
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
}

// s_waitcnt with lgkmcnt(0), expcnt(7) and vmcnt(N), N one of the store counts a full tile leaves behind (gfx9 encoding:
// vmcnt in bits [3:0] and [15:14])
__device__ __forceinline__ void wait_copies_behind_stores(int stores) {
  if (stores == 16)
    __builtin_amdgcn_s_waitcnt(0x4070);
  else if (stores == 8)
    __builtin_amdgcn_s_waitcnt(0x0078);
  else if (stores == 4)
    __builtin_amdgcn_s_waitcnt(0x0074);
  else
    __builtin_amdgcn_s_waitcnt(0x0070);
}

template <bool IS_I8, bool DENSE, int GELU, int OUT>
__global__ void __launch_bounds__(512, 4) gemm_tile2_kernel(const GemmArgs a, const TilePlan plan) {
  typedef T2<IS_I8, DENSE> G;
  typedef typename AccT<IS_I8>::type acc_t;
  typedef typename G::b_t b_t;
  constexpr bool RAW = IS_I8 && OUT == GPUSQ_I32;
  __shared__ __attribute__((aligned(1024))) uint8_t ring[2 * G::STAGE];
  __shared__ __attribute__((aligned(1024))) float prm[2][256];  // per 128-channel half: 128 weight scales, 128 biases

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wn = wave & 1, wm = wave >> 1;
  const int64_t k_bytes = (int64_t)a.K * G::ES;
  const int ksteps = (int)(k_bytes / G::STEP);
  const uint8_t* Xg = (const uint8_t*)a.X;
  const uint8_t* Wg = (const uint8_t*)a.W;
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
  const float s_out = OUT == GPUSQ_I8 ? a.out_scale[0] : 1.0f, r_out = scale_reciprocal(s_out);
  if (!has_bias && wm == 0) {  // the bias half stays zero for the whole launch (visible after the first barrier)
    prm[wn][128 + lane] = 0.0f;
    prm[wn][192 + lane] = 0.0f;
  }
  const uint32_t ring_lds = lds_address(ring), prm_lds = lds_address(prm[wn]);
  // the 128 channels [n0, n0 + 128) of epilogue constants of this wavefront's half of a tile, requested by the first
  // wavefront of the half
  auto request_constants = [&](int n0) {
    if constexpr (!RAW) {
      if (wm == 0) {
        int lane_now = lane;
        asm volatile("" : "+v"(lane_now));  // computed here, per tile: nothing lane-dependent is carried across the K loop
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          int n = n0 + i * 64 + lane_now;
          n = n < a.N ? n : a.N - 1;  // channels past the end are never stored
          if constexpr (IS_I8) copy4_to_lds(a.w_scale, (uint32_t)n * 4u, prm_lds + (uint32_t)i * 256u);
          if (has_bias) copy4_to_lds(a.bias, (uint32_t)n * 4u, prm_lds + 512u + (uint32_t)i * 256u);
        }
      }
    }
  };

  // ---- the copy requests of one K step: cursor (tile, step) with its source addresses -------------------------------
  const uint32_t wave_lds = (uint32_t)wave * 1024u;
  int pf_item = 0, pf_ks = 0;
  bool pf_more = true;
  const uint8_t *pf_x = Xg, *pf_w = Wg;
  uint32_t pf_xoff[G::XBLOCKS];
  uint32_t pf_woff[2];  // sparse: lane * 16 (+ 8192); dense: the lane's two weight rows of the tile
  auto seek = [&](int item) {
    pf_item = item;
    pf_ks = 0;
    const Tile t = tile_of(item);
    int l = lane;
    asm volatile("" : "+v"(l));  // (computed here, per tile)
    int64_t last = (int64_t)a.M - 1 - t.m0;  // >= 0: a tile starts inside X
    last = last < kTileUnitRows * t.tm - 1 ? last : kTileUnitRows * t.tm - 1;  // a short tile draws no rows it does not use
#pragma unroll
    for (int i = 0; i < G::XBLOCKS; ++i) {
      // block j = wave + 8 i of the slab: rows 8j..8j+7 (128-byte rows) / 16j..16j+15 (64-byte rows); the 16-byte chunk c of
      // row r is stored at chunk position c ^ swizzle(r), applied by choosing which global chunk a lane fetches, so that
      // the 16 rows a quarter-wavefront reads at one K offset fall into 16 different bank groups.  Rows past the end of X
      // or of a short tile re-read the last row they may (their results are never stored).
      const int j = wave + 8 * i;
      int r, c;
      if constexpr (DENSE) {
        r = 16 * j + (l >> 2);
        c = (l & 3) ^ ((r >> 2) & 3);
      } else {
        r = 8 * j + (l >> 3);
        c = (l & 7) ^ ((r >> 1) & 7);
      }
      const int64_t rr = r < last ? r : last;
      pf_xoff[i] = (uint32_t)(rr * k_bytes + c * 16);
    }
    pf_x = Xg + t.m0 * k_bytes;
    if constexpr (DENSE) {
      const int n_tile = t.n_blk * kTileBN;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int f = wave + 8 * i;  // fragment of the tile; its row l % 16 is this channel (packed_row_to_channel)
        int ch = 64 * (f >> 2) + packed_row_to_channel(f & 3, l & 15);
        ch = n_tile + ch < a.N ? ch : a.N - 1 - n_tile;  // channels past the end re-read the last row
        pf_woff[i] = (uint32_t)((int64_t)ch * k_bytes + 16 * (l >> 4));
      }
      pf_w = Wg + (int64_t)n_tile * k_bytes;
    } else {
      pf_woff[0] = (uint32_t)l * 16u;
      pf_woff[1] = (uint32_t)l * 16u + 8192u;
      pf_w = Wg + (int64_t)t.n_blk * ksteps * tile_bytes(IS_I8) + wave_lds;
    }
  };
  auto advance = [&]() {
    if (pf_ks + 1 < ksteps) {
      ++pf_ks;
      pf_x += G::STEP;
      pf_w += DENSE ? G::STEP : tile_bytes(IS_I8);
    } else if (pf_item + 1 < my_items) {
      seek(pf_item + 1);
    } else {
      pf_more = false;
    }
  };
  auto request_step = [&](uint32_t stage_lds) {
    const uint32_t base = stage_lds + wave_lds;
    copy16_to_lds_at<0>(pf_x, pf_xoff[0], base);
    if constexpr (G::XBLOCKS == 2) copy16_to_lds_at<8192>(pf_x, pf_xoff[G::XBLOCKS - 1], base);
    copy16_to_lds_at<G::XSLAB>(pf_w, pf_woff[0], base);
    copy16_to_lds_at<G::XSLAB + 8192>(pf_w, pf_woff[1], base);
    if constexpr (!DENSE) {
      if (wave < G::IDX_BLOCKS) copy16_to_lds_at<G::XSLAB + kTileValueBytes>(pf_w, pf_woff[0] + (uint32_t)kTileValueBytes, base);
    }
  };

  acc_t acc[kTileTN][kT2TM];
  const uint32_t a_off = (uint32_t)(G::XSLAB + wn * kTileTN * kFragValueBytes + lane * 16);
  const uint32_t i_off = DENSE ? 0u : (uint32_t)(G::XSLAB + index_offset(IS_I8, wn * kTileTN, lane));

  request_constants(tile_of(0).n_blk * kTileBN + wn * (kTileTN * 16));
  seek(0);
  request_step(ring_lds);
  advance();

  int stage = 0;          // ring stage of the current K step
  int stores_behind = 0;  // output stores this wavefront issued behind the copies of the coming step
  for (int item = 0; item < my_items; ++item) {
    const Tile t = tile_of(item);
    int l = lane;
    asm volatile("" : "+v"(l));  // the offsets are computed here, per tile, not once per kernel and kept (or spilled)
    const int c16 = l & 15, q = l >> 4;
    // per-lane byte offset of the B operand inside an X slab: row wm * 16 tm + 16 mt + c16, chunk q (and 4 + q) at its
    // swizzled position
    uint32_t b_lo, b_hi = 0;
    if constexpr (DENSE) {
      b_lo = (uint32_t)(wm * t.tm * 16 + c16) * G::STEP + (uint32_t)((q ^ ((c16 >> 2) & 3)) * 16);
    } else {
      const int sw = c16 >> 1;
      b_lo = (uint32_t)(wm * t.tm * 16 + c16) * G::STEP + (uint32_t)((q ^ sw) * 16);
      b_hi = (uint32_t)(wm * t.tm * 16 + c16) * G::STEP + (uint32_t)(((4 + q) ^ sw) * 16);
    }
#pragma unroll
    for (int i = 0; i < kTileTN; ++i)
#pragma unroll
      for (int j = 0; j < kT2TM; ++j) acc[i][j] = acc_t{0, 0, 0, 0};

    auto k_loop = [&](auto tma) {
      constexpr int TMA = decltype(tma)::value;
      for (int ks = 0; ks < ksteps; ++ks) {
        __builtin_amdgcn_sched_barrier(0);
        wait_copies_behind_stores(ks == 0 ? stores_behind : 0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");  // no LDS read moves above the barrier
        // behind the barrier: every wavefront has left the previous tile's epilogue, so its constants may be replaced
        if (ks == 0 && item > 0) request_constants(t.n_blk * kTileBN + wn * (kTileTN * 16));
        if (pf_more) {
          request_step(ring_lds + (uint32_t)((stage ^ 1) * G::STAGE));
          advance();
        }
        const uint8_t* st = ring + stage * G::STAGE;
        b_t b[TMA];
#pragma unroll
        for (int mt = 0; mt < TMA; ++mt) {
          if constexpr (DENSE) {
            b[mt] = *(const v4i*)(st + b_lo + mt * 16 * G::STEP);
          } else {
            const v4i lo = *(const v4i*)(st + b_lo + mt * 16 * G::STEP), hi = *(const v4i*)(st + b_hi + mt * 16 * G::STEP);
            b[mt] = v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          }
        }
        int ai[kTileTN];
        if constexpr (!DENSE) {
          load_index_half<IS_I8>(ai, 0, st + i_off);
          load_index_half<IS_I8>(ai, 1, st + i_off);
        }
        // The fragments are read three ahead of the matrix instructions that use them, each into registers of its own
        // (left to itself the compiler reads every fragment into the same registers and waits for each in turn), and the
        // reads are pinned between the matrix instructions so that every other instruction issues in the shadow of one.
        v4i av[4];
#pragma unroll
        for (int f = 0; f < 3; ++f) av[f] = *(const v4i*)(st + a_off + f * kFragValueBytes);
#pragma unroll
        for (int tn = 0; tn < kTileTN; ++tn) {
#pragma unroll
          for (int mt = 0; mt < TMA; ++mt) {
            if (mt == 0 && tn + 3 < kTileTN) av[(tn + 3) & 3] = *(const v4i*)(st + a_off + (tn + 3) * kFragValueBytes);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (DENSE)
              acc[tn][mt] = mfma_dense<IS_I8>(av[tn & 3], b[mt], acc[tn][mt]);
            else
              acc[tn][mt] = smfmac<IS_I8>(av[tn & 3], b[mt], acc[tn][mt], ai[tn]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        stage ^= 1;
      }
    };
    if (t.tm == 2)
      k_loop(std::integral_constant<int, 2>{});
    else
      k_loop(std::integral_constant<int, 1>{});
    if (ksteps == 1 && item > 0) {
      // a single step has no later barrier that publishes the tile's constants (requested behind its only barrier)
      __builtin_amdgcn_s_waitcnt(0x0070);
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    }

    const int n_wave = t.n_blk * kTileBN + wn * (kTileTN * 16);
    const int64_t m_wave = t.m0 + wm * t.tm * 16;
    const int64_t rows = (int64_t)a.M - m_wave;
    const int chans = a.N - n_wave;
    const bool lines = OUT == GPUSQ_F16 ? (a.N & 7) == 0 : (OUT == GPUSQ_I8 ? (a.N & 15) == 0 : true);
    stores_behind = 0;
    if (lines) {
      if (t.tm == kT2TM && rows >= kT2TM * 16 && chans >= kTileTN * 16) {
        line_epilogue<IS_I8, GELU, OUT, false, kT2TM>(a, acc, prm[wn], s_a, s_out, r_out, n_wave, m_wave, lane, kT2TM);
        // store instructions of a wavefront whose 128 channels x 32 rows all lie inside Y: per 16-row slab two per line of
        // its 128 channels (fp16: 2 lines, int8: 1, int32: 4)
        stores_behind = kT2TM * 2 * (OUT == GPUSQ_F16 ? 2 : (OUT == GPUSQ_I8 ? 1 : 4));
      } else {
        line_epilogue<IS_I8, GELU, OUT, true, kT2TM>(a, acc, prm[wn], s_a, s_out, r_out, n_wave, m_wave, lane, t.tm);
      }
    } else {
      batch_epilogue<IS_I8, GELU, OUT, kT2TM>(a, acc, prm[wn], s_a, n_wave, m_wave, lane, t.tm);
    }
  }
}

// ---------------------------------------------------------------------------------------------------------- host side
// Estimated run time (microseconds) of one tile of 64 * tm rows on a CU that it shares with a second workgroup.
static double tile2_cost(int tm, int ksteps, bool gelu, bool dense) {
  const double step = dense ? 0.22 + 0.16 * tm : 0.30 + 0.20 * tm;
  return ksteps * step + (gelu ? 1.3 : 0.9) * tm + 0.3;
}

static double tile2_makespan(const TilePlan& p, int grid, int ksteps, bool gelu, bool dense) {
  const int W = grid / 8;
  const double cf = tile2_cost(p.full_tm, ksteps, gelu, dense), ct = tile2_cost(p.tail_tm, ksteps, gelu, dense);
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

static int tile2_grid(const TilePlan& p, int resident) { return (int)ceil_div(p.total < resident ? p.total : resident, 8) * 8; }

// Full tiles of 128 (or 64) rows for as many whole rounds over the resident workgroups (two per CU) as the problem has,
// the remaining rows in tail tiles of 128 or 64 rows; the candidate whose busiest workgroup finishes first.
TilePlan make_tile2_plan(int M, int N, int resident, int ksteps, bool gelu, bool dense) {
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
    const int64_t rows_left = (int64_t)M - (int64_t)full_chunks * kTileUnitRows * ftm;
    p.total = p.full_tiles + (rows_left > 0 ? (int)ceil_div(rows_left, kTileUnitRows * ttm) * tiles_n : 0);
    p.inv_tiles_n = (tiles_n > 1 && tiles_n <= 4096 && p.total < (1 << 20)) ? (uint32_t)((((uint64_t)1 << 32) + tiles_n - 1) / tiles_n) : 0u;
    const double c = tile2_makespan(p, tile2_grid(p, resident), ksteps, gelu, dense);
    if (best_cost < 0 || c < best_cost) {
      best_cost = c;
      best = p;
    }
  };
  for (int ftm = kT2TM; ftm >= 1; --ftm) {
    const int chunks = (int)ceil_div(M, kTileUnitRows * ftm);
    consider(ftm, chunks, ftm);
    const int all_tiles = chunks * tiles_n;
    if (all_tiles > resident && all_tiles % resident != 0) {
      const int full_chunks = (all_tiles / resident) * resident / tiles_n;
      for (int ttm = ftm; ttm >= 1; --ttm) consider(ftm, full_chunks, ttm);
    }
  }
  return best;
}

int tile2_grid_of(const TilePlan& p, int resident) { return tile2_grid(p, resident); }

bool tile2_supports(bool is_i8, bool dense, const GemmArgs& a) {
  const int64_t k_bytes = (int64_t)a.K * (is_i8 ? 1 : 2);
  const int step = dense ? 64 : kStepBytes;
  if (k_bytes % step != 0 || a.patch_P != 0 || a.x_f16) return false;
  if (127 * k_bytes + step >= ((int64_t)1 << 32)) return false;                   // 32-bit lane offsets inside a tile's rows of X
  if (dense && 255 * k_bytes + step >= ((int64_t)1 << 32)) return false;          // and inside its rows of W
  if ((int64_t)a.N * 16 * 4 >= ((int64_t)1 << 31)) return false;                  // 32-bit lane offsets inside 16 rows of Y
  return true;
}

template <bool IS_I8, bool DENSE>
static gpusq_status launch_tile2_typed(const GemmArgs& a, const TilePlan& plan, int grid, hipStream_t s) {
  const bool gelu = (a.epilogue & GPUSQ_EPI_GELU) != 0;
  const dim3 g((unsigned)grid);
  if constexpr (IS_I8) {
    if (a.out_dt == GPUSQ_I32)
      gemm_tile2_kernel<true, DENSE, 0, GPUSQ_I32><<<g, 512, 0, s>>>(a, plan);
    else if (a.out_dt == GPUSQ_I8 && gelu)
      gemm_tile2_kernel<true, DENSE, 1, GPUSQ_I8><<<g, 512, 0, s>>>(a, plan);
    else if (a.out_dt == GPUSQ_I8)
      gemm_tile2_kernel<true, DENSE, 0, GPUSQ_I8><<<g, 512, 0, s>>>(a, plan);
    else if (gelu)
      gemm_tile2_kernel<true, DENSE, 1, GPUSQ_F16><<<g, 512, 0, s>>>(a, plan);
    else
      gemm_tile2_kernel<true, DENSE, 0, GPUSQ_F16><<<g, 512, 0, s>>>(a, plan);
  } else {
    if (gelu)
      gemm_tile2_kernel<false, DENSE, 1, GPUSQ_F16><<<g, 512, 0, s>>>(a, plan);
    else
      gemm_tile2_kernel<false, DENSE, 0, GPUSQ_F16><<<g, 512, 0, s>>>(a, plan);
  }
  return check_launch();
}

gpusq_status launch_tile2(bool is_i8, bool dense, const GemmArgs& a, const TilePlan& plan, int grid, hipStream_t s) {
  if (dense) return is_i8 ? launch_tile2_typed<true, true>(a, plan, grid, s) : launch_tile2_typed<false, true>(a, plan, grid, s);
  return is_i8 ? launch_tile2_typed<true, false>(a, plan, grid, s) : launch_tile2_typed<false, false>(a, plan, grid, s);
}

}  // namespace gpusq
