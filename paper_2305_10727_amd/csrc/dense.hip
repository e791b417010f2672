// Dense twin of the sparse GEMM: the same product computed from the masked but uncompressed weights on dense matrix
// instructions, the baseline of the "T cycles vs T/2 cycles" comparison of Sec. 3.1; it reads K bytes of W per output
// channel where the sparse kernel reads K/2 + K/8.
//
// Wherever the tile kernels can run the problem, the twin is the dense instantiation of the two-workgroup tile kernel
// (tile2.hip: same template, plan, launch path, LDS ring, fused epilogue and whole-line stores as its sparse
// instantiation), so that the sparse/dense ratio compares like with like.  The kernel in this file is the small one
// for the rest (few outputs, K that is not a whole number of 64-byte steps): 4 wavefronts, 64 x 128 or 128 x 128
// tiles, operands through registers into a double-buffered LDS stage, v_mfma_i32_32x32x32_i8 / v_mfma_f32_32x32x16_f16,
// the per-batch epilogue of epilogue.h.  It is a simpler pipeline than the sparse small kernel's and its times are not
// used for any sparse/dense ratio that the reports quote for the tile-kernel sizes.
//
// Register semantics of the 32x32 instructions (measured): A (4 VGPRs) lane l byte i -> row l%32, K index 16*(l/32)+i
// (8*(l/32)+i for fp16 elements); B likewise with column l%32; D (16 VGPRs) lane l register r -> row 8*(r/4) + 4*(l/32) +
// r%4, column l%32.
#include <atomic>

#include "tile_common.h"

namespace gpusq {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kLdsRowD = kStepBytes + 16;

template <bool IS_I8>
struct AccD { typedef v16f type; };
template <>
struct AccD<true> { typedef v16i type; };

template <bool IS_I8>
__device__ __forceinline__ typename AccD<IS_I8>::type mfma32(v4i a, v4i b, typename AccD<IS_I8>::type c) {
  if constexpr (IS_I8)
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
}

// LDS row of output channel c (0..63) inside a wavefront's 64-channel block.  Accumulator register r of lane half h
// in 32-row tile t is tile row 8*(r/4)+4h+r%4; placing channel 32t + 8*(r/4) + 4h... is the natural order, and we
// want instead that lane half h holds, in registers 8u..8u+7 of tile t, the 8 consecutive channels
// 32t + 16u + 8h .. +7: then a store of 8 channels per lane writes 16 contiguous bytes and the two lane halves 32.
__device__ __forceinline__ int lds_row_of_channel(int c) {
  const int t = c >> 5, u = (c >> 4) & 1, h = (c >> 3) & 1, r = 8 * u + (c & 7);
  return 32 * t + 8 * (r >> 2) + 4 * h + (r & 3);
}

// Workgroup = 4 wavefronts WN x WM; a wavefront owns 2 x TM accumulator tiles of 32 x 32 (64 channels x TM*32 rows).
template <bool IS_I8, int TM, int WN, int WM>
__global__ void __launch_bounds__(256) dense_kernel(const GemmArgs a, const int tiles_n, const int tiles_total) {
  static_assert(WN * WM == 4, "4 wavefronts");
  typedef typename AccD<IS_I8>::type acc_t;
  constexpr int BN = WN * 64, BM = WM * TM * 32;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int XCH = BM / 32, WCH = BN / 32;

  __shared__ __attribute__((aligned(16))) uint8_t Xs[2][BM * kLdsRowD];
  __shared__ __attribute__((aligned(16))) uint8_t Ws[2][BN * kLdsRowD];
  __shared__ __attribute__((aligned(16))) float cs[BN];
  __shared__ __attribute__((aligned(16))) float bs[BN];

  const int per_xcd = (tiles_total + 7) / 8;
  const int tile = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (tile >= tiles_total) return;
  const int n_blk = tile % tiles_n, m_blk = tile / tiles_n;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % WN, wm = wave / WN;
  const int M = a.M, N = a.N;
  const int64_t k_bytes = (int64_t)a.K * ES;
  const int ksteps = (int)((k_bytes + kStepBytes - 1) / kStepBytes);
  const uint8_t* Xg = (const uint8_t*)a.X;
  const uint8_t* Wg = (const uint8_t*)a.W;
  if (tid < BN) {
    ChannelParams prm;
    prm.fetch<IS_I8>(a, n_blk * BN + tid);
    prm.publish(cs, bs, tid);  // made visible by the barriers of the main loop
  }

  acc_t acc[2][TM];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  v4i xr[XCH], wr[WCH];
  auto load_tiles = [&](int ks) {
#pragma unroll
    for (int j = 0; j < XCH; ++j) {
      const int c = tid + 256 * j;
      const int64_t m = (int64_t)m_blk * BM + (c >> 3);
      const int64_t off = (int64_t)ks * kStepBytes + (c & 7) * 16;
      xr[j] = (m < M && off < k_bytes) ? *(const v4i*)(Xg + m * k_bytes + off) : v4i{0, 0, 0, 0};
    }
#pragma unroll
    for (int j = 0; j < WCH; ++j) {
      const int c = tid + 256 * j;
      const int64_t n = (int64_t)n_blk * BN + (c >> 3);
      const int64_t off = (int64_t)ks * kStepBytes + (c & 7) * 16;
      wr[j] = (n < N && off < k_bytes) ? *(const v4i*)(Wg + n * k_bytes + off) : v4i{0, 0, 0, 0};
    }
  };
  auto store_tiles = [&](int buf) {
#pragma unroll
    for (int j = 0; j < XCH; ++j) {
      const int c = tid + 256 * j;
      *(v4i*)(&Xs[buf][(c >> 3) * kLdsRowD + (c & 7) * 16]) = xr[j];
    }
#pragma unroll
    for (int j = 0; j < WCH; ++j) {
      const int c = tid + 256 * j;
      const int ch = c >> 3;  // channel inside the workgroup tile
      const int row = (ch & ~63) + lds_row_of_channel(ch & 63);
      *(v4i*)(&Ws[buf][row * kLdsRowD + (c & 7) * 16]) = wr[j];
    }
  };

  load_tiles(0);
  store_tiles(0);
  __syncthreads();

  const int l32 = lane & 31, h16 = (lane >> 5) * 16;
  for (int ks = 0; ks < ksteps; ++ks) {
    const int cur = ks & 1;
    const bool more = ks + 1 < ksteps;
    if (more) load_tiles(ks + 1);
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      v4i af[2], bf[TM];
#pragma unroll
      for (int t = 0; t < 2; ++t) af[t] = *(const v4i*)(&Ws[cur][(wn * 64 + 32 * t + l32) * kLdsRowD + 32 * sub + h16]);
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) bf[mt] = *(const v4i*)(&Xs[cur][((wm * TM + mt) * 32 + l32) * kLdsRowD + 32 * sub + h16]);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int mt = 0; mt < TM; ++mt) acc[t][mt] = mfma32<IS_I8>(af[t], bf[mt], acc[t][mt]);
    }
    if (more) store_tiles(cur ^ 1);
    __syncthreads();
  }

  // epilogue: lane half h holds, in registers 8u..8u+7 of tile t, channels n_wave + 32t + 16u + 8h .. +7
  const bool use_gelu = (a.epilogue & GPUSQ_EPI_GELU) != 0;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int n = n_blk * BN + wn * 64 + 32 * t + 16 * u + (lane >> 5) * 8;
      float c8[8], b8[8];
#pragma unroll
      for (int j = 0; j < 8; j += 4) {
        const float4 cc = *(const float4*)(cs + (n - n_blk * BN) + j), bb = *(const float4*)(bs + (n - n_blk * BN) + j);
        c8[j] = cc.x; c8[j + 1] = cc.y; c8[j + 2] = cc.z; c8[j + 3] = cc.w;
        b8[j] = bb.x; b8[j + 1] = bb.y; b8[j + 2] = bb.z; b8[j + 3] = bb.w;
      }
#pragma unroll
      for (int mt = 0; mt < TM; ++mt) {
        const int64_t m = (int64_t)m_blk * BM + (wm * TM + mt) * 32 + l32;
        float v[8];
        int raw[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if constexpr (IS_I8) {
            raw[j] = acc[t][mt][8 * u + j];
            v[j] = epilogue_value<true>(raw[j], 0.0f, c8[j], b8[j], use_gelu);
          } else {
            raw[j] = 0;
            v[j] = epilogue_value<false>(0, acc[t][mt][8 * u + j], c8[j], b8[j], use_gelu);
          }
        }
        if (m < M) store_8<IS_I8>(a, m, n, v, raw);
      }
    }
}

template <bool IS_I8, int TM, int WN, int WM>
static gpusq_status launch_cfg(const GemmArgs& a, hipStream_t s) {
  constexpr int BN = WN * 64, BM = WM * TM * 32;
  const int tiles_n = (int)ceil_div(a.N, BN), tiles_m = (int)ceil_div(a.M, BM);
  const int total = tiles_n * tiles_m;
  const int grid = (int)ceil_div(total, 8) * 8;
  dense_kernel<IS_I8, TM, WN, WM><<<grid, 256, 0, s>>>(a, tiles_n, total);
  return check_launch();
}

static int dense_cus() {
  static std::atomic<int> cus{0};
  int n = cus.load(std::memory_order_relaxed);
  if (n == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cus.store(n, std::memory_order_relaxed);
  }
  return n;
}

gpusq_status launch_dense(bool is_i8, const GemmArgs& a, hipStream_t s) {
  const int64_t work = (int64_t)a.M * a.N;
  // the twin of the sparse tile kernel (same template, same launch path) wherever that kernel can run the problem
  // (forcing the sparse GEMMs onto one of the small kernels, a testing aid, keeps the dense side on its small kernel too)
  const int forced = forced_kernel();
  if (work > (int64_t)256 * 1024 && forced != 0 && forced != 1 && tile2_supports(is_i8, true, a)) {
    const int resident = 2 * dense_cus();
    const int ksteps = (int)((int64_t)a.K * (is_i8 ? 1 : 2) / 64);
    const TilePlan plan = make_tile2_plan(a.M, a.N, resident, ksteps, (a.epilogue & GPUSQ_EPI_GELU) != 0, true);
    return launch_tile2(is_i8, true, a, plan, tile2_grid_of(plan, resident), s);
  }
  if (work <= (int64_t)256 * 1024)
    return is_i8 ? launch_cfg<true, 1, 1, 4>(a, s) : launch_cfg<false, 1, 1, 4>(a, s);  // 64 x 128 tiles
  return is_i8 ? launch_cfg<true, 2, 2, 2>(a, s) : launch_cfg<false, 2, 2, 2>(a, s);    // 128 x 128 tiles
}

}  // namespace gpusq
