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
#include "common.h"

namespace gpusq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v16h __attribute__((ext_vector_type(16)));

constexpr int kLdsRow = kStepBytes + 16;  // 144-byte row pitch: 16 rows x 16-byte reads hit 16 distinct bank groups

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

// exact-erf GELU, written with erfc so that the negative tail keeps its relative accuracy
__device__ __forceinline__ float gelu_f32(float v) { return 0.5f * v * erfcf(-0.70710678118654752f * v); }

__device__ __forceinline__ int requantize_code(float v, float s) {
  float r = rintf(__fdiv_rn(v, s));
  r = fminf(fmaxf(r, -127.0f), 127.0f);
  return (v != v) ? 0 : (int)r;
}

// Converts and stores the 16 consecutive output channels [n, n+16) a lane holds for activation row m.
template <bool IS_I8>
__device__ __forceinline__ void store_16(const GemmArgs& a, int64_t m, int n, const float (&v)[16], const int (&raw)[16]) {
  const int N = a.N;
  const bool full = n + 16 <= N;
  if (IS_I8 && a.out_dt == GPUSQ_I32) {
    int* y = (int*)a.Y + m * N + n;
    if (full) {  // N % 4 == 0 is checked on the host, so the row start is 16-byte aligned
#pragma unroll
      for (int j = 0; j < 4; ++j) *(v4i*)(y + 4 * j) = v4i{raw[4 * j], raw[4 * j + 1], raw[4 * j + 2], raw[4 * j + 3]};
    } else {
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (n + j < N) y[j] = raw[j];
    }
  } else if (IS_I8 && a.out_dt == GPUSQ_I8) {
    const float so = a.out_scale[0];
    int8_t* y = (int8_t*)a.Y + m * N + n;
    int q[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) q[j] = requantize_code(v[j], so) & 0xFF;
    if (full && (N & 15) == 0) {
      v4i pk;
#pragma unroll
      for (int j = 0; j < 4; ++j) pk[j] = q[4 * j] | (q[4 * j + 1] << 8) | (q[4 * j + 2] << 16) | (q[4 * j + 3] << 24);
      *(v4i*)y = pk;
    } else {
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (n + j < N) y[j] = (int8_t)q[j];
    }
  } else {
    _Float16* y = (_Float16*)a.Y + m * N + n;
    if (full && (N & 7) == 0) {
      v8h lo, hi;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        lo[j] = (_Float16)v[j];
        hi[j] = (_Float16)v[8 + j];
      }
      *(v8h*)y = lo;
      *(v8h*)(y + 8) = hi;
    } else {
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (n + j < N) y[j] = (_Float16)v[j];
    }
  }
}

// Workgroup = 4 wavefronts arranged WN (along n) x WM (along m); a wavefront owns TN x TM accumulator tiles.
// Workgroup tile: BN = WN*TN*16 output channels x BM = WM*TM*16 activation rows.
template <bool IS_I8, int TN, int TM, int WN, int WM>
__global__ void __launch_bounds__(256) spgemm_kernel(const GemmArgs a, const int tiles_n, const int tiles_total) {
  static_assert(WN * WM == 4 && TN % 4 == 0, "4 wavefronts; a wavefront spans whole 64-row blocks");
  typedef typename AccT<IS_I8>::type acc_t;
  constexpr int BN = WN * TN * 16, BM = WM * TM * 16;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int FB = frag_bytes(IS_I8);
  constexpr int XCH = BM / 32;  // 16-byte chunks of the X slab each thread moves per K step

  __shared__ __attribute__((aligned(16))) uint8_t Xs[2][BM * kLdsRow];

  // XCD-aware tile order: consecutive workgroup ids land on different XCDs (8 of them, each with its own L2), so
  // give every XCD one contiguous run of tiles; tiles that share an X slab (same m block) then share an L2.
  const int per_xcd = (tiles_total + 7) / 8;
  const int tile = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (tile >= tiles_total) return;
  const int n_blk = tile % tiles_n, m_blk = tile / tiles_n;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % WN, wm = wave / WN;
  const int M = a.M, N = a.N;
  const int64_t k_bytes = (int64_t)a.K * ES;
  const int ksteps = (int)((k_bytes + kStepBytes - 1) / kStepBytes);
  const int row_blocks = (N + kRowBlock - 1) / kRowBlock;
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
        const uint8_t* f = Wg + (((int64_t)rb * ksteps + ks) * 4 + (tn & 3)) * FB;
        av[slot][tn] = *(const v4i*)(f + lane * 16);
        if constexpr (IS_I8)
          ai[slot][tn] = *(const int*)(f + kFragValueBytes + lane * 4);
        else
          ai[slot][tn] = (int)*(const uint16_t*)(f + kFragValueBytes + lane * 2);
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

  // ---- epilogue: dequantise, bias, GELU, convert, store.  Lane (q = lane/16, c = lane%16) holds, for 64-row block
  // b and tile mt, the 16 channels n = n_wave + 64*b + 16*q + 4*t + r of activation row m = m_wave + 16*mt + c.
  const bool use_bias = (a.epilogue & GPUSQ_EPI_BIAS) != 0, use_gelu = (a.epilogue & GPUSQ_EPI_GELU) != 0;
  const bool raw_out = IS_I8 && a.out_dt == GPUSQ_I32;
  float s_a = 1.0f;
  if (IS_I8 && !raw_out) s_a = a.act_scale[0];
#pragma unroll
  for (int b = 0; b < TN / 4; ++b) {
    const int n = n_blk * BN + wn * TN * 16 + b * kRowBlock + (lane >> 4) * 16;
    if (n >= N) continue;
    float cs[16], bs[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const bool ok = n + j < N;
      cs[j] = (IS_I8 && !raw_out && ok) ? s_a * a.w_scale[n + j] : 1.0f;
      bs[j] = (use_bias && ok && !raw_out) ? a.bias[n + j] : 0.0f;
    }
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
      const int64_t m = (int64_t)m_blk * BM + (wm * TM + mt) * 16 + (lane & 15);
      if (m >= M) continue;
      float v[16];
      int raw[16];
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int j = 4 * t + r;
          if constexpr (IS_I8) {
            raw[j] = acc[4 * b + t][mt][r];
            const float f = (float)raw[j];
            v[j] = use_bias ? __fmaf_rn(f, cs[j], bs[j]) : f * cs[j];
          } else {
            raw[j] = 0;
            v[j] = acc[4 * b + t][mt][r] + bs[j];
          }
          if (use_gelu) v[j] = gelu_f32(v[j]);
        }
      store_16<IS_I8>(a, m, n, v, raw);
    }
  }
}

template <bool IS_I8, int TN, int TM, int WN, int WM>
static gpusq_status launch_cfg(const GemmArgs& a, hipStream_t s) {
  constexpr int BN = WN * TN * 16, BM = WM * TM * 16;
  const int tiles_n = (int)ceil_div(a.N, BN), tiles_m = (int)ceil_div(a.M, BM);
  const int total = tiles_n * tiles_m;
  const int grid = (int)ceil_div(total, 8) * 8;  // whole rounds over the 8 XCDs; surplus workgroups exit at once
  spgemm_kernel<IS_I8, TN, TM, WN, WM><<<grid, 256, 0, s>>>(a, tiles_n, total);
  return check_launch();
}

template <bool IS_I8>
static gpusq_status launch_typed(const GemmArgs& a, hipStream_t s) {
  const int64_t work = (int64_t)a.M * a.N;
  if (work <= (int64_t)256 * 1024) return launch_cfg<IS_I8, 4, 1, 1, 4>(a, s);  // 64 x 64 tiles: latency-bound sizes
  return launch_cfg<IS_I8, 4, 4, 2, 2>(a, s);                                  // 128 x 128 tiles
}

gpusq_status launch_spgemm(bool is_i8, const GemmArgs& a, hipStream_t s) {
  return is_i8 ? launch_typed<true>(a, s) : launch_typed<false>(a, s);
}

}  // namespace gpusq
