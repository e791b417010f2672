// Weight / activation preparation kernels: 2:4 pruning, symmetric INT8 quantisation, compression to kept values +
// 2-bit metadata, decompression, and re-tiling into the kernel-native packed format.
// All of them stream their operands once and are bound by HBM bandwidth; work is laid out wavefront-parallel over
// groups of 4 (one lane per group or per pair of groups), with 16-byte accesses where the layout allows.
#include <atomic>

#include "common.h"

namespace gpusq {

// ------------------------------------------------------------------------------------------------------------ prune
__global__ void __launch_bounds__(256) prune_f32_kernel(const float4* __restrict__ in, float4* __restrict__ out,
                                                        uint8_t* __restrict__ mask, int64_t groups) {
  const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= groups) return;
  const float4 w = in[g];
  const unsigned m = keep_mask_of_4(__float_as_uint(w.x) & 0x7FFFFFFFu, __float_as_uint(w.y) & 0x7FFFFFFFu,
                                    __float_as_uint(w.z) & 0x7FFFFFFFu, __float_as_uint(w.w) & 0x7FFFFFFFu);
  float4 o;
  o.x = (m & 1u) ? w.x : 0.0f;
  o.y = (m & 2u) ? w.y : 0.0f;
  o.z = (m & 4u) ? w.z : 0.0f;
  o.w = (m & 8u) ? w.w : 0.0f;
  out[g] = o;
  if (mask) mask[g] = (uint8_t)m;
}

__global__ void __launch_bounds__(256) prune_f16_kernel(const uint2* __restrict__ in, uint2* __restrict__ out,
                                                        uint8_t* __restrict__ mask, int64_t groups) {
  const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= groups) return;
  const uint2 w = in[g];
  const unsigned h0 = w.x & 0xFFFFu, h1 = w.x >> 16, h2 = w.y & 0xFFFFu, h3 = w.y >> 16;
  const unsigned m = keep_mask_of_4(h0 & 0x7FFFu, h1 & 0x7FFFu, h2 & 0x7FFFu, h3 & 0x7FFFu);
  uint2 o;
  o.x = ((m & 1u) ? h0 : 0u) | (((m & 2u) ? h1 : 0u) << 16);
  o.y = ((m & 4u) ? h2 : 0u) | (((m & 8u) ? h3 : 0u) << 16);
  out[g] = o;
  if (mask) mask[g] = (uint8_t)m;
}

gpusq_status launch_prune(const void* Win, void* Wout, uint8_t* mask, gpusq_dtype dt, int64_t N, int64_t K, hipStream_t s) {
  const int64_t groups = N * K / 4;
  const unsigned blocks = (unsigned)ceil_div(groups, 256);
  if (dt == GPUSQ_F32)
    prune_f32_kernel<<<blocks, 256, 0, s>>>((const float4*)Win, (float4*)Wout, mask, groups);
  else
    prune_f16_kernel<<<blocks, 256, 0, s>>>((const uint2*)Win, (uint2*)Wout, mask, groups);
  return check_launch();
}

// ------------------------------------------------------------------------------------------------------------ cast
__global__ void __launch_bounds__(256) cast_f16_kernel(const float* __restrict__ in, _Float16* __restrict__ out, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
  for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < n; i += stride) {
    if (i + 3 < n) {
      const float4 v = *(const float4*)(in + i);
      typedef _Float16 h4 __attribute__((ext_vector_type(4)));
      *(h4*)(out + i) = h4{(_Float16)v.x, (_Float16)v.y, (_Float16)v.z, (_Float16)v.w};
    } else {
      for (int64_t j = i; j < n; ++j) out[j] = (_Float16)in[j];
    }
  }
}

// ---- patch embedding: images [B][C][H][W] -> flattened patches X [B*(H/P)*(W/P)][K_pad] (Sec. 3.3) ------------------------
// Row m = (b, py, px) of X holds patch (py, px) of image b, column k = (c*P + i)*P + j holds pixel (py*P + i, px*P + j) of
// channel c (the order of a convolution weight [D][C][P][P] flattened along its last three axes); columns C*P*P..K_pad-1
// are zero.  One thread moves VEC consecutive columns, which lie in one image row when P % VEC == 0.
template <typename T, int VEC>
__global__ void __launch_bounds__(256) im2col_patches_kernel(const T* __restrict__ img, T* __restrict__ X, int C, int H, int W, int P,
                                                             int K, int K_pad, int64_t units) {
  typedef T vec_t __attribute__((ext_vector_type(VEC)));
  const int kv = K_pad / VEC, px_n = W / P, py_n = H / P;
  for (int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x; u < units; u += (int64_t)gridDim.x * 256) {
    const int64_t m = u / kv;
    const int k0 = (int)(u - m * kv) * VEC;
    vec_t v = vec_t(0);
    if (k0 < K) {
      const int c = k0 / (P * P), r = k0 - c * P * P, i = r / P, j = r - i * P;
      const int px = (int)(m % px_n), py = (int)((m / px_n) % py_n);
      const int64_t b = m / ((int64_t)px_n * py_n);
      const T* src = img + ((b * C + c) * H + (int64_t)py * P + i) * W + (int64_t)px * P + j;
      if constexpr (VEC == 1)
        v = vec_t(*src);
      else
        v = *(const vec_t*)src;
    }
    *(vec_t*)(X + m * K_pad + k0) = v;
  }
}

// The same for patch sizes whose rows are not multiples of 16 bytes (P = 14): one workgroup per (image, channel, row of
// patches).  The P image rows of that strip are one contiguous span of P*W elements: it is read into LDS with 4-byte
// loads, and written out as W/P runs of P*P consecutive columns (one per patch), 4 bytes per thread and store, each word
// gathered from LDS.  The workgroups of channel 0 also zero the padding columns of their rows.
// Needs (W * sizeof(T)) % 4 == 0, (P*P * sizeof(T)) % 4 == 0, (K_pad * sizeof(T)) % 4 == 0 and a span of at most 48 KB.
template <typename T>
__global__ void __launch_bounds__(256) im2col_strip_kernel(const T* __restrict__ img, T* __restrict__ X, int C, int H, int W, int P,
                                                           int K, int K_pad) {
  extern __shared__ __attribute__((aligned(16))) uint8_t strip_raw[];
  T* strip = (T*)strip_raw;
  constexpr int EPW = 4 / (int)sizeof(T);  // elements per 4-byte word
  const int py_n = H / P, px_n = W / P;
  const int py = blockIdx.x % py_n, c = (blockIdx.x / py_n) % C;
  const int64_t b = blockIdx.x / (py_n * C);
  const int span_words = P * W / EPW;
  const uint32_t* src = (const uint32_t*)(img + ((b * C + c) * H + (int64_t)py * P) * W);
  for (int q = threadIdx.x; q < span_words; q += 256) ((uint32_t*)strip)[q] = src[q];
  __syncthreads();
  const int wpr = P * P / EPW;  // words per run
  const int64_t m0 = (b * py_n + py) * px_n;
  for (int q = threadIdx.x; q < span_words; q += 256) {
    const int px = q / wpr, rq = q - px * wpr;
    T e[EPW];
#pragma unroll
    for (int t = 0; t < EPW; ++t) {
      const int r = rq * EPW + t, i = r / P, j = r - i * P;
      e[t] = strip[i * W + px * P + j];
    }
    uint32_t word;
    __builtin_memcpy(&word, e, 4);
    *(uint32_t*)(X + (m0 + px) * K_pad + (int64_t)c * P * P + rq * EPW) = word;
  }
  if (c == 0) {
    const int pad_words = (K_pad - K) / EPW;
    for (int q = threadIdx.x; q < pad_words * px_n; q += 256) {
      const int px = q / pad_words, w = q - px * pad_words;
      *(uint32_t*)(X + (m0 + px) * K_pad + K + w * EPW) = 0u;
    }
  }
}

template <typename T>
static gpusq_status launch_im2col_typed(const T* img, T* X, int64_t B, int64_t C, int64_t H, int64_t W, int64_t P, int64_t K_pad,
                                        hipStream_t s) {
  const int64_t M = B * (H / P) * (W / P);
  const int K = (int)(C * P * P);
  // the widest power-of-two move (up to 16 bytes) for which every source and destination address is aligned: it must
  // divide P (a move stays inside one image row and pixel offsets are multiples of it), W and K_pad
  int vec = 16 / (int)sizeof(T);
  while (vec > 1 && (P % vec != 0 || W % vec != 0 || K_pad % vec != 0)) vec >>= 1;
  const int64_t span_bytes = P * W * (int64_t)sizeof(T);
  if (vec * sizeof(T) < 16 && (W * sizeof(T)) % 4 == 0 && (P * P * sizeof(T)) % 4 == 0 && (K_pad * sizeof(T)) % 4 == 0 &&
      (K * sizeof(T)) % 4 == 0 && span_bytes <= 48 * 1024 && B * C * (H / P) <= INT32_MAX) {
    im2col_strip_kernel<T><<<(unsigned)(B * C * (H / P)), 256, (size_t)span_bytes, s>>>(img, X, (int)C, (int)H, (int)W, (int)P, K, (int)K_pad);
    return check_launch();
  }
  const int64_t units = M * (K_pad / vec);
  const int64_t want = ceil_div(units, 256);
  const unsigned grid = (unsigned)(want < 16384 ? want : 16384);
#define GPUSQ_IM2COL_CASE(V) \
  case V:                    \
    im2col_patches_kernel<T, V><<<grid, 256, 0, s>>>(img, X, (int)C, (int)H, (int)W, (int)P, K, (int)K_pad, units); \
    break;
  switch (vec) {
    GPUSQ_IM2COL_CASE(16)
    GPUSQ_IM2COL_CASE(8)
    GPUSQ_IM2COL_CASE(4)
    GPUSQ_IM2COL_CASE(2)
    default:
      im2col_patches_kernel<T, 1><<<grid, 256, 0, s>>>(img, X, (int)C, (int)H, (int)W, (int)P, K, (int)K_pad, units);
      break;
  }
#undef GPUSQ_IM2COL_CASE
  return check_launch();
}

gpusq_status launch_im2col_patches(const void* img, void* X, gpusq_dtype dt, int64_t B, int64_t C, int64_t H, int64_t W, int64_t P,
                                   int64_t K_pad, hipStream_t s) {
  if (dt == GPUSQ_I8) return launch_im2col_typed<int8_t>((const int8_t*)img, (int8_t*)X, B, C, H, W, P, K_pad, s);
  return launch_im2col_typed<_Float16>((const _Float16*)img, (_Float16*)X, B, C, H, W, P, K_pad, s);
}

gpusq_status launch_cast_f16(const float* in, void* out, int64_t n, hipStream_t s) {
  const int64_t want = ceil_div(n, 256 * 4);
  cast_f16_kernel<<<(unsigned)(want < 8192 ? want : 8192), 256, 0, s>>>(in, (_Float16*)out, n);
  return check_launch();
}

// n:m pruning [Sec. 5, limitation paragraph: 1:4, 2:16]: the n largest magnitudes of every M contiguous elements are kept
// (ties: the lower index).  One thread per group; an element is kept iff fewer than n elements beat it.
template <int M>
__global__ void __launch_bounds__(256) prune_n_of_m_kernel(const float4* __restrict__ in, float4* __restrict__ out, int n_keep,
                                                           int64_t groups) {
  const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= groups) return;
  float v[M];
#pragma unroll
  for (int q = 0; q < M / 4; ++q) {
    const float4 w = in[g * (M / 4) + q];
    v[4 * q] = w.x; v[4 * q + 1] = w.y; v[4 * q + 2] = w.z; v[4 * q + 3] = w.w;
  }
  unsigned key[M];
#pragma unroll
  for (int i = 0; i < M; ++i) key[i] = __float_as_uint(v[i]) & 0x7FFFFFFFu;
#pragma unroll
  for (int i = 0; i < M; ++i) {
    int beaten = 0;
#pragma unroll
    for (int j = 0; j < M; ++j)
      if (j != i) beaten += (j < i) ? (key[j] >= key[i]) : (key[j] > key[i]);
    if (beaten >= n_keep) v[i] = 0.0f;
  }
#pragma unroll
  for (int q = 0; q < M / 4; ++q) out[g * (M / 4) + q] = float4{v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]};
}

gpusq_status launch_prune_n_of_m(const float* Win, float* Wout, int n_keep, int m, int64_t N, int64_t K, hipStream_t s) {
  const int64_t groups = N * (K / m);
  const unsigned blocks = (unsigned)ceil_div(groups, 256);
  if (m == 4)
    prune_n_of_m_kernel<4><<<blocks, 256, 0, s>>>((const float4*)Win, (float4*)Wout, n_keep, groups);
  else if (m == 8)
    prune_n_of_m_kernel<8><<<blocks, 256, 0, s>>>((const float4*)Win, (float4*)Wout, n_keep, groups);
  else
    prune_n_of_m_kernel<16><<<blocks, 256, 0, s>>>((const float4*)Win, (float4*)Wout, n_keep, groups);
  return check_launch();
}

// ------------------------------------------------------------------------------------------------------------ quantise
__device__ __forceinline__ float load_as_f32(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float load_as_f32(const _Float16* p, int64_t i) { return (float)p[i]; }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// One wavefront per row (= per output channel), 4 rows per workgroup.
template <typename T>
__global__ void __launch_bounds__(256) quantize_rows_kernel(const T* __restrict__ X, int8_t* __restrict__ Q,
                                                            float* __restrict__ scale, int scale_is_input,
                                                            int64_t rows, int64_t cols, float qmax) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* x = X + row * cols;
  float s;
  if (scale_is_input) {
    s = scale[row];
  } else {
    float amax = 0.0f;
    for (int64_t c = lane; c < cols; c += 64) amax = fmaxf(amax, fabsf(load_as_f32(x, c)));
    amax = wave_max(amax);
    s = (amax == 0.0f) ? 1.0f : __fdiv_rn(amax, qmax);
    if (lane == 0) scale[row] = s;
  }
  const float rs = scale_reciprocal(s);
  int8_t* q = Q + row * cols;
  if ((cols & 3) == 0) {
    for (int64_t c = (int64_t)lane * 4; c < cols; c += 256) {
      const float xs[4] = {load_as_f32(x, c), load_as_f32(x, c + 1), load_as_f32(x, c + 2), load_as_f32(x, c + 3)};
      int qc[4];
      quantize_codes<4>(xs, s, rs, qc, qmax);
      *(uint32_t*)(q + c) = (uint32_t)(qc[0] & 0xFF) | ((uint32_t)(qc[1] & 0xFF) << 8) | ((uint32_t)(qc[2] & 0xFF) << 16) |
                            ((uint32_t)(qc[3] & 0xFF) << 24);
    }
  } else {
    for (int64_t c = lane; c < cols; c += 64) q[c] = (int8_t)quantize_code(load_as_f32(x, c), s, rs, qmax);
  }
}

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v) { *p = v; }

constexpr int kAmaxMaxBlocks = 1024;  // per-block partial maxima kept in the caller's workspace (4 KB)

// 8 consecutive elements as fp32, one 16-byte (fp16) or two 16-byte (fp32) loads
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const _Float16* p, float (&v)[8]) {
  typedef _Float16 h8 __attribute__((ext_vector_type(8)));
  const h8 a = *(const h8*)p;
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = (float)a[j];
}

__device__ __forceinline__ float block_max(float v) {
  __shared__ float part[4];
  v = wave_max(v);
  __syncthreads();  // a previous use of part[] has been read
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
}

// per-tensor max |x|, first pass: every workgroup streams its share with 16-byte loads and leaves one partial
// maximum in the workspace; the quantising pass folds the partials (no atomics, nothing to clear beforehand)
template <typename T>
__global__ void __launch_bounds__(256) tensor_amax_kernel(const T* __restrict__ X, int64_t n, float* __restrict__ partial) {
  float amax = 0.0f;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x * 8;
  for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 8; i < n; i += stride) {
    if (i + 8 <= n) {
      float v[8];
      load8(X + i, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(v[j]));
    } else {
      for (int64_t j = i; j < n; ++j) amax = fmaxf(amax, fabsf(load_as_f32(X, j)));
    }
  }
  amax = block_max(amax);
  if (threadIdx.x == 0) partial[blockIdx.x] = amax;
}

template <typename T>
__global__ void __launch_bounds__(256) quantize_tensor_kernel(const T* __restrict__ X, int8_t* __restrict__ Q,
                                                              float* __restrict__ scale, const float* __restrict__ partial,
                                                              int npartial, int64_t n) {
  float s;
  if (partial) {
    float amax = 0.0f;
    for (int i = threadIdx.x; i < npartial; i += 256) amax = fmaxf(amax, partial[i]);
    amax = block_max(amax);
    s = (amax == 0.0f) ? 1.0f : __fdiv_rn(amax, 127.0f);
    if (blockIdx.x == 0 && threadIdx.x == 0) scale[0] = s;
  } else {
    s = scale[0];
  }
  const float rs = scale_reciprocal(s);
  const int64_t stride = (int64_t)gridDim.x * blockDim.x * 8;
  for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 8; i < n; i += stride) {
    if (i + 8 <= n) {
      float v[8];
      load8(X + i, v);
      unsigned lo, hi;
      quantize_bytes8(v, s, rs, lo, hi);  // the same codes as quantize_codes with about half the arithmetic
      *(uint2*)(Q + i) = uint2{lo, hi};
    } else {
      for (int64_t j = i; j < n; ++j) Q[j] = (int8_t)quantize_code(load_as_f32(X, j), s, rs);
    }
  }
}

template <typename T>
static gpusq_status quantize_typed(const T* X, int8_t* Xq, float* scale, int mode, int scale_is_input, int64_t rows,
                                   int64_t cols, void* workspace, hipStream_t s) {
  if (mode == GPUSQ_PER_ROW) {
    quantize_rows_kernel<T><<<(unsigned)ceil_div(rows, 4), 256, 0, s>>>(X, Xq, scale, scale_is_input, rows, cols, 127.0f);
    return check_launch();
  }
  const int64_t n = rows * cols;
  const int64_t want = ceil_div(n, 256 * 8 * 2);  // two 8-element vectors per thread ...
  // ... up to 2048 workgroups (every workgroup of the quantising pass first reduces the partial maxima: with 8192 of them the
  // pass took 1.5 us longer on 12608 x 768 activations, with 1024 or fewer the large tensors slow down)
  const unsigned blocks_q = (unsigned)(want < 2048 ? want : 2048);
  const unsigned blocks_a = (unsigned)(want < kAmaxMaxBlocks ? want : kAmaxMaxBlocks);
  const float* partial = nullptr;
  if (!scale_is_input) {
    tensor_amax_kernel<T><<<blocks_a, 256, 0, s>>>(X, n, (float*)workspace);
    partial = (const float*)workspace;
  }
  quantize_tensor_kernel<T><<<blocks_q, 256, 0, s>>>(X, Xq, scale, partial, (int)blocks_a, n);
  return check_launch();
}

gpusq_status launch_quantize(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int mode, int scale_is_input,
                             int64_t rows, int64_t cols, void* workspace, hipStream_t s) {
  if (dt == GPUSQ_F32) return quantize_typed<float>((const float*)X, Xq, scale, mode, scale_is_input, rows, cols, workspace, s);
  return quantize_typed<_Float16>((const _Float16*)X, Xq, scale, mode, scale_is_input, rows, cols, workspace, s);
}

// ---- per-tensor quantiser for callers that cannot allocate -------------------------------------------------------
// The per-workgroup partial maxima of the range pass live in this file-scope device array instead of a caller's
// workspace.  Every GPU the library runs on holds its own copy until the process ends; its address on a device is
// looked up once per device (hipGetSymbolAddress with that device current) and kept.  The array's name is only a
// host-side handle: host code passes the looked-up pointer to the kernels, never the name.
static __device__ __align__(256) float g_amax_scratch[kAmaxMaxBlocks];

static float* amax_scratch_of_current_device(gpusq_status* st) {
  constexpr int kMaxDevices = 64;
  static std::atomic<float*> ptrs[kMaxDevices];
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    if (e != hipSuccess) set_last_hip_error(e);
    *st = e != hipSuccess ? GPUSQ_ERR_HIP : GPUSQ_ERR_UNSUPPORTED;
    return nullptr;
  }
  float* p = ptrs[dev].load(std::memory_order_acquire);
  if (!p) {
    void* sym = nullptr;
    e = hipGetSymbolAddress(&sym, HIP_SYMBOL(g_amax_scratch));
    if (e != hipSuccess || !sym) {
      set_last_hip_error(e);
      *st = GPUSQ_ERR_HIP;
      return nullptr;
    }
    p = (float*)sym;
    ptrs[dev].store(p, std::memory_order_release);  // (a racing first call looks up the same address)
  }
  *st = GPUSQ_OK;
  return p;
}

gpusq_status launch_quantize_tensor_static(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int scale_is_input,
                                           int64_t rows, int64_t cols, hipStream_t s) {
  float* scratch = nullptr;
  if (!scale_is_input) {  // a given scale needs no range pass and no scratch
    gpusq_status st;
    scratch = amax_scratch_of_current_device(&st);
    if (!scratch) return st;
  }
  // Nothing has to be cleared: the range pass overwrites the partial maxima the quantising pass reads (the same
  // number of them in both launches), whatever an earlier call left behind.
  return launch_quantize(X, dt, Xq, scale, GPUSQ_PER_TENSOR, scale_is_input, rows, cols, scratch, s);
}

// The same per-row quantiser with the 4-bit range: codes -7..7 in int8 containers, scale = max|row| / 7.
gpusq_status launch_quantize_rows_int4(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int scale_is_input, int64_t rows,
                                       int64_t cols, hipStream_t s) {
  const unsigned blocks = (unsigned)ceil_div(rows, 4);
  if (dt == GPUSQ_F32)
    quantize_rows_kernel<float><<<blocks, 256, 0, s>>>((const float*)X, Xq, scale, scale_is_input, rows, cols, 7.0f);
  else
    quantize_rows_kernel<_Float16><<<blocks, 256, 0, s>>>((const _Float16*)X, Xq, scale, scale_is_input, rows, cols, 7.0f);
  return check_launch();
}

// ------------------------------------------------------------------------------------------------------------ compress
// One lane per metadata byte = per pair of groups (the last byte of a row holds one group when K/4 is odd).
template <typename T>
__device__ __forceinline__ unsigned magnitude_key(T v);
template <>
__device__ __forceinline__ unsigned magnitude_key<uint32_t>(uint32_t v) { return v & 0x7FFFFFFFu; }
template <>
__device__ __forceinline__ unsigned magnitude_key<uint16_t>(uint16_t v) { return v & 0x7FFFu; }
template <>
__device__ __forceinline__ unsigned magnitude_key<int8_t>(int8_t v) { return (unsigned)(v < 0 ? -(int)v : (int)v); }

template <typename T>
__global__ void __launch_bounds__(256) compress_kernel(const T* __restrict__ W, T* __restrict__ values,
                                                       uint8_t* __restrict__ meta, int32_t* __restrict__ violations,
                                                       int64_t N, int64_t K) {
  const int64_t groups_per_row = K / 4;
  const int64_t mrb = (groups_per_row + 1) / 2;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int bad = 0;
  if (id < N * mrb) {
    const int64_t n = id / mrb, b = id % mrb;
    unsigned byte = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int64_t g = 2 * b + h;
      if (g < groups_per_row) {
        const T* w = W + n * K + 4 * g;
        const T w0 = w[0], w1 = w[1], w2 = w[2], w3 = w[3];
        const unsigned k0 = magnitude_key<T>(w0), k1 = magnitude_key<T>(w1), k2 = magnitude_key<T>(w2), k3 = magnitude_key<T>(w3);
        const unsigned m = keep_mask_of_4(k0, k1, k2, k3);
        const unsigned nib = nibble_of_mask(m);
        const unsigned p0 = nib & 3u, p1 = nib >> 2;
        const T v0 = p0 == 0 ? w0 : (p0 == 1 ? w1 : w2);
        const T v1 = p1 == 1 ? w1 : (p1 == 2 ? w2 : w3);
        values[n * (K / 2) + 2 * g] = v0;
        values[n * (K / 2) + 2 * g + 1] = v1;
        byte |= nib << (4 * h);
        bad += (int)(((m & 1u) == 0 && k0 != 0) || ((m & 2u) == 0 && k1 != 0) || ((m & 4u) == 0 && k2 != 0) ||
                     ((m & 8u) == 0 && k3 != 0));
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

gpusq_status launch_compress(const void* W, void* values, uint8_t* meta, int32_t* violations, gpusq_dtype dt,
                             int64_t N, int64_t K, hipStream_t s) {
  const int64_t mrb = (K / 4 + 1) / 2;
  const unsigned blocks = (unsigned)ceil_div(N * mrb, 256);
  if (violations) fill_u32_kernel<<<1, 1, 0, s>>>((uint32_t*)violations, 0u);
  if (dt == GPUSQ_F16)
    compress_kernel<uint16_t><<<blocks, 256, 0, s>>>((const uint16_t*)W, (uint16_t*)values, meta, violations, N, K);
  else
    compress_kernel<int8_t><<<blocks, 256, 0, s>>>((const int8_t*)W, (int8_t*)values, meta, violations, N, K);
  return check_launch();
}

// Groups of 4 along K with more than two non-zero elements (Sec. 3.1: a 2:4 tensor keeps at most two of every four).
// One thread per 16 bytes of a row (4 groups of fp32 ... 16 of int8: K % 4 == 0 makes rows whole groups, the pointer is
// 16-byte aligned, and the tail of the tensor that does not fill 16 bytes goes element by element); -0 counts as zero.
template <typename T>
__global__ void __launch_bounds__(256) count_violations_kernel(const T* __restrict__ W, int32_t* __restrict__ violations, int64_t elems) {
  constexpr int PER = 16 / (int)sizeof(T);  // elements per 16-byte piece: whole groups
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t e0 = id * PER;
  int bad = 0;
  if (e0 < elems) {
    alignas(16) T w[PER];
    if (e0 + PER <= elems) {
      *(uint4*)w = *(const uint4*)(W + e0);
    } else {
      for (int i = 0; i < PER; ++i) w[i] = e0 + i < elems ? W[e0 + i] : (T)0;
    }
#pragma unroll
    for (int g = 0; g < PER / 4; ++g) {
      int nz = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) nz += (int)(magnitude_key<T>(w[4 * g + i]) != 0u);
      bad += (int)(nz > 2);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) bad += __shfl_xor(bad, o, 64);
  if ((threadIdx.x & 63) == 0 && bad) atomicAdd(violations, bad);
}

gpusq_status launch_count_violations(const void* W, gpusq_dtype dt, int32_t* violations, int64_t N, int64_t K, hipStream_t s) {
  const int64_t elems = N * K;
  fill_u32_kernel<<<1, 1, 0, s>>>((uint32_t*)violations, 0u);
  if (dt == GPUSQ_F32)
    count_violations_kernel<uint32_t><<<(unsigned)ceil_div(ceil_div(elems, 4), 256), 256, 0, s>>>((const uint32_t*)W, violations, elems);
  else if (dt == GPUSQ_F16)
    count_violations_kernel<uint16_t><<<(unsigned)ceil_div(ceil_div(elems, 8), 256), 256, 0, s>>>((const uint16_t*)W, violations, elems);
  else
    count_violations_kernel<int8_t><<<(unsigned)ceil_div(ceil_div(elems, 16), 256), 256, 0, s>>>((const int8_t*)W, violations, elems);
  return check_launch();
}

template <typename T>
__global__ void __launch_bounds__(256) decompress_kernel(const T* __restrict__ values, const uint8_t* __restrict__ meta,
                                                         T* __restrict__ W, int64_t N, int64_t K) {
  const int64_t groups_per_row = K / 4;
  const int64_t mrb = (groups_per_row + 1) / 2;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= N * mrb) return;
  const int64_t n = id / mrb, b = id % mrb;
  const unsigned byte = meta[n * mrb + b];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int64_t g = 2 * b + h;
    if (g < groups_per_row) {
      const unsigned nib = (byte >> (4 * h)) & 0xFu;
      const unsigned p0 = nib & 3u, p1 = nib >> 2;
      const T v0 = values[n * (K / 2) + 2 * g], v1 = values[n * (K / 2) + 2 * g + 1];
      T* w = W + n * K + 4 * g;
#pragma unroll
      for (unsigned i = 0; i < 4; ++i) w[i] = (i == p0) ? v0 : ((i == p1) ? v1 : (T)0);
    }
  }
}

gpusq_status launch_decompress(const void* values, const uint8_t* meta, void* W, gpusq_dtype dt, int64_t N, int64_t K,
                               hipStream_t s) {
  const int64_t mrb = (K / 4 + 1) / 2;
  const unsigned blocks = (unsigned)ceil_div(N * mrb, 256);
  if (dt == GPUSQ_F16)
    decompress_kernel<uint16_t><<<blocks, 256, 0, s>>>((const uint16_t*)values, meta, (uint16_t*)W, N, K);
  else
    decompress_kernel<int8_t><<<blocks, 256, 0, s>>>((const int8_t*)values, meta, (int8_t*)W, N, K);
  return check_launch();
}

// ------------------------------------------------------------------------------------------------------------ pack
// Re-tiles the canonical (values, meta) arrays into the packed tile format described in common.h.
// Lane l of fragment f (0..15) of tile (nb, ks) serves output channel nb*256 + 64*(f/4) + packed_row_to_channel(f%4,
// l%16) and the dense K range [ks*E + (l/16)*E/4, +E/4) with E = elements per step; the sparse matrix instruction
// wants, per lane, the kept values of that range in order (16 bytes) and their 2-bit positions in order starting at
// bit 0 of the index register.  Both are contiguous byte runs of the canonical arrays:
// values[n][k0/2 .. k0/2 + kept) and meta[n][k0/8 ..).  Rows >= N and K beyond the row end are zero-filled.
template <bool IS_I8>
__global__ void __launch_bounds__(256) pack_kernel(const uint8_t* __restrict__ values, const uint8_t* __restrict__ meta,
                                                   uint8_t* __restrict__ packed, int64_t N, int64_t K, int64_t ksteps,
                                                   int64_t total_lanes) {
  constexpr int E = step_elems(IS_I8);  // dense elements per step
  constexpr int ES = IS_I8 ? 1 : 2;     // element size
  constexpr int KL = E / 4;             // dense elements per lane
  constexpr int IB = IS_I8 ? 4 : 2;     // index bytes per lane
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= total_lanes) return;
  const int lane = (int)(id & 63);
  const int f = (int)((id >> 6) & 15);
  const int64_t tile = id >> 10;
  const int64_t ks = tile % ksteps, nb = tile / ksteps;
  const int64_t n = nb * kTileRows + (f >> 2) * kRowBlock + packed_row_to_channel(f & 3, lane & 15);
  const int64_t k0 = ks * E + (int64_t)(lane >> 4) * KL;  // first dense element of this lane
  const int64_t mrb = (K / 4 + 1) / 2;
  uint8_t v[16];
  uint8_t ix[IB];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int64_t byte = (k0 / 2) * ES + i;  // byte offset inside the row of kept values
    v[i] = (n < N && byte < (K / 2) * ES) ? values[n * (K / 2) * ES + byte] : (uint8_t)0;
  }
#pragma unroll
  for (int i = 0; i < IB; ++i) {
    const int64_t byte = k0 / 8 + i;
    // padding (rows >= N, K beyond the row end) carries zero values; its positions are irrelevant
    ix[i] = (n < N && byte < mrb) ? meta[n * mrb + byte] : (uint8_t)0;
  }
  uint8_t* t = packed + tile * tile_bytes(IS_I8);
  uint4 vv;
  vv.x = v[0] | (v[1] << 8) | (v[2] << 16) | ((uint32_t)v[3] << 24);
  vv.y = v[4] | (v[5] << 8) | (v[6] << 16) | ((uint32_t)v[7] << 24);
  vv.z = v[8] | (v[9] << 8) | (v[10] << 16) | ((uint32_t)v[11] << 24);
  vv.w = v[12] | (v[13] << 8) | (v[14] << 16) | ((uint32_t)v[15] << 24);
  *(uint4*)(t + f * kFragValueBytes + lane * 16) = vv;
  uint8_t* ip = t + index_offset(IS_I8, f, lane);
  if constexpr (IS_I8)
    *(uint32_t*)ip = ix[0] | (ix[1] << 8) | (ix[2] << 16) | ((uint32_t)ix[3] << 24);
  else
    *(uint16_t*)ip = (uint16_t)(ix[0] | (ix[1] << 8));
}

gpusq_status launch_pack(const void* values, const uint8_t* meta, void* packed, gpusq_dtype dt, int64_t N, int64_t K,
                         hipStream_t s) {
  const bool is_i8 = dt == GPUSQ_I8;
  const int64_t ksteps = ceil_div(K, step_elems(is_i8));
  const int64_t tiles = ceil_div(N, kTileRows) * ksteps;
  const int64_t total_lanes = tiles * 16 * 64;
  const unsigned blocks = (unsigned)ceil_div(total_lanes, 256);
  if (is_i8)
    pack_kernel<true><<<blocks, 256, 0, s>>>((const uint8_t*)values, meta, (uint8_t*)packed, N, K, ksteps, total_lanes);
  else
    pack_kernel<false><<<blocks, 256, 0, s>>>((const uint8_t*)values, meta, (uint8_t*)packed, N, K, ksteps, total_lanes);
  return check_launch();
}

// ------------------------------------------------------------------------------------------------------------ fused
// prune -> (INT8: per-output-channel quantise | FP16: round) -> compress -> pack for one weight matrix in one launch.
// One workgroup per output channel.  Phase 1 streams the fp32 row into LDS and reduces max|w| (pruning never removes
// the row maximum, so this is also the maximum of the pruned row).  Phase 2 gives each thread one "lane unit" of the
// packed format: the 32 (INT8) or 16 (FP16) consecutive dense elements whose kept values fill one lane's 16 value
// bytes and 4 (2) index bytes; the thread prunes its groups of 4, quantises or rounds them, applies the compression
// rule to the low-precision group, and writes the unit to every requested output.  All arithmetic is the same
// sequence of operations as the separate kernels above, so the results are bit-identical to running them in turn.
// A workgroup handles `rows_per_block` (1, 2, 4 or 8) consecutive channels with 256 / rows_per_block threads each, so
// that short rows (K = 768 has only 24 lane units) still keep most of the workgroup busy.
template <bool IS_I8>
__global__ void __launch_bounds__(256) prepare_weights_kernel(const float* __restrict__ W, float* __restrict__ Wp,
                                                              uint8_t* __restrict__ Wlow, float* __restrict__ w_scale,
                                                              uint8_t* __restrict__ values, uint8_t* __restrict__ meta,
                                                              uint8_t* __restrict__ packed, int64_t N, int64_t K, int64_t ksteps,
                                                              int rows_per_block) {
  extern __shared__ float rows_lds[];  // rows_per_block rows of K floats
  __shared__ float red[256];
  constexpr int E = step_elems(IS_I8), ES = IS_I8 ? 1 : 2, KL = E / 4, IB = IS_I8 ? 4 : 2;
  const int tpr = 256 / rows_per_block;         // threads per row
  const int lr = (int)threadIdx.x / tpr;        // local row
  const int tr = (int)threadIdx.x % tpr;        // thread within the row
  const int64_t n = (int64_t)blockIdx.x * rows_per_block + lr;
  const bool live = n < N;
  float* row = rows_lds + (int64_t)lr * K;
  float amax = 0.0f;
  if (live) {
    const float* w = W + n * K;
    for (int64_t k = (int64_t)tr * 4; k < K; k += (int64_t)tpr * 4) {
      const float4 v = *(const float4*)(w + k);
      *(float4*)(row + k) = v;
      amax = fmaxf(fmaxf(amax, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
  }
  float s = 1.0f;
  if constexpr (IS_I8) {  // max over the row's threads (any order gives the same maximum), through LDS
    red[threadIdx.x] = amax;
    __syncthreads();  // also publishes the rows
    for (int h = tpr >> 1; h > 0; h >>= 1) {
      if (tr < h) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + h]);
      __syncthreads();
    }
    amax = red[lr * tpr];
    s = (amax == 0.0f) ? 1.0f : __fdiv_rn(amax, 127.0f);
    if (live && tr == 0) w_scale[n] = s;
  } else {
    __syncthreads();
  }
  if (!live) return;
  const float rs = scale_reciprocal(s);
  const int64_t mrb = (K / 4 + 1) / 2;
  const int64_t units = (K + KL - 1) / KL;
  // packed position of this channel: tile nb, fragment f, row r of the fragment
  const int64_t nb = n / kTileRows;
  const int in_tile = (int)(n % kTileRows), blk = in_tile / kRowBlock, c64 = in_tile % kRowBlock;
  // inverse of packed_row_to_channel: c64 = 32*(t/2) + 8*(r/4) + 4*(t%2) + r%4
  const int t = 2 * (c64 >> 5) + ((c64 >> 2) & 1), r = 4 * ((c64 >> 3) & 3) + (c64 & 3);
  const int f = blk * 4 + t;
  for (int64_t u = tr; u < units; u += tpr) {
    const int64_t k0 = u * KL;
    uint8_t vbytes[16];
    uint8_t ibytes[IB];
#pragma unroll
    for (int i = 0; i < 16; ++i) vbytes[i] = 0;
#pragma unroll
    for (int i = 0; i < IB; ++i) ibytes[i] = 0;
#pragma unroll
    for (int g = 0; g < KL / 4; ++g) {
      const int64_t k = k0 + 4 * g;
      if (k < K) {
        const float4 x = *(const float4*)(row + k);
        const unsigned m = keep_mask_of_4(__float_as_uint(x.x) & 0x7FFFFFFFu, __float_as_uint(x.y) & 0x7FFFFFFFu,
                                          __float_as_uint(x.z) & 0x7FFFFFFFu, __float_as_uint(x.w) & 0x7FFFFFFFu);
        float4 p;
        p.x = (m & 1u) ? x.x : 0.0f; p.y = (m & 2u) ? x.y : 0.0f; p.z = (m & 4u) ? x.z : 0.0f; p.w = (m & 8u) ? x.w : 0.0f;
        if (Wp) *(float4*)(Wp + n * K + k) = p;
        unsigned nib;
        if constexpr (IS_I8) {
          const float ps[4] = {p.x, p.y, p.z, p.w};
          int qc[4];
          quantize_codes<4>(ps, s, rs, qc);
          const int q0 = qc[0], q1 = qc[1], q2 = qc[2], q3 = qc[3];
          if (Wlow) *(uint32_t*)(Wlow + n * K + k) = (uint32_t)(q0 & 0xFF) | ((uint32_t)(q1 & 0xFF) << 8) | ((uint32_t)(q2 & 0xFF) << 16) | ((uint32_t)(q3 & 0xFF) << 24);
          const unsigned mq = keep_mask_of_4((unsigned)abs(q0), (unsigned)abs(q1), (unsigned)abs(q2), (unsigned)abs(q3));
          nib = nibble_of_mask(mq);
          const unsigned p0 = nib & 3u, p1 = nib >> 2;
          vbytes[2 * g] = (uint8_t)(p0 == 0 ? q0 : (p0 == 1 ? q1 : q2));
          vbytes[2 * g + 1] = (uint8_t)(p1 == 1 ? q1 : (p1 == 2 ? q2 : q3));
        } else {
          const _Float16 h0 = (_Float16)p.x, h1 = (_Float16)p.y, h2 = (_Float16)p.z, h3 = (_Float16)p.w;
          const unsigned b0 = __builtin_bit_cast(unsigned short, h0), b1 = __builtin_bit_cast(unsigned short, h1);
          const unsigned b2 = __builtin_bit_cast(unsigned short, h2), b3 = __builtin_bit_cast(unsigned short, h3);
          if (Wlow) *(uint2*)(Wlow + (n * K + k) * 2) = uint2{b0 | (b1 << 16), b2 | (b3 << 16)};
          const unsigned mq = keep_mask_of_4(b0 & 0x7FFFu, b1 & 0x7FFFu, b2 & 0x7FFFu, b3 & 0x7FFFu);
          nib = nibble_of_mask(mq);
          const unsigned p0 = nib & 3u, p1 = nib >> 2;
          const unsigned v0 = p0 == 0 ? b0 : (p0 == 1 ? b1 : b2), v1 = p1 == 1 ? b1 : (p1 == 2 ? b2 : b3);
          vbytes[4 * g] = (uint8_t)v0; vbytes[4 * g + 1] = (uint8_t)(v0 >> 8);
          vbytes[4 * g + 2] = (uint8_t)v1; vbytes[4 * g + 3] = (uint8_t)(v1 >> 8);
        }
        ibytes[g >> 1] |= (uint8_t)(nib << (4 * (g & 1)));
      }
    }
    uint4 vv;
    vv.x = vbytes[0] | (vbytes[1] << 8) | (vbytes[2] << 16) | ((uint32_t)vbytes[3] << 24);
    vv.y = vbytes[4] | (vbytes[5] << 8) | (vbytes[6] << 16) | ((uint32_t)vbytes[7] << 24);
    vv.z = vbytes[8] | (vbytes[9] << 8) | (vbytes[10] << 16) | ((uint32_t)vbytes[11] << 24);
    vv.w = vbytes[12] | (vbytes[13] << 8) | (vbytes[14] << 16) | ((uint32_t)vbytes[15] << 24);
    const bool whole = k0 + KL <= K;
    if (values) {
      uint8_t* dst = values + (n * (K / 2) + k0 / 2) * ES;
      if (whole && ((K / 2) * ES) % 16 == 0) {  // rows of the values array are 16-byte aligned
        *(uint4*)dst = vv;
      } else {
        const int64_t nbytes = whole ? 16 : ((K - k0) / 2) * ES;
        for (int64_t i = 0; i < nbytes; ++i) dst[i] = vbytes[i];
      }
    }
    if (meta) {
      uint8_t* dst = meta + n * mrb + k0 / 8;
      const int64_t nbytes = whole ? IB : (mrb - k0 / 8);
      for (int64_t i = 0; i < nbytes; ++i) dst[i] = ibytes[i];
    }
    const int64_t ks = k0 / E;
    const int lane = r + 16 * (int)((k0 % E) / KL);
    uint8_t* tp = packed + (nb * ksteps + ks) * tile_bytes(IS_I8);
    *(uint4*)(tp + f * kFragValueBytes + lane * 16) = vv;
    uint8_t* ip = tp + index_offset(IS_I8, f, lane);
    if constexpr (IS_I8)
      *(uint32_t*)ip = ibytes[0] | (ibytes[1] << 8) | (ibytes[2] << 16) | ((uint32_t)ibytes[3] << 24);
    else
      *(uint16_t*)ip = (uint16_t)(ibytes[0] | (ibytes[1] << 8));
  }
}

// zero-fills the part of the packed buffer that no real channel / K range writes (rows >= N, K beyond the row end)
template <bool IS_I8>
__global__ void __launch_bounds__(256) clear_packed_padding_kernel(uint8_t* __restrict__ packed, int64_t N, int64_t K, int64_t ksteps,
                                                                   int64_t total_lanes) {
  constexpr int E = step_elems(IS_I8), KL = E / 4;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= total_lanes) return;
  const int lane = (int)(id & 63);
  const int f = (int)((id >> 6) & 15);
  const int64_t tile = id >> 10;
  const int64_t ks = tile % ksteps, nb = tile / ksteps;
  const int64_t n = nb * kTileRows + (f >> 2) * kRowBlock + packed_row_to_channel(f & 3, lane & 15);
  const int64_t k0 = ks * E + (int64_t)(lane >> 4) * KL;
  if (n < N && k0 < K) return;  // written by prepare_weights_kernel
  uint8_t* t = packed + tile * tile_bytes(IS_I8);
  *(uint4*)(t + f * kFragValueBytes + lane * 16) = uint4{0, 0, 0, 0};
  uint8_t* ip = t + index_offset(IS_I8, f, lane);
  if constexpr (IS_I8)
    *(uint32_t*)ip = 0u;
  else
    *(uint16_t*)ip = (uint16_t)0;
}

gpusq_status launch_prepare_weights(const float* W, gpusq_dtype dt, float* Wp, void* Wlow, float* w_scale, void* values,
                                    uint8_t* meta, void* packed, int64_t N, int64_t K, hipStream_t s) {
  const bool is_i8 = dt == GPUSQ_I8;
  const int64_t ksteps = ceil_div(K, step_elems(is_i8));
  // as many rows per workgroup as keep every row's threads busy (one thread per 32-byte lane unit) within 64 KB of LDS
  const int64_t units = ceil_div(K, step_elems(is_i8) / 4);
  int rpb = 1;
  while (rpb < 8 && 256 / (rpb * 2) >= units && (size_t)K * sizeof(float) * (rpb * 2) <= 64 * 1024) rpb *= 2;
  const size_t lds = (size_t)K * sizeof(float) * rpb;
  const unsigned grid = (unsigned)ceil_div(N, rpb);
  const bool padded = (N % kTileRows) != 0 || (K % step_elems(is_i8)) != 0;
  if (padded) {
    const int64_t total_lanes = ceil_div(N, kTileRows) * ksteps * 16 * 64;
    const unsigned blocks = (unsigned)ceil_div(total_lanes, 256);
    if (is_i8)
      clear_packed_padding_kernel<true><<<blocks, 256, 0, s>>>((uint8_t*)packed, N, K, ksteps, total_lanes);
    else
      clear_packed_padding_kernel<false><<<blocks, 256, 0, s>>>((uint8_t*)packed, N, K, ksteps, total_lanes);
  }
  if (is_i8)
    prepare_weights_kernel<true><<<grid, 256, lds, s>>>(W, Wp, (uint8_t*)Wlow, w_scale, (uint8_t*)values, meta, (uint8_t*)packed, N, K,
                                                        ksteps, rpb);
  else
    prepare_weights_kernel<false><<<grid, 256, lds, s>>>(W, Wp, (uint8_t*)Wlow, w_scale, (uint8_t*)values, meta, (uint8_t*)packed, N, K,
                                                         ksteps, rpb);
  return check_launch();
}

}  // namespace gpusq
