// Fused epilogue shared by the sparse and dense GEMM kernels: dequantise, bias, GELU, convert, store.
#pragma once
#include "common.h"

namespace gpusq {

typedef int ep_v4i __attribute__((ext_vector_type(4)));
typedef int ep_v2i __attribute__((ext_vector_type(2)));
typedef unsigned ep_v2u __attribute__((ext_vector_type(2)));
typedef _Float16 ep_v8h __attribute__((ext_vector_type(8)));
typedef _Float16 ep_v4h __attribute__((ext_vector_type(4)));

// Exact-erf GELU, GELU(x) = x * Phi(x), evaluated as  max(x, 0) - t * Phi(-t),  t = |x|, with Phi(-t) = 2^P(t) and P a
// degree-5 polynomial fitted to log2 Phi(-t) on [0, 6.5] (weighted so that the result is within 0.15 fp16 ulp of the
// exact value everywhere, including the negative tail down to fp16 subnormals).  Beyond 6.5 P keeps falling
// monotonically (to -inf for large t), so the subtracted term stays below 3e-10 there and no clamp of t is needed
// for finite x; x = +-inf gives NaN.
// One transcendental (v_exp_f32) and eight full-rate VALU operations per element: the fp32 epilogue of a GEMM whose
// output is written in fp16 is VALU-limited on this chip, so the library erf (dozens of operations) is not an option.
constexpr float kGeluP5 = -0.0003336848458275199f, kGeluP4 = 0.005954924505203962f, kGeluP3 = -0.04866418614983559f,
                kGeluP2 = -0.46354809403419495f, kGeluP1 = -1.149438738822937f, kGeluP0 = -1.0001022815704346f;

__device__ __forceinline__ float gelu_f32(float x) {
  const float t = fabsf(x);
  float p = __fmaf_rn(t, kGeluP5, kGeluP4);
  p = __fmaf_rn(p, t, kGeluP3);
  p = __fmaf_rn(p, t, kGeluP2);
  p = __fmaf_rn(p, t, kGeluP1);
  p = __fmaf_rn(p, t, kGeluP0);
  const float q = __builtin_amdgcn_exp2f(p);
  return __fmaf_rn(-t, q, fmaxf(x, 0.0f));
}

// Pins 8 values in registers at this point of the instruction stream (an empty volatile asm that "modifies" them): the
// instructions that produce them cannot be moved below it, sunk into a later conditional block, or merged with the
// instructions that consume them.
__device__ __forceinline__ void pin8(float (&x)[8]) {
  asm volatile("" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]));
}

// The same function on 8 values at once, written stage by stage so that the 8 dependency chains interleave: a lone
// wavefront on a SIMD then issues an independent instruction every slot instead of waiting on each result.  The pins
// between the stages keep the compiler from folding the chains back into pairs (which it does to save registers).
__device__ __forceinline__ void gelu_f32_x8(float (&v)[8]) {
  float p[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) p[j] = __fmaf_rn(fabsf(v[j]), kGeluP5, kGeluP4);
  pin8(p);
#pragma unroll
  for (int j = 0; j < 8; ++j) p[j] = __fmaf_rn(p[j], fabsf(v[j]), kGeluP3);
  pin8(p);
#pragma unroll
  for (int j = 0; j < 8; ++j) p[j] = __fmaf_rn(p[j], fabsf(v[j]), kGeluP2);
  pin8(p);
#pragma unroll
  for (int j = 0; j < 8; ++j) p[j] = __fmaf_rn(p[j], fabsf(v[j]), kGeluP1);
  pin8(p);
#pragma unroll
  for (int j = 0; j < 8; ++j) p[j] = __fmaf_rn(p[j], fabsf(v[j]), kGeluP0);
  pin8(p);
#pragma unroll
  for (int j = 0; j < 8; ++j) p[j] = __builtin_amdgcn_exp2f(p[j]);
  pin8(p);
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = __fmaf_rn(-fabsf(v[j]), p[j], fmaxf(v[j], 0.0f));
  pin8(v);
}

// Per-channel epilogue constants of a workgroup's output channels, staged in LDS: c[n] = act_scale * w_scale[n]
// (1 on the FP16 path) and b[n] = bias[n] (0 when there is no bias, which leaves fma(x, c, 0) == x * c and
// acc + 0 == acc bit for bit).  fetch() issues the global loads early (one channel per thread), publish() writes
// them to LDS; the caller puts a barrier between publish() and the first read.
struct ChannelParams {
  float c, b;
  template <bool IS_I8>
  __device__ __forceinline__ void fetch(const GemmArgs& a, int n) {
    const bool ok = n < a.N;
    const bool raw_out = IS_I8 && a.out_dt == GPUSQ_I32;
    c = 1.0f;
    b = 0.0f;
    if (IS_I8 && !raw_out && ok) c = a.act_scale[0] * a.w_scale[n];
    if ((a.epilogue & GPUSQ_EPI_BIAS) && !raw_out && ok) b = a.bias[n];
  }
  __device__ __forceinline__ void publish(float* cs, float* bs, int i) const {
    cs[i] = c;
    bs[i] = b;
  }
};

// INT8 path: v = fma((float)acc, c, b); FP16 path: v = acc + b.  Then optional GELU.
template <bool IS_I8>
__device__ __forceinline__ float epilogue_value(int raw, float accf, float c, float b, bool use_gelu) {  // use_gelu: uniform
  float v;
  if constexpr (IS_I8)
    v = __fmaf_rn((float)raw, c, b);
  else
    v = accf + b;
  return use_gelu ? gelu_f32(v) : v;
}

// Converts and stores 8 consecutive output channels [n, n+8) of one activation row held by one lane; `yp` points at
// the element (row, n) of Y.
// N % 4 == 0 is guaranteed by the host, so each half of 4 channels is entirely inside or outside the matrix and
// 4-channel stores are naturally aligned; with N % 8 == 0 the 8 channels go out in one store.
// STREAM: give that 16-byte fp16 store the non-temporal hint.  Y is written once and not read again, and in the tile
// kernel (operands re-read by every tile through the L2) the hint keeps Y from pushing the operands out of the L2:
// measured there, it cuts the HBM reads by 40% and the run time by 8%.  It is a measured choice per kernel and store
// shape: the same hint makes the dense kernel's stores, and narrower or strided stores (int8 / int32 output), markedly
// slower.
// OUT: output dtype fixed at compile time (a gpusq_dtype value), or -1 to take it from the arguments at run time.
template <bool IS_I8, int OUT = -1, bool STREAM = false>
__device__ __forceinline__ void store_8_at(const GemmArgs& a, void* yp, int n, const float (&v)[8], const int (&raw)[8]) {
  const int N = a.N;
  const int out_dt = OUT >= 0 ? OUT : a.out_dt;
  if (n >= N) return;
  const bool whole = (N & 7) == 0;  // then n + 8 <= N as well, because n is a multiple of 8
  const bool second = n + 8 <= N;
  if (IS_I8 && out_dt == GPUSQ_I32) {
    int* y = (int*)yp;
    *(ep_v4i*)y = ep_v4i{raw[0], raw[1], raw[2], raw[3]};
    if (second) *(ep_v4i*)(y + 4) = ep_v4i{raw[4], raw[5], raw[6], raw[7]};
  } else if (IS_I8 && out_dt == GPUSQ_I8) {
    const float so = a.out_scale[0], rso = scale_reciprocal(so);  // the same code rule as the quantiser of the activations
    int8_t* y = (int8_t*)yp;
    int q[8];
    quantize_codes<8>(v, so, rso, q);
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] &= 0xFF;
    const int lo = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24), hi = q[4] | (q[5] << 8) | (q[6] << 16) | (q[7] << 24);
    if (whole) {
      *(ep_v2i*)y = ep_v2i{lo, hi};
    } else {
      *(int*)y = lo;
      if (second) *(int*)(y + 4) = hi;
    }
  } else {
    _Float16* y = (_Float16*)yp;
    // The fp32 value is rounded to fp32 before it is rounded to fp16: without the pin the compiler may fuse the last
    // fp32 operation with the conversion (v_fma_mix*), which rounds once and differs in rare last bits.
    float w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = v[j];
    pin8(w);
    if (whole) {
      ep_v8h h;
#pragma unroll
      for (int j = 0; j < 8; ++j) h[j] = (_Float16)w[j];
      if constexpr (STREAM)
        __builtin_nontemporal_store(h, (ep_v8h*)y);
      else
        *(ep_v8h*)y = h;
    } else {
      *(ep_v4h*)y = ep_v4h{(_Float16)w[0], (_Float16)w[1], (_Float16)w[2], (_Float16)w[3]};
      if (second) *(ep_v4h*)(y + 4) = ep_v4h{(_Float16)w[4], (_Float16)w[5], (_Float16)w[6], (_Float16)w[7]};
    }
  }
}

__host__ __device__ constexpr int dtype_bytes(int dt) { return dt == GPUSQ_I8 ? 1 : (dt == GPUSQ_F16 ? 2 : 4); }

// The same with the address computed from the row m and channel n.
template <bool IS_I8, int OUT = -1>
__device__ __forceinline__ void store_8(const GemmArgs& a, int64_t m, int n, const float (&v)[8], const int (&raw)[8]) {
  const int out_dt = OUT >= 0 ? OUT : a.out_dt;
  store_8_at<IS_I8, OUT>(a, (uint8_t*)a.Y + (m * a.N + n) * dtype_bytes(out_dt), n, v, raw);
}

}  // namespace gpusq
