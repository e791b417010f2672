// Hardware probes for MI355X (gfx950): the measured denominators that the GEMM's roofline fractions are quoted against, and
// the in-CU facts the tile kernels were designed around.  Stand-alone program (no library needed except for the last
// section, which loops the c1 sparse GEMM through the C ABI while a one-wavefront kernel on a second stream samples the
// shader clock).  Prints one line per measurement and, with --json FILE, the same numbers as JSON.
//
//   matrix rates   register-only loops of 32 independent matrix instructions per wavefront, random operands, 8
//                  wavefronts per CU on every CU; timed with HIP events around the launch (a timestamp taken by one
//                  wavefront of a workgroup would only show that wavefront's share: the matrix pipe of a SIMD serves
//                  its wavefronts one instruction at a time, 16 clocks each for the 16x16 shapes, and the oldest first)
//   vector ALU     fp32 fma and the GELU epilogue's instruction mix on every CU, with the clock they run at
//   stream         copy and fill kernels on 512 MiB, 16 bytes per lane
//   LDS            ds_read_b128 from 16 wavefronts per CU, conflict-free and in the GEMM's swizzled B-operand pattern
//   copies         global_load_lds_dwordx4 from an L2-resident buffer, 16 wavefronts per CU
//   co-issue       a wavefront of matrix instructions and a wavefront of fp32 fma on one SIMD, alone and side by side
//   clock          wall_clock64 (100 MHz) against clock64 (shader clock) inside the kernels
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/gpusq.h"

#define CK(x)                                                                                   \
  do {                                                                                          \
    hipError_t e_ = (x);                                                                        \
    if (e_ != hipSuccess) {                                                                     \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);            \
      exit(1);                                                                                  \
    }                                                                                           \
  } while (0)

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v16h __attribute__((ext_vector_type(16)));

static std::string g_json;
static void emit(const char* key, double value, const char* unit, const char* note) {
  printf("%-44s %12.2f %-10s %s\n", key, value, unit, note);
  char buf[512];
  snprintf(buf, sizeof buf, "%s\n  \"%s\": {\"value\": %.4f, \"unit\": \"%s\", \"note\": \"%s\"}", g_json.empty() ? "" : ",", key, value, unit, note);
  g_json += buf;
}

// KIND 0: v_smfmac_i32_16x16x128_i8, 1: v_mfma_i32_16x16x64_i8, 2: v_smfmac_f32_16x16x64_f16, 3: v_mfma_f32_16x16x32_f16
template <int KIND, bool BARRIER>
__global__ void __launch_bounds__(512) matrix_rate(const int* __restrict__ src, int* __restrict__ out, long long* __restrict__ clk, int iters) {
  const int lane = threadIdx.x & 63;
  v4i a[8];
  v8i b[4];
  int idx[8];
  for (int i = 0; i < 8; ++i) {
    for (int j = 0; j < 4; ++j) a[i][j] = src[(i * 4 + j) * 64 + lane];
    idx[i] = src[(32 + i) * 64 + lane];
  }
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 8; ++j) b[i][j] = src[(48 + i * 8 + j) * 64 + lane];
  v4i acc[8][4];
  for (int i = 0; i < 8; ++i)
    for (int j = 0; j < 4; ++j) acc[i][j] = v4i{0, 0, 0, 0};
  __syncthreads();
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
    if (BARRIER) __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int tn = 0; tn < 8; ++tn)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        if (KIND == 0)
          acc[tn][mt] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(a[tn], b[mt], acc[tn][mt], idx[tn], 0, 0);
        else if (KIND == 1)
          acc[tn][mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[tn], v4i{b[mt][0], b[mt][1], b[mt][2], b[mt][3]}, acc[tn][mt], 0, 0, 0);
        else if (KIND == 2)
          acc[tn][mt] = __builtin_bit_cast(v4i, __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(v8h, a[tn]), __builtin_bit_cast(v16h, b[mt]),
                                                                                         __builtin_bit_cast(v4f, acc[tn][mt]), idx[tn] & 0xFFFF, 0, 0));
        else
          acc[tn][mt] = __builtin_bit_cast(v4i, __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a[tn]),
                                                                                       __builtin_bit_cast(v8h, v4i{b[mt][0], b[mt][1], b[mt][2], b[mt][3]}),
                                                                                       __builtin_bit_cast(v4f, acc[tn][mt]), 0, 0, 0));
      }
    __builtin_amdgcn_sched_barrier(0);
  }
  __syncthreads();  // the clocks below are those of the whole workgroup, not of its first wavefront
  const long long c1 = clock64(), w1 = wall_clock64();
  int s = 0;
  for (int i = 0; i < 8; ++i)
    for (int j = 0; j < 4; ++j) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0) {
    clk[2 * blockIdx.x] = c1 - c0;
    clk[2 * blockIdx.x + 1] = w1 - w0;
  }
}

template <int KIND, bool BARRIER>
static void run_matrix(const char* key, double ops_per_instr, const int* src, int* out, long long* clk, int wgs, int threads, const char* note) {
  const int iters = 2000;
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  matrix_rate<KIND, BARRIER><<<wgs, threads>>>(src, out, clk, iters);  // warm-up at full length: the clocks settle
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  matrix_rate<KIND, BARRIER><<<wgs, threads>>>(src, out, clk, iters);
  CK(hipEventRecord(e1));
  CK(hipDeviceSynchronize());
  float ms;
  CK(hipEventElapsedTime(&ms, e0, e1));
  std::vector<long long> h(2 * wgs);
  CK(hipMemcpy(h.data(), clk, sizeof(long long) * 2 * wgs, hipMemcpyDeviceToHost));
  double cs = 0, ws = 0;
  for (int i = 0; i < wgs; ++i) {
    cs += h[2 * i];
    ws += h[2 * i + 1];
  }
  const double waves = threads / 64.0, instr_per_simd = iters * 32.0 * waves / 4.0;
  char k[128], n[256];
  snprintf(k, sizeof k, "%s_rate", key);
  emit(k, (double)wgs * waves * iters * 32 * ops_per_instr / (ms * 1e-3) / 1e12, "Tops/s", note);
  snprintf(k, sizeof k, "%s_clocks_per_instruction_per_simd", key);
  emit(k, cs / wgs / instr_per_simd, "clk", "in-kernel shader clocks of the whole workgroup / instructions per SIMD");
  snprintf(k, sizeof k, "%s_shader_clock", key);
  snprintf(n, sizeof n, "clock64 / wall_clock64 x 100 MHz during the loop (%d workgroups of %d threads)", wgs, threads);
  emit(k, cs / ws * 100.0, "MHz", n);
}

// Vector ALU under load.  8 wavefronts per CU run 16 independent fp32 chains per lane.  MIX 0: fma only; MIX 1: the shape of
// the fused GELU epilogue per output (convert from int32, scale-and-bias fma, five fma of a polynomial, exp2, max, closing fma).
template <int MIX>
__global__ void __launch_bounds__(512) vector_rate(const int* __restrict__ src, int* __restrict__ out, long long* __restrict__ clk, int iters) {
  float f[16];
  int q[16];
  for (int i = 0; i < 16; ++i) {
    q[i] = src[(threadIdx.x + 64 * i) & 4095] & 0xfffff;
    f[i] = (float)(q[i] & 0xffff) * 1e-5f;
  }
  const float c = 0.999f + (float)(src[threadIdx.x & 63] & 1) * 1e-6f, b = 1e-3f;
  __syncthreads();
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (MIX == 0) {
#pragma unroll
        for (int r = 0; r < 8; ++r) f[i] = __builtin_fmaf(f[i], c, b);
      } else {
        const float x = __builtin_fmaf((float)(q[i] + it), c * 1e-5f, f[i] * 1e-3f - 3.0f);
        const float t = __builtin_fabsf(x);
        float p = __builtin_fmaf(t, -0.01f, 0.02f);
        p = __builtin_fmaf(p, t, -0.03f);
        p = __builtin_fmaf(p, t, -0.3f);
        p = __builtin_fmaf(p, t, -1.0f);
        p = __builtin_fmaf(p, t, -1.0f);
        f[i] = __builtin_fmaf(-t, __builtin_amdgcn_exp2f(p), __builtin_fmaxf(x, 0.0f));
      }
    }
  }
  __syncthreads();
  const long long c1 = clock64(), w1 = wall_clock64();
  float s = 0;
  for (int i = 0; i < 16; ++i) s += f[i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = (int)s;
  if (threadIdx.x == 0) {
    clk[2 * blockIdx.x] = c1 - c0;
    clk[2 * blockIdx.x + 1] = w1 - w0;
  }
}

template <int MIX>
static void run_vector(const char* key, double instr_per_iter, const int* src, int* out, long long* clk, int wgs, const char* note) {
  const int iters = 4000;
  vector_rate<MIX><<<wgs, 512>>>(src, out, clk, iters);  // warm-up at full length: the clocks settle
  CK(hipDeviceSynchronize());
  vector_rate<MIX><<<wgs, 512>>>(src, out, clk, iters);
  CK(hipDeviceSynchronize());
  std::vector<long long> h(2 * wgs);
  CK(hipMemcpy(h.data(), clk, sizeof(long long) * 2 * wgs, hipMemcpyDeviceToHost));
  double cs = 0, ws = 0;
  for (int i = 0; i < wgs; ++i) {
    cs += h[2 * i];
    ws += h[2 * i + 1];
  }
  char k[128];
  snprintf(k, sizeof k, "%s_clocks_per_instruction_per_simd", key);
  emit(k, cs / wgs / (iters * instr_per_iter * 2.0), "clk", note);  // 8 wavefronts per CU = 2 per SIMD
  snprintf(k, sizeof k, "%s_shader_clock", key);
  emit(k, cs / ws * 100.0, "MHz", "clock64 / wall_clock64 x 100 MHz during the loop, all CUs");
}

__global__ void __launch_bounds__(256) copy_kernel(const v4i* __restrict__ in, v4i* __restrict__ out, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) out[i] = in[i];
}
__global__ void __launch_bounds__(256) fill_kernel(v4i* __restrict__ out, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) out[i] = v4i{1, 2, 3, 4};
}

// PAT 0: contiguous 1 KB per wavefront; 1: 16 rows x 128-byte pitch, 16-byte chunk (q ^ (row >> 1)) -- the swizzled B operand of
// the sparse GEMM; 2: the same rows without the swizzle
template <int PAT>
__global__ void __launch_bounds__(1024) lds_rate(int* out, long long* clk, int iters) {
  __shared__ __attribute__((aligned(16))) char buf[64 * 1024];
  for (int i = threadIdx.x; i < 16 * 1024; i += blockDim.x) ((int*)buf)[i] = i;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int off;
  if (PAT == 0) {
    off = lane * 16;
  } else {
    const int c = lane & 15, q = lane >> 4;
    off = c * 128 + ((PAT == 1 ? (q ^ (c >> 1)) : q) * 16);
  }
  off += (wave & 7) * 4096 + (int)(uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)buf;  // LDS address of the lane's piece
  v4i acc = {0, 0, 0, 0};
  const long long c0 = clock64();
  for (int it = 0; it < iters; ++it) {
    // 8 independent reads in flight per wavefront, then one wait for all of them
    v4i x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(x[u]) : "v"(off), "n"(0) : "memory");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= x[u];
  }
  __syncthreads();
  const long long c1 = clock64();
  out[blockIdx.x * blockDim.x + threadIdx.x] = acc[0] + acc[1] + acc[2] + acc[3];
  if (threadIdx.x == 0) clk[blockIdx.x] = c1 - c0;
}

__global__ void __launch_bounds__(1024) lds_copy_rate(const char* __restrict__ src, long long* clk, int iters) {
  __shared__ __attribute__((aligned(1024))) char buf[64 * 1024];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)buf + (uint32_t)wave * 4096u;
  const char* g = src + (size_t)(blockIdx.x & 31) * 65536;  // 2 MiB in all: stays in the L2
  const uint32_t voff = (uint32_t)(wave * 4096 + lane * 16);
  __syncthreads();
  const long long c0 = clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
      asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff + (uint32_t)u * 1024u), "s"(g), "n"(0)
                   : "memory", "m0", "scc");
    __builtin_amdgcn_s_waitcnt(0x0074);  // at most 4 copies in flight per wavefront behind this point
  }
  __builtin_amdgcn_s_waitcnt(0x0070);
  __syncthreads();
  const long long c1 = clock64();
  if (threadIdx.x == 0) clk[blockIdx.x] = c1 - c0;
}

// Matrix against vector issue on one SIMD.  8 wavefronts per CU, two per SIMD: wavefronts 0..3 (one per SIMD) run
// sparse matrix instructions, wavefronts 4..7 a chain of 8 independent fp32 fma streams (MODE bit 0 / bit 1; both bits:
// side by side); MODE 4: wavefronts 0..3 alone run 8 x (one matrix instruction, two fma) interleaved in program order.
// clk[16 wg + wave] = clocks that wavefront spent in its loop.
template <int MODE>
__global__ void __launch_bounds__(512, 1) coissue_probe(const int* __restrict__ src, int* __restrict__ out, long long* __restrict__ clk, int iters) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const v4i a = *(const v4i*)(src + (threadIdx.x & 63) * 4);
  const v8i b = *(const v8i*)(src + 1024 + (threadIdx.x & 63) * 8);
  v4i acc[8];
  float f[8];
  for (int i = 0; i < 8; ++i) {
    acc[i] = v4i{0, 0, 0, 0};
    f[i] = (float)(src[(threadIdx.x + i) & 1023] & 0xffff) * 1e-6f;
  }
  __syncthreads();
  const long long c0 = clock64();
  if (MODE == 4) {
    if (wave < 4)
      for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          acc[i] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(a, b, acc[i], 0x44444444, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          f[i] = __builtin_fmaf(f[i], 0.999f, 0.001f);
          f[(i + 4) & 7] = __builtin_fmaf(f[(i + 4) & 7], 0.999f, 0.001f);
          __builtin_amdgcn_sched_barrier(0);
        }
  } else if (wave < 4) {
    if (MODE & 1)
      for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(a, b, acc[i], 0x44444444, 0, 0);
  } else if (MODE & 2) {
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = __builtin_fmaf(f[i], 0.999f, 0.001f);
  }
  const long long c1 = clock64();
  int s = 0;
  for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3] + (int)f[i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if ((threadIdx.x & 63) == 0) clk[blockIdx.x * 16 + wave] = c1 - c0;
}

template <int MODE>
static void run_coissue(const int* src, int* out, long long* clk, int wgs, int iters, double* matrix_clk, double* vector_clk) {
  coissue_probe<MODE><<<wgs, 512>>>(src, out, clk, 50);
  CK(hipDeviceSynchronize());
  coissue_probe<MODE><<<wgs, 512>>>(src, out, clk, iters);
  CK(hipDeviceSynchronize());
  std::vector<long long> h(16 * wgs);
  CK(hipMemcpy(h.data(), clk, sizeof(long long) * 16 * wgs, hipMemcpyDeviceToHost));
  double m = 0, v = 0;
  for (int i = 0; i < wgs; ++i) {
    m += (double)h[16 * i];
    v += (double)h[16 * i + 4];
  }
  *matrix_clk = m / wgs / iters;
  *vector_clk = v / wgs / iters;
}

__global__ void clock_sampler(long long* out, int n, int spin) {
  for (int i = 0; i < n; ++i) {
    out[2 * i] = clock64();
    out[2 * i + 1] = wall_clock64();
    for (int k = 0; k < spin; ++k) __builtin_amdgcn_s_sleep(64);
  }
}

static double mean_clk(const long long* clk, int wgs) {
  std::vector<long long> h(wgs);
  CK(hipMemcpy(h.data(), clk, sizeof(long long) * wgs, hipMemcpyDeviceToHost));
  double s = 0;
  for (auto v : h) s += v;
  return s / wgs;
}

int main(int argc, char** argv) {
  const char* json_path = nullptr;
  bool with_gemm = true;
  for (int i = 1; i < argc; ++i) {
    if (!strcmp(argv[i], "--json") && i + 1 < argc) json_path = argv[++i];
    if (!strcmp(argv[i], "--no-gemm")) with_gemm = false;
  }
  int cus = 0, clock_khz = 0, wall_khz = 0;
  CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  CK(hipDeviceGetAttribute(&clock_khz, hipDeviceAttributeClockRate, 0));
  CK(hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, 0));
  emit("compute_units", cus, "CUs", "hipDeviceAttributeMultiprocessorCount");
  emit("nominal_shader_clock", clock_khz / 1e3, "MHz", "hipDeviceAttributeClockRate");
  emit("wall_clock_rate", wall_khz / 1e3, "MHz", "hipDeviceAttributeWallClockRate");

  std::vector<int> hs(80 * 64);
  srand(1);
  for (auto& v : hs) v = rand() ^ (rand() << 16);
  int *src, *out;
  long long* clk;
  CK(hipMalloc(&src, hs.size() * 4));
  CK(hipMemcpy(src, hs.data(), hs.size() * 4, hipMemcpyHostToDevice));
  CK(hipMalloc(&out, (size_t)1024 * 1024 * 4));
  CK(hipMalloc(&clk, 16 * 1024));

  // ---- matrix instruction rates (dense-equivalent operations: 2 * 16 * 16 * K per instruction)
  run_matrix<0, false>("sparse_int8_16x16x128", 2.0 * 16 * 16 * 128, src, out, clk, cus, 512, "register-only loop, random operands, 8 wavefronts per CU, all CUs, event-timed");
  run_matrix<1, false>("dense_int8_16x16x64", 2.0 * 16 * 16 * 64, src, out, clk, cus, 512, "same loop, dense instruction");
  run_matrix<2, false>("sparse_fp16_16x16x64", 2.0 * 16 * 16 * 64, src, out, clk, cus, 512, "same loop, random bit patterns as fp16");
  run_matrix<3, false>("dense_fp16_16x16x32", 2.0 * 16 * 16 * 32, src, out, clk, cus, 512, "same loop, dense instruction");
  run_matrix<0, false>("sparse_int8_one_wave_per_simd", 2.0 * 16 * 16 * 128, src, out, clk, cus, 256, "4 wavefronts per CU: one per SIMD");
  run_matrix<0, true>("sparse_int8_barrier_every_32", 2.0 * 16 * 16 * 128, src, out, clk, cus, 512, "8 wavefronts per CU, a workgroup barrier every 32 instructions");
  run_matrix<0, false>("sparse_int8_quarter_of_the_chip", 2.0 * 16 * 16 * 128, src, out, clk, cus / 4, 512, "one workgroup on a quarter of the CUs: the clocks stay up");
  CK(hipMemset(src, 0, hs.size() * 4));
  run_matrix<0, false>("sparse_int8_zero_operands", 2.0 * 16 * 16 * 128, src, out, clk, cus, 512, "all-zero operands: fewer toggling bits, higher clock");
  CK(hipMemcpy(src, hs.data(), hs.size() * 4, hipMemcpyHostToDevice));

  // ---- vector ALU rates and the clock they run at
  run_vector<0>("vector_fp32_fma", 16 * 8, src, out, clk, cus, "8 wavefronts per CU, 16 independent chains of fp32 fma per lane");
  run_vector<1>("vector_gelu_epilogue_mix", 16 * 13, src, out, clk, cus, "per output 13 instructions as compiled: 8 fma-class, integer add, convert, multiply, max, v_exp_f32");

  // ---- streaming
  {
    const size_t bytes = (size_t)512 << 20, n = bytes / 16;
    v4i *a, *b;
    CK(hipMalloc(&a, bytes));
    CK(hipMalloc(&b, bytes));
    CK(hipMemset(a, 1, bytes));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    float ms;
    copy_kernel<<<cus * 16, 256>>>(a, b, n);
    CK(hipEventRecord(e0));
    for (int i = 0; i < 5; ++i) copy_kernel<<<cus * 16, 256>>>(a, b, n);
    CK(hipEventRecord(e1));
    CK(hipDeviceSynchronize());
    CK(hipEventElapsedTime(&ms, e0, e1));
    emit("stream_copy_bandwidth", 2.0 * bytes * 5 / (ms * 1e-3) / 1e9, "GB/s", "copy kernel, 512 MiB read + 512 MiB written per launch, 16 bytes per lane");
    fill_kernel<<<cus * 16, 256>>>(b, n);
    CK(hipEventRecord(e0));
    for (int i = 0; i < 5; ++i) fill_kernel<<<cus * 16, 256>>>(b, n);
    CK(hipEventRecord(e1));
    CK(hipDeviceSynchronize());
    CK(hipEventElapsedTime(&ms, e0, e1));
    emit("stream_fill_bandwidth", 1.0 * bytes * 5 / (ms * 1e-3) / 1e9, "GB/s", "fill kernel, 512 MiB written per launch");
    CK(hipFree(a));
    CK(hipFree(b));
  }

  // ---- LDS reads and global->LDS copies per CU
  {
    const int iters = 2000, wgs = cus;
    lds_rate<0><<<wgs, 1024>>>(out, clk, iters);
    CK(hipDeviceSynchronize());
    emit("lds_read_b128_contiguous", 1024.0 * 16 * 8 * iters / mean_clk(clk, wgs), "B/clk/CU", "16 wavefronts per CU, 8 reads in flight each, conflict-free");
    lds_rate<1><<<wgs, 1024>>>(out, clk, iters);
    CK(hipDeviceSynchronize());
    emit("lds_read_b128_swizzled_rows", 1024.0 * 16 * 8 * iters / mean_clk(clk, wgs), "B/clk/CU", "16 rows x 128-byte pitch with the GEMM's XOR swizzle");
    lds_rate<2><<<wgs, 1024>>>(out, clk, iters);
    CK(hipDeviceSynchronize());
    emit("lds_read_b128_unswizzled_rows", 1024.0 * 16 * 8 * iters / mean_clk(clk, wgs), "B/clk/CU", "the same rows without the swizzle (4-way bank conflicts)");
    char* l2buf;
    CK(hipMalloc(&l2buf, (size_t)32 * 65536 + 65536));
    CK(hipMemset(l2buf, 7, (size_t)32 * 65536 + 65536));
    lds_copy_rate<<<wgs, 1024>>>(l2buf, clk, 200);
    CK(hipDeviceSynchronize());
    lds_copy_rate<<<wgs, 1024>>>(l2buf, clk, iters);
    CK(hipDeviceSynchronize());
    emit("global_to_lds_copy_l2_resident", 16.0 * 4 * 1024 * iters / mean_clk(clk, wgs), "B/clk/CU", "global_load_lds_dwordx4, 16 wavefronts per CU, 4 copies in flight each, all CUs");
    CK(hipFree(l2buf));
  }

  // ---- matrix against vector issue on one SIMD (a quarter of the CUs, so that the clock stays up and the counts are per clock)
  {
    const int wgs = cus / 4, iters = 2000;
    double m, v, m2, v2;
    run_coissue<1>(src, out, clk, wgs, iters, &m, &v);
    emit("coissue_8_matrix_instructions_alone", m, "clk", "one wavefront per SIMD, 8 independent sparse INT8 matrix instructions per iteration");
    run_coissue<2>(src, out, clk, wgs, iters, &m, &v);
    emit("coissue_32_fma_alone", v, "clk", "one wavefront per SIMD, 32 fp32 fma per iteration (8 independent chains)");
    run_coissue<3>(src, out, clk, wgs, iters, &m2, &v2);
    emit("coissue_matrix_wavefront_beside_fma_wavefront", m2, "clk", "per iteration of the matrix wavefront while an fma wavefront shares its SIMD");
    emit("coissue_fma_wavefront_beside_matrix_wavefront", v2, "clk", "per iteration of the fma wavefront, averaged over its whole run (it runs alone once the matrix wavefront is done)");
    emit("coissue_fma_rate_while_matrix_pipe_busy", (v2 > m2 && v > 0) ? (1.0 - (v2 - m2) / v) * v / m2 : 0.0, "of alone",
         "share of its stand-alone rate the fma wavefront reaches while the matrix wavefront runs");
    run_coissue<4>(src, out, clk, wgs, iters, &m, &v);
    emit("coissue_one_wavefront_8_matrix_16_fma_interleaved", m, "clk", "8 x (matrix instruction, 2 fma) in one wavefront's program order");
  }

  // ---- the shader clock while the c1 sparse INT8 GEMM runs back to back (ViT-Base fc1 at batch 64)
  if (with_gemm) {
    const int64_t M = 12608, K = 768, N = 3072;
    float *W, *wscale, *ascale, *bias;
    _Float16 *Xh, *Y;
    int8_t* Xq;
    void *packed, *ws;
    CK(hipMalloc(&W, N * K * 4));
    CK(hipMalloc(&Xh, M * K * 2));
    CK(hipMalloc(&Xq, M * K));
    CK(hipMalloc(&wscale, N * 4));
    CK(hipMalloc(&ascale, 16));
    CK(hipMalloc(&bias, N * 4));
    CK(hipMalloc(&Y, M * N * 2));
    CK(hipMalloc(&ws, 4096));
    CK(hipMalloc(&packed, gpusq_packed_bytes(GPUSQ_I8, N, K)));
    {
      std::vector<float> w(N * K);
      for (auto& v : w) v = ((rand() % 2001) - 1000) * 2e-5f;
      CK(hipMemcpy(W, w.data(), w.size() * 4, hipMemcpyHostToDevice));
      std::vector<_Float16> x(M * K);
      for (auto& v : x) v = (_Float16)(((rand() % 2001) - 1000) * 3e-3f);
      CK(hipMemcpy(Xh, x.data(), x.size() * 2, hipMemcpyHostToDevice));
      std::vector<float> b(N, 0.01f);
      CK(hipMemcpy(bias, b.data(), N * 4, hipMemcpyHostToDevice));
    }
    if (gpusq_prepare_weights(W, GPUSQ_I8, nullptr, nullptr, wscale, nullptr, nullptr, packed, N, K, nullptr) != GPUSQ_OK ||
        gpusq_quantize_int8(Xh, GPUSQ_F16, Xq, ascale, GPUSQ_PER_TENSOR, 0, M, K, ws, nullptr) != GPUSQ_OK) {
      fprintf(stderr, "weight or activation preparation failed\n");
      return 1;
    }
    CK(hipDeviceSynchronize());
    hipStream_t s1, s2;
    CK(hipStreamCreate(&s1));
    CK(hipStreamCreate(&s2));
    const int NS = 400, reps = 100;
    long long* samp;
    CK(hipMalloc(&samp, NS * 16));
    for (int i = 0; i < 5; ++i) gpusq_spgemm_int8(Xq, packed, ascale, wscale, bias, Y, GPUSQ_F16, nullptr, M, N, K, 3, s1);
    CK(hipDeviceSynchronize());
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    clock_sampler<<<1, 64, 0, s2>>>(samp, NS, 8);
    CK(hipEventRecord(e0, s1));
    for (int i = 0; i < reps; ++i) gpusq_spgemm_int8(Xq, packed, ascale, wscale, bias, Y, GPUSQ_F16, nullptr, M, N, K, 3, s1);
    CK(hipEventRecord(e1, s1));
    CK(hipDeviceSynchronize());
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    std::vector<long long> h(2 * NS);
    CK(hipMemcpy(h.data(), samp, NS * 16, hipMemcpyDeviceToHost));
    // samples taken while the GEMMs ran: those inside the first `ms` milliseconds of the sampler's wall clock
    std::vector<double> mhz;
    for (int i = 10; i < NS; i += 10) {
      if ((h[2 * i + 1] - h[1]) / 100.0 > ms * 1e3) break;
      mhz.push_back(100.0 * (h[2 * i] - h[2 * (i - 10)]) / (double)(h[2 * i + 1] - h[2 * (i - 10) + 1]));
    }
    std::sort(mhz.begin(), mhz.end());
    emit("c1_gemm_us", ms * 1e3 / reps, "us", "sparse INT8 GEMM of ViT-Base fc1 at batch 64 (bias + GELU, fp16 out), 100 launches back to back");
    if (!mhz.empty()) {
      emit("c1_gemm_shader_clock_median", mhz[mhz.size() / 2], "MHz", "one-wavefront sampler kernel on a second stream while the GEMMs run");
      emit("c1_gemm_shader_clock_min", mhz.front(), "MHz", "lowest 10-sample window");
    }
    clock_sampler<<<1, 64, 0, s2>>>(samp, NS, 8);
    CK(hipDeviceSynchronize());
    CK(hipMemcpy(h.data(), samp, NS * 16, hipMemcpyDeviceToHost));
    emit("idle_shader_clock", 100.0 * (h[2 * NS - 2] - h[2 * (NS / 2)]) / (double)(h[2 * NS - 1] - h[2 * (NS / 2) + 1]), "MHz", "the sampler alone");
  }
  if (json_path) {
    FILE* f = fopen(json_path, "w");
    if (f) {
      fprintf(f, "{%s\n}\n", g_json.c_str());
      fclose(f);
    }
  }
  return 0;
}
