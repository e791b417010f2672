/*
 * gpusq.h -- C ABI of libgpusq: 2:4 fine-grained structured-sparse linear layers (FP16 and INT8) for AMD MI355X.
 *
 * The library implements the deployment hot path of "Boost Vision Transformer with GPU-Friendly Sparsity and
 * Quantization" (CVPR 2023): the sparse x dense -> dense GEMM of Sec. 3.1 / Fig. 1 behind the Q/K/V projection,
 * attention output projection and feed-forward linears named in Sec. 3.2, with the weight-preparation steps
 * (2:4 pruning, symmetric INT8 quantisation, compression to kept values + 2-bit metadata).
 *
 * Notation.  The paper's sparse operand "A" (M x K, 2:4 along K) is the weight matrix W [N][K] here (nn.Linear
 * layout, K contiguous); the dense operand is the activation matrix X [M][K] (tokens x features, K contiguous);
 * the result is Y [M][N] = X * W^T (+ bias, + GELU), row-major.
 *
 * Conventions for every call.
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library never allocates, frees or keeps
 *     device memory.  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Calls enqueue work on `stream` and return; they do not synchronise.
 *   - The return value is a gpusq_status.  Argument errors are detected on the host before anything is launched
 *     and leave the outputs untouched.  A failed launch returns GPUSQ_ERR_HIP; gpusq_last_hip_error() gives the
 *     HIP error code.  No exception crosses this boundary.
 *   - Tensors are dense row-major without padding; all pointers must be 16-byte aligned (GPUSQ_ERR_ALIGN).
 *   - K must be a multiple of 4 (a row is made of whole groups of 4; GPUSQ_ERR_SHAPE otherwise).  The GEMM entry
 *     points additionally need K % 16 == 0 and N % 4 == 0 (GPUSQ_ERR_UNSUPPORTED otherwise); M is arbitrary.
 *     Sizes must be positive, each dimension below 2^31 and each tensor below 2^40 elements (GPUSQ_ERR_SHAPE).
 *   - Thread safety: calls on distinct streams may run concurrently; the library holds no mutable global state
 *     besides the last HIP error code, each device's CU count (read once), the testing override of
 *     gpusq_force_kernel and, per host thread, the kernel choices and tile plans of the last few distinct GEMM
 *     problems.
 */
#ifndef GPUSQ_H
#define GPUSQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GPUSQ_OK = 0,
  GPUSQ_ERR_NULL = 1,        /* a required pointer is NULL */
  GPUSQ_ERR_SHAPE = 2,       /* non-positive size, K % 4 != 0, or a size beyond the supported range */
  GPUSQ_ERR_ALIGN = 3,       /* a pointer is not 16-byte aligned */
  GPUSQ_ERR_UNSUPPORTED = 4, /* valid for the method but not implemented (dtype, divisibility, epilogue bits) */
  GPUSQ_ERR_HIP = 5,         /* a HIP call or kernel launch failed */
  GPUSQ_ERR_NOT_2TO4 = 6     /* gpusq_check_2to4 only: a group of 4 has more than two non-zero elements */
} gpusq_status;

typedef enum { GPUSQ_F32 = 0, GPUSQ_F16 = 1, GPUSQ_I8 = 2, GPUSQ_I32 = 3 } gpusq_dtype;

/* epilogue bit flags */
enum { GPUSQ_EPI_NONE = 0, GPUSQ_EPI_BIAS = 1, GPUSQ_EPI_GELU = 2 };

/* quantisation granularity */
enum { GPUSQ_PER_ROW = 0, GPUSQ_PER_TENSOR = 1 };

const char* gpusq_status_string(gpusq_status s);
int gpusq_last_hip_error(void);
int gpusq_version(void);

/* ---- 2:4 pruning [Sec. 1; Sec. 3.1: two of every four contiguous elements on a row of the sparse operand are
 * zero].  The paper does not print the selection rule; this library keeps the two largest magnitudes of each group
 * of 4 along K (ties: the lower index is kept) and writes +0 to the other two.
 *   W_in, W_out : [N][K] of dt (GPUSQ_F32 or GPUSQ_F16); W_out may be the same pointer as W_in.
 *   mask_out    : optional [N][K/4] bytes; bit i of a byte is set iff element 4g+i of the group was kept. */
gpusq_status gpusq_prune_2to4(const void* W_in, void* W_out, uint8_t* mask_out, gpusq_dtype dt,
                              int64_t N, int64_t K, void* stream);

/* ---- FP32 -> FP16 rounding (round-to-nearest-even) of n contiguous elements: the step from the pruned FP32
 * weights to the "2:4 FP16 sparse" model that the paper's pipeline produces first [Sec. 3.1, last sentence of the
 * storage-format paragraph].  Also usable for activations. */
gpusq_status gpusq_cast_f16(const float* in, void* out, int64_t n, void* stream);

/* ---- symmetric INT8 quantisation with a scale factor [Sec. 2.2; Sec. 3.4].  q = clamp(rint(x / s), -127, 127),
 * fp32 division, round-half-even; s = max|x| / 127 over a row (GPUSQ_PER_ROW: per output channel, scale has `rows`
 * floats) or over the whole tensor (GPUSQ_PER_TENSOR: scale has 1 float); an all-zero range gives s = 1.
 *   X [rows][cols] of dt (GPUSQ_F32 or GPUSQ_F16), Xq [rows][cols] int8, scale: device floats.
 *   scale_is_input != 0: use the caller's scale(s) (calibrated / learned values) instead of computing them.
 *   workspace: device scratch of gpusq_quantize_workspace_bytes(mode, rows, cols) bytes (may be NULL when that is 0);
 *   its previous contents do not matter. */
size_t gpusq_quantize_workspace_bytes(int mode, int64_t rows, int64_t cols);
gpusq_status gpusq_quantize_int8(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int mode,
                                 int scale_is_input, int64_t rows, int64_t cols, void* workspace, void* stream);

/* ---- the per-tensor form of gpusq_quantize_int8 for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (mode is
 * GPUSQ_PER_TENSOR, there is no workspace), same kernels, bit-identical Xq and scale; the partial maxima of the range
 * pass live in a 4 KB device array inside the library (one per GPU, held until the process ends), which serves every
 * size gpusq_quantize_int8 accepts: rows * cols up to 2^40, GPUSQ_ERR_SHAPE beyond.  The call allocates and frees
 * nothing.  Its first use on a device looks up the array's address there (hipGetSymbolAddress), so make that first call
 * outside a graph capture.  All calls on one GPU share the array: calls that overlap in time on the same GPU (different
 * streams, or graph branches that run side by side) race on it and must be ordered by the caller. */
gpusq_status gpusq_quantize_tensor_int8_noalloc(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale,
                                                int scale_is_input, int64_t rows, int64_t cols, void* stream);

/* ---- compression [Sec. 3.1, Fig. 1 and Fig. 2 captions]: the N x K operand becomes N x K/2 kept values plus
 * 2 bits of metadata per kept value giving its position in its group of 4.
 *   W      : [N][K] of dt (GPUSQ_F16 or GPUSQ_I8)
 *   values : [N][K/2] of dt; the two kept values of group g at 2g, 2g+1, in ascending position order
 *   meta   : [N][ceil(K/8)] bytes; byte b of a row holds group 2b in bits 0..3 and group 2b+1 in bits 4..7; inside
 *            a nibble, bits 0..1 = position of the first kept value, bits 2..3 = position of the second (first <
 *            second).  Positions are chosen by the pruning rule applied to W itself, so the non-zeros of a 2:4
 *            tensor are always kept and spare slots go to the lowest-index zeros.
 *   violations : optional device int32, set to the number of groups in which a dropped element was non-zero
 *            (0 iff W obeys the 2:4 pattern). */
gpusq_status gpusq_compress(const void* W, void* values, uint8_t* meta, int32_t* violations, gpusq_dtype dt,
                            int64_t N, int64_t K, void* stream);
/* ---- validation [Sec. 3.1: in a 2:4 tensor every group of four contiguous elements along K holds at most two
 * non-zero values].  Counts the groups of W [N][K] (GPUSQ_F32, GPUSQ_F16 or GPUSQ_I8) with more than two non-zero
 * elements (-0 is zero) into *violations (device int32, required, 4-byte aligned; N*K/4 must fit an int32) and, the one
 * call of this library that waits for the device, synchronises `stream` and returns GPUSQ_OK for a count of 0,
 * GPUSQ_ERR_NOT_2TO4 otherwise (not usable under stream capture: GPUSQ_ERR_HIP there).  The other calls stay
 * asynchronous and never return this status: gpusq_compress reports the same count through its optional counter. */
gpusq_status gpusq_check_2to4(const void* W, gpusq_dtype dt, int32_t* violations, int64_t N, int64_t K, void* stream);

/* inverse: zero-fill W [N][K] and scatter the values to the recorded positions */
gpusq_status gpusq_decompress(const void* values, const uint8_t* meta, void* W, gpusq_dtype dt,
                              int64_t N, int64_t K, void* stream);

/* ---- other n:m patterns [Sec. 5, limitation paragraph: a hardware generation might support 1:4 or 2:16 instead]: the
 * n largest magnitudes of every m contiguous elements of a row are kept (ties: the lower index), the rest become +0.
 * W_in, W_out [N][K] fp32 (may alias); m = 4, 8 or 16 (GPUSQ_ERR_UNSUPPORTED otherwise), 1 <= n < m, K % m == 0
 * (GPUSQ_ERR_SHAPE otherwise).  n = 2, m = 4 gives what gpusq_prune_2to4 gives; 1:4 and 2:16 tensors are 2:4 tensors as
 * well and go through gpusq_compress / gpusq_spgemm_* unchanged (with half or more of the kept slots holding zeros). */
gpusq_status gpusq_prune_n_of_m(const float* W_in, float* W_out, int n, int m, int64_t N, int64_t K, void* stream);

/* ---- INT4 operands: the pair-wise 4:8 pattern [Sec. 3.1, the paragraph on the INT4 instruction: every chunk of 8
 * adjacent elements of a row holds four zeros and four non-zeros, clustered in 2-wide sub-chunks that are all zero or
 * all non-zero; the compressed row stores the four non-zero values and two 2-bit indices with the positions of the two
 * kept sub-chunks].  The paper prints no selection rule; this library keeps the two sub-chunks with the largest
 * |a| + |b| (one fp32 addition; ties: the lower index).  gfx950 has no 4-bit integer matrix instruction and the pattern
 * is not a 2:4 pattern, so the product runs on the decoded INT8 operand (gpusq_gemm_int8_dense with the 4-bit scales);
 * the format's gain here is storage: 2.5 bits per weight.  K % 8 == 0 for all four calls (GPUSQ_ERR_SHAPE otherwise).
 *   gpusq_prune_4to8_pairs : W_in, W_out [N][K] fp32 (may alias); mask_out optional [N][K/8] bytes, bit p = sub-chunk p kept.
 *       one_per_group != 0: of the two kept sub-chunks one lies in each group of 4 (the one with the larger |a| + |b|;
 *       4 of the 6 choices): the tensor then obeys the pair-wise 4:8 pattern and the 2:4 pattern at once, and its INT4
 *       storage can be turned into the INT8 2:4 operand of gpusq_spgemm_int8 (gpusq_int4_to_sparse_int8 + gpusq_pack):
 *       4-bit storage at the speed of the 2:4 INT8 path.
 *   gpusq_quantize_rows_int4 : q = clamp(rint(x / s), -7, 7) in int8 containers, s = max|row| / 7 (1 for an all-zero
 *       row) written to scale[rows], or the caller's scales when scale_is_input != 0; X of dt GPUSQ_F32 or GPUSQ_F16.
 *   gpusq_compress_int4 : W [N][K] int8 holding 4-bit codes -> values [N][K/4] bytes (the 4 kept codes of chunk c in
 *       ascending position as two's-complement nibbles: code j in byte 2c + j/2, low nibble for even j) and meta
 *       [N][ceil(K/16)] bytes (chunk c in the low nibble of byte c/2 for even c, the high nibble for odd c; bits 0..1 =
 *       first kept sub-chunk, bits 2..3 = second, first < second).  Positions follow the selection rule applied to W
 *       itself.  violations (optional device int32): chunks with a dropped non-zero or a code outside -8..7.
 *   gpusq_decompress_int4 : the inverse, W [N][K] int8 zero-filled with the codes sign-extended.
 *   gpusq_int4_to_sparse_int8 : (values, meta) of gpusq_compress_int4 -> the 2:4 compressed INT8 form of gpusq_compress
 *       (values8 [N][K/2] int8, meta8 [N][K/8] bytes), chunk by chunk without the dense matrix; a group of 4 keeps its
 *       non-zero sub-chunk (its first one if it has none).  mismatches (optional device int32): groups of 4 with two
 *       non-zero sub-chunks (not a 2:4 row; they keep the second sub-chunk only), 0 for tensors pruned with one_per_group. */
gpusq_status gpusq_prune_4to8_pairs(const float* W_in, float* W_out, uint8_t* mask_out, int one_per_group, int64_t N, int64_t K,
                                    void* stream);
gpusq_status gpusq_int4_to_sparse_int8(const uint8_t* values4, const uint8_t* meta4, int8_t* values8, uint8_t* meta8,
                                       int32_t* mismatches, int64_t N, int64_t K, void* stream);
gpusq_status gpusq_quantize_rows_int4(const void* X, gpusq_dtype dt, int8_t* Xq, float* scale, int scale_is_input,
                                      int64_t rows, int64_t cols, void* stream);
gpusq_status gpusq_compress_int4(const int8_t* W, uint8_t* values, uint8_t* meta, int32_t* violations, int64_t N,
                                 int64_t K, void* stream);
gpusq_status gpusq_decompress_int4(const uint8_t* values, const uint8_t* meta, int8_t* W, int64_t N, int64_t K,
                                   void* stream);

/* ---- kernel-native packing of the compressed operand: re-tiles (values, meta) into the per-lane register order
 * of the gfx950 sparse matrix instructions (v_smfmac_*), rows and K zero-padded to whole tiles.  The packed buffer
 * is opaque; its size is gpusq_packed_bytes(dt, N, K) bytes (0 for invalid arguments). */
size_t gpusq_packed_bytes(gpusq_dtype dt, int64_t N, int64_t K);
gpusq_status gpusq_pack(const void* values, const uint8_t* meta, void* packed, gpusq_dtype dt,
                        int64_t N, int64_t K, void* stream);

/* ---- the whole weight-side preparation in one launch: prune 2:4 -> (dt = GPUSQ_I8: per-output-channel INT8
 * quantisation | dt = GPUSQ_F16: rounding to FP16) -> compress -> pack, the order the paper gives ("first compress as
 * 2:4 FP16 sparse, then further quantize", Sec. 3.1).  Results are bit-identical to calling gpusq_prune_2to4,
 * gpusq_quantize_int8(GPUSQ_PER_ROW) / gpusq_cast_f16, gpusq_compress and gpusq_pack in turn.
 *   W [N][K] fp32 (input);  packed: gpusq_packed_bytes(dt, N, K) bytes (required);  w_scale [N] (required for I8).
 *   Optional outputs (NULL to skip): W_pruned [N][K] fp32, W_low [N][K] of dt (the masked low-precision weights, the
 *   dense twins' operand), values [N][K/2] of dt, meta [N][ceil(K/8)].
 *   K is limited to 16384 (GPUSQ_ERR_UNSUPPORTED beyond): one fp32 row is staged in LDS. */
gpusq_status gpusq_prepare_weights(const float* W, gpusq_dtype dt, float* W_pruned, void* W_low, float* w_scale,
                                   void* values, uint8_t* meta, void* packed, int64_t N, int64_t K, void* stream);

/* ---- sparse GEMM with fused epilogue [Sec. 3.1: sparse matrix x dense matrix = dense matrix, the same result as
 * the dense GEMM on the zero-filled operand, computed over the kept values only].
 * FP16: Y[m][n] = fp16( act( sum_k X[m][k] * W[n][k]  (fp32 accumulation) + bias[n] ) )
 *   X [M][K] fp16, Wpacked from gpusq_pack(GPUSQ_F16), bias [N] fp32 (required iff GPUSQ_EPI_BIAS), Y [M][N] fp16;
 *   act = GELU in its exact (erf) form x * Phi(x) iff GPUSQ_EPI_GELU [Sec. 2.2 / 3.4: the activation of the MLP block],
 *   evaluated in fp32 as max(x, 0) - |x| * 2^P(|x|) with a degree-5 polynomial P fitted to log2 Phi(-t): within 0.15
 *   units in the last place of the exact value as an fp16 number over the whole fp16 range (negative tail included),
 *   so the fp16 output is within one fp16 ulp of the exactly rounded value.  The same evaluation serves every call
 *   below that takes GPUSQ_EPI_GELU. */
gpusq_status gpusq_spgemm_fp16(const void* X, const void* Wpacked, const float* bias, void* Y,
                               int64_t M, int64_t N, int64_t K, int epilogue, void* stream);
/* INT8: acc[m][n] = sum_k Xq[m][k] * Wq[n][k] in int32 (exact);
 *   out_dt = GPUSQ_I32: Y [M][N] int32 = acc (scales, bias, epilogue ignored);
 *   out_dt = GPUSQ_F16: Y = fp16( act( fma((float)acc, act_scale[0] * w_scale[n], bias[n]) ) );
 *   out_dt = GPUSQ_I8 : Y = clamp(rint( act(...) / out_scale[0] ), -127, 127) as int8 (re-quantised for the next layer).
 *   act_scale, out_scale: device pointers to 1 float; w_scale: device [N] floats. */
gpusq_status gpusq_spgemm_int8(const int8_t* Xq, const void* Wpacked, const float* act_scale, const float* w_scale,
                               const float* bias, void* Y, gpusq_dtype out_dt, const float* out_scale,
                               int64_t M, int64_t N, int64_t K, int epilogue, void* stream);

/* The same product with the quantise node of the activations [Sec. 2.2: activations are quantised at run time with a
 * calibrated scale before every quantised layer] folded into the GEMM: X [M][K] fp16 is turned into the codes
 * Xq = clamp(rint(X / act_scale[0]), -127, 127) on its way to the matrix instructions (the code rule of
 * gpusq_quantize_int8 with scale_is_input != 0; bit-identical to calling that first), so a layer with a static scale is
 * one launch instead of two.  Only the latency kernel, through whose registers X passes, can do this: a problem that
 * gpusq_spgemm_plan assigns to a tile kernel (kernel >= 2) returns GPUSQ_ERR_UNSUPPORTED and is served by
 * gpusq_quantize_int8 + gpusq_spgemm_int8.  Every workgroup quantises the rows of its own tile, so the saving is that
 * of a launch (a few microseconds) against extra work per K step: it pays for short K (up to about 384).
 * All other arguments as for gpusq_spgemm_int8. */
gpusq_status gpusq_spgemm_int8_xf16(const void* X, const void* Wpacked, const float* act_scale, const float* w_scale,
                                    const float* bias, void* Y, gpusq_dtype out_dt, const float* out_scale,
                                    int64_t M, int64_t N, int64_t K, int epilogue, void* stream);

/* ---- patch embedding [Sec. 3.3: the patch-embedding layer is a convolution with C input channels, D_embed output
 * channels and kernel size = stride = P on images N x C x H x W, each P x P patch becoming one token; 2:4 sparsity is
 * applied to it like to the linear layers].  With kernel = stride the convolution is the product of the flattened patches
 * with the flattened weights, so it runs on the same sparse GEMM: this call writes the flattened patches,
 *   X[(b*(H/P) + py)*(W/P) + px][(c*P + i)*P + j] = img[b][c][py*P + i][px*P + j],   X[.][k] = 0 for C*P*P <= k < K_pad,
 * and gpusq_spgemm_* with K = K_pad on weights [D_embed][C][P][P] flattened to [D_embed][C*P*P] (zero-padded to K_pad,
 * pruned / quantised / compressed / packed like any other weight) gives Y [B*(H/P)*(W/P)][D_embed].
 *   img [B][C][H][W] and X [B*(H/P)*(W/P)][K_pad] of dt (GPUSQ_I8: an image quantised with gpusq_quantize_int8, or
 *   GPUSQ_F16); H % P == 0, W % P == 0, K_pad >= C*P*P (else GPUSQ_ERR_SHAPE); the GEMM needs K_pad % 16 == 0. */
gpusq_status gpusq_im2col_patches(const void* img, void* X, gpusq_dtype dt, int64_t B, int64_t C, int64_t H, int64_t W,
                                  int64_t P, int64_t K_pad, void* stream);

/* The same layer without the flattened-patch buffer, for P = 16: the sparse GEMM fetches its activation tiles from the
 * images directly (for P = 16 a 16-byte piece of a flattened patch is 16 consecutive pixels of one image row).
 *   img [B][C][H][W] int8 (quantised with gpusq_quantize_int8, scale act_scale[0]) or fp16; Wpacked from
 *   gpusq_pack(dt, D, C*256) on the weights [D][C][16][16] flattened; Y [B*(H/16)*(W/16)][D] fp16
 *   = fp16( fma((float)acc, act_scale[0] * w_scale[d], bias[d]) ) (int8) / fp16(acc + bias[d]) (fp16); epilogue: GPUSQ_EPI_NONE
 *   or GPUSQ_EPI_BIAS.  H % 16 == 0, W % 16 == 0, D % 4 == 0; the image batch must be smaller than 4 GiB.
 *   GPUSQ_ERR_UNSUPPORTED for problems with B*(H/16)*(W/16)*D <= 262144 (use gpusq_im2col_patches + gpusq_spgemm_*). */
gpusq_status gpusq_patch_embed16_int8(const int8_t* img, const void* Wpacked, const float* act_scale, const float* w_scale,
                                      const float* bias, void* Y, int64_t B, int64_t C, int64_t H, int64_t W, int64_t D,
                                      int epilogue, void* stream);
gpusq_status gpusq_patch_embed16_fp16(const void* img, const void* Wpacked, const float* bias, void* Y, int64_t B, int64_t C,
                                      int64_t H, int64_t W, int64_t D, int epilogue, void* stream);

/* ---- host-side introspection (no GPU work, no device access when cus > 0): how gpusq_spgemm_fp16 / gpusq_spgemm_int8
 * (dt = GPUSQ_F16 / GPUSQ_I8 = the operand type) decompose a problem on a device with `cus` compute units (cus <= 0: the
 * current device).  out[0] = kernel (0: small kernel, 64 x 64 tiles; 1: small kernel, 128 x 128 tiles, any K % 16 == 0;
 * 2: tile kernel with one workgroup per CU, tiles of 256 channels x up to 256 rows; 3: tile kernel with two workgroups per
 * CU, tiles of 256 channels x up to 128 rows, the template the dense twins are built from); for the tile kernels out[1] =
 * rows per tile unit u, out[2] = 256-channel blocks, out[3] = full_tm (a full tile has u * full_tm rows), out[4] = row
 * chunks covered by full tiles, out[5] = tail_tm (the remaining rows are cut into tiles of u * tail_tm rows), out[6] =
 * tiles in all, out[7] = workgroups launched.  Same argument checks as the GEMM calls (sizes only).
 * The query describes gpusq_spgemm_fp16 / gpusq_spgemm_int8 only: the fused patch-embedding calls
 * (gpusq_patch_embed16_*) always run on tile kernel 2, whatever this query reports for a GEMM of the same sizes. */
gpusq_status gpusq_spgemm_plan(gpusq_dtype dt, int64_t M, int64_t N, int64_t K, int epilogue, int cus, int32_t out[8]);

/* Testing aid: kernel = 0, 1, 2 or 3 makes the sparse GEMM entry points (and gpusq_spgemm_plan's out[0]) take that kernel
 * for every problem it can run (the tile kernels need K * element size % 128 == 0), so that every kernel can be checked on
 * the same shapes; 0 and 1 also keep the dense twins on their small kernel; any other value gives the choice back to the
 * size rules.  Returns the previous setting (-1 = none).  Process-wide; the environment variable GPUSQ_FORCE_KERNEL (0..3)
 * gives the initial setting and is read once, when the library is loaded.  Not meant for production callers. */
int gpusq_force_kernel(int kernel);

/* ---- dense twins [Sec. 1; Sec. 3.1, Fig. 1: the dense GEMM takes T cycles where the sparse one takes T/2]: the same
 * computation from the masked but uncompressed W [N][K] on the dense matrix instructions: the baseline the sparse kernels
 * are compared with.  Problems with M * N > 262144 and K * element size % 64 == 0 run on the dense instantiation of tile
 * kernel 3 (same template, tile plan, launch path and epilogue as the sparse instantiation; a dense K step is 64 bytes and
 * holds as many matrix instructions as a sparse step of 128 bytes); smaller or ragged-K problems on a small dense kernel. */
gpusq_status gpusq_gemm_fp16_dense(const void* X, const void* W, const float* bias, void* Y,
                                   int64_t M, int64_t N, int64_t K, int epilogue, void* stream);
gpusq_status gpusq_gemm_int8_dense(const int8_t* Xq, const int8_t* Wq, const float* act_scale, const float* w_scale,
                                   const float* bias, void* Y, gpusq_dtype out_dt, const float* out_scale,
                                   int64_t M, int64_t N, int64_t K, int epilogue, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GPUSQ_H */
