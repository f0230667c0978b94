// Shared declarations of the wmdec HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/wmdec.h"

namespace wmdec {

// ---------------------------------------------------------------- 16-bit types
// Storage types are raw bit patterns; conversions are explicit so that every
// rounding point is visible in the kernels.
struct bf16_t { uint16_t bits; };
struct f16_t  { uint16_t bits; };

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return __uint_as_float(((uint32_t)v.bits) << 16); }
__device__ __forceinline__ float to_float(f16_t v) {
  _Float16 h; __builtin_memcpy(&h, &v.bits, 2); return (float)h;
}

template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float v) {
  __bf16 h = (__bf16)v;  // v_cvt_pk_bf16_f32: round to nearest even; NaN stays NaN
  bf16_t r; __builtin_memcpy(&r.bits, &h, 2); return r;
}
template <> __device__ __forceinline__ f16_t from_float<f16_t>(float v) {
  _Float16 h = (_Float16)v;  // v_cvt_f16_f32: round to nearest even
  f16_t r; __builtin_memcpy(&r.bits, &h, 2); return r;
}

// round a float through the 16-bit type T (identity for float)
template <typename T> __device__ __forceinline__ float round_through(float v) { return to_float(from_float<T>(v)); }

__device__ __forceinline__ float silu_f(float t) {
  // t * sigmoid(t); exp2 of -t*log2(e) keeps it to one transcendental plus one reciprocal
  return t * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * t));
}

// ---------------------------------------------------------------- host side
void set_error(const char* fmt, ...);
int hip_fail(hipError_t e, const char* what);

#define WMDEC_REQUIRE(cond, code, ...)        \
  do {                                        \
    if (!(cond)) {                            \
      ::wmdec::set_error(__VA_ARGS__);        \
      return (code);                          \
    }                                         \
  } while (0)

#define WMDEC_HIP(expr)                                           \
  do {                                                            \
    hipError_t e__ = (expr);                                      \
    if (e__ != hipSuccess) return ::wmdec::hip_fail(e__, #expr);  \
  } while (0)

inline bool is_16bit(int dt) { return dt == WMDEC_BF16 || dt == WMDEC_F16; }
inline bool valid_dtype(int dt) { return dt == WMDEC_F32 || is_16bit(dt); }
inline size_t dtype_size(int dt) { return dt == WMDEC_F32 ? 4 : 2; }

// Arguments of every convolution launch (3x3 / 1x1, optional fused pieces).
struct ConvArgs {
  const void* x = nullptr;       // input activations
  int x_dtype = WMDEC_F32;       // storage type of x
  int x_nchw = 0;                // 1: x is [n,cin,h_in,w_in] (decoder latent), else NHWC
  const void* x_step = nullptr;  // non-null (few-input-channel kernel only): one tensor shaped like a sample of x, of
  float step_scale = 0.f;        //   x_dtype; sample i of the input is x[0] + (i + 1) * step_scale * x_step
  const float* mean = nullptr;   // [n*groups] or null: no normalisation
  const float* rstd = nullptr;
  const float* gamma = nullptr;  // [cin]
  const float* beta = nullptr;
  int groups = 1;
  int groups_norm = 0;           // label queries only: the launch will normalise although mean is not known yet
  int silu = 0;
  const void* wt = nullptr;      // packed [k*k][cout][cin] in op dtype
  const void* wt_phase = nullptr;  // upsample only: the 16-tap phase pack (pre-summed 2x2 weights of the four output phases)
  int op_dtype = WMDEC_F32;      // arithmetic: F32 (FMA) or BF16 / F16 (operands rounded to it)
  const float* bias = nullptr;   // [cout] or null
  const void* res = nullptr;     // [n,h,w,cout] of res_dtype or null
  int res_dtype = WMDEC_F32;
  void* y = nullptr;
  int y_dtype = WMDEC_F32;
  int y_nchw = 0;                // 1: y is [n,cout,h,w] (decoder frame)
  int n = 0, h = 0, w = 0;       // OUTPUT height / width
  int cin = 0, cout = 0;
  int ksize = 3;                 // 1 or 3
  int upsample = 0;              // 1: input is [n,h/2,w/2,cin], gathered at (y>>1, x>>1)
  const void* x2 = nullptr;      // matrix-core 3x3 kernel only: y += W2 * x2 + bias2, the 1x1 shortcut of a channel-changing
  const void* w2 = nullptr;      //   ResBlock folded into the contraction; x2 [n,h,w,cin2] of op_dtype, w2 packed with k = 1
  const float* bias2 = nullptr;
  int cin2 = 0;
  void* stats_ws = nullptr;      // non-null: also emit GroupNorm moments of y, [n][stats_groups][slots] triples
  int stats_groups = 0;
  // matrix-core kernel only: statistics handed from producer to consumer without a merge launch
  void* rows_out = nullptr;      // non-null (with stats_ws, tickets): one triple per (sample, group, tile row) of y
  void* tickets = nullptr;       // zeroed counters, one per (sample, tile row, channel tile); left at zero
  const void* rows_in = nullptr; // non-null instead of mean / rstd: row triples of x, [n][groups][rows_in_count]
  int rows_in_count = 0;
  float eps = 0.f;               // with rows_in: rstd = 1/sqrt(var + eps)
};

// kernels_conv_direct.hip: general VALU convolution (any shape, all dtypes).
int launch_conv_direct(const ConvArgs& a, hipStream_t s);
// same file: 3x3 convolution with at most 8 input channels, no normalisation / residual, NHWC output (conv_in)
bool conv_small_cin_supported(const ConvArgs& a);
int conv_small_cin_stats_slots(const ConvArgs& a);   // triples per (sample, group) it would emit with stats_ws set; 0: none
int launch_conv_small_cin(const ConvArgs& a, hipStream_t s);
// kernels_conv_mfma.hip: implicit-GEMM MFMA convolution; returns 1 if the shape
// is not one it handles (caller falls back to the direct kernel), 0 if launched.
bool conv_mfma_supported(const ConvArgs& a);
int launch_conv_mfma(const ConvArgs& a, hipStream_t s);
// true if the launch evaluates an upsampling convolution per output phase (2x2 taps, 4/9 of the products)
bool conv_mfma_uses_phase(const ConvArgs& a);
// moment slots per (sample, group) the MFMA kernel would write for this launch; 0: it cannot emit statistics
int conv_mfma_stats_slots(const ConvArgs& a);
void conv_mfma_row_extents(const ConvArgs& a, int* tile_rows, int* channel_tiles, int* tiles_per_row);
const char* conv_mfma_label(const ConvArgs& a);   // instantiation name, valid until the thread's next call
// kernels_conv_taps.hip: 3x3 convolution with at most three output channels into a planar fp32 tensor (the frame),
// evaluated as a 1x1 contraction onto (tap, channel) pairs followed by nine shifted adds
bool conv_taps_supported(const ConvArgs& a);
int launch_conv_taps(const ConvArgs& a, hipStream_t s);
const char* conv_taps_label(const ConvArgs& a);
// picks the kernel
int launch_conv(const ConvArgs& a, hipStream_t s);
const char* conv_kernel_label(const ConvArgs& a);

// kernels_gn.hip
// ticket: one zero-initialised counter per sample (gn_stats_ticket_bytes(n) bytes), left zero by every launch;
// moments: scratch of at least gn_stats_moments_bytes(n, groups) bytes
size_t gn_stats_ticket_bytes(int n);
size_t gn_stats_moments_bytes(int n, int groups);
int gn_stats_num_launches(int x_dtype, int h, int w, int c, int groups);   // 1: single-launch kernel, 2: partial + merge
int launch_gn_stats(const void* x, int x_dtype, int n, int h, int w, int c, int groups, float eps,
                    float* mean, float* rstd, unsigned* ticket, void* moments, size_t moments_bytes, hipStream_t s);

// same statistics with the library's built-in scratch (a file-scope device array) instead of a caller workspace
int launch_gn_stats_static(const void* x, int x_dtype, int n, int h, int w, int c, int groups, float eps,
                           float* mean, float* rstd, hipStream_t s);

// merges `slots` moment triples per (sample, group) from ws[n_groups][slots] into mean / rstd
int launch_gn_finalize(const void* ws, int n_groups, int slots, float eps, float* mean, float* rstd, hipStream_t s);

// kernels_misc.hip
int launch_upsample2x(const void* x, void* y, int dtype, int n, int h_in, int w_in, int c, hipStream_t s);
int launch_pack_conv(const void* src, int src_dtype, int cout, int cin, int k, void* dst, int op_dtype,
                     int dst_row_offset, int dst_rows_total, hipStream_t s);
// weights of a nearest-2x-upsample + 3x3 convolution: the 9-tap pack followed by the 16-tap phase pack
size_t upconv_phase_offset_bytes(int cout, int cin, int op_dtype);
size_t upconv_packed_bytes(int cout, int cin, int op_dtype);
int launch_pack_upconv(const void* src, int src_dtype, int cout, int cin, void* dst, int op_dtype, hipStream_t s);
// dst[n][i][j] (dst_dtype) = src[n][j][i] (src_dtype); src is [rows=j][cols=i] with row stride src_ld
int launch_transpose(const void* src, int src_dtype, void* dst, int dst_dtype, int batch, int rows, int cols,
                     size_t src_ld, size_t src_batch_stride, size_t dst_ld, size_t dst_batch_stride, hipStream_t s);
int launch_copy_f32(const float* src, float* dst, size_t count, hipStream_t s);
int launch_copy_u128(const void* src, void* dst, size_t bytes, hipStream_t s);   // bytes % 16 == 0
// out[i] = fma(scale, v[i], z[i]) in fp32, rounded once to out_dtype; z, v of `dtype`
int launch_axpy(const void* z, const void* v, int dtype, float scale, void* out, int out_dtype, size_t count, hipStream_t s);
int launch_zero_u32(void* p, int count, hipStream_t s);   // a fill kernel (safe under graph capture, unlike a memset node)

// kernels_adaln.hip: out[b][j] = bias[j] + sum_k w[j][k] * act(c[b][k]); w row-major [rows][d_cond], out fp32 [batch][rows]
int adaln_max_batch(int d_cond);   // conditioning vectors one launch can take (they are held in LDS)
int adaln_max_d_cond(int w_dtype);  // longest conditioning vector (a lane keeps a row's weights in registers)
int launch_adaln_projection(const void* c, int c_dtype, const void* w, int w_dtype, const float* bias, float* out, int batch,
                            int d_cond, int rows, int apply_silu, hipStream_t s);

// kernels_attn.hip
// q,k: [n][t][ld] rows of d elements (16-bit type), vt: [n][t_pad / 32][d][40] (V transposed in blocks of 32 keys, rows padded to 40 elements, keys past t zero), o: [n][t][d]
// scratch: flash_attention_scratch_bytes(n, t, d) bytes (partial outputs of the key splits), may be null if 0
size_t flash_attention_scratch_bytes(int n, int t, int d);
// elements of V^T per sample in the blocked, row-padded layout the kernel reads (see launch_transpose with dst_ld = 0)
size_t flash_attention_vt_elems(int t, int d);
int launch_flash_attention(const void* q, const void* k, size_t qk_ld, size_t qk_batch_stride,
                           const void* vt, int t_pad, void* o, void* scratch, int dtype, int n, int t, int d,
                           float scale, hipStream_t s);

}  // namespace wmdec
