// General convolution on the vector ALUs: any channel counts, any supported
// dtype, 3x3 or 1x1, optional normalise(+SiLU)-on-load, folded nearest-2x
// upsample, bias and residual in the epilogue, NHWC or NCHW at either end.
// It is the fp32 path (operands and FMAs in fp32) and the path for shapes the
// matrix-core kernel does not take (C_in = 4 of conv_in, C_out = 3 of conv_out).
// For 16-bit operand types the activated input is rounded to that type before
// the product and accumulated in fp32, i.e. the arithmetic of the MFMA kernel.
#include "moments.hpp"
#include "pack_layout.hpp"

namespace wmdec {
namespace {

constexpr int TH = 8, TW = 8;     // output pixels per workgroup: 8 x 8
constexpr int TCO = 64;           // output channels per workgroup
constexpr int KC = 8;             // input channels per LDS stage
constexpr int HALO = TW + 2;      // staged tile is (TH+2) x (TW+2) for 3x3

__device__ __forceinline__ float load_as_float(const void* p, int dtype, size_t i) {
  switch (dtype) {
    case WMDEC_F32: return ((const float*)p)[i];
    case WMDEC_BF16: return to_float(((const bf16_t*)p)[i]);
    default: return to_float(((const f16_t*)p)[i]);
  }
}
__device__ __forceinline__ void store_from_float(void* p, int dtype, size_t i, float v) {
  switch (dtype) {
    case WMDEC_F32: ((float*)p)[i] = v; break;
    case WMDEC_BF16: ((bf16_t*)p)[i] = from_float<bf16_t>(v); break;
    default: ((f16_t*)p)[i] = from_float<f16_t>(v); break;
  }
}
__device__ __forceinline__ float round_op(float v, int op_dtype) {
  switch (op_dtype) {
    case WMDEC_F32: return v;
    case WMDEC_BF16: return round_through<bf16_t>(v);
    default: return round_through<f16_t>(v);
  }
}

struct DirectParams {
  const void* x; const float* mean; const float* rstd; const float* gamma; const float* beta;
  const void* w; const float* bias; const void* res; void* y;
  int x_dtype, op_dtype, res_dtype, y_dtype;
  int x_nchw, y_nchw, silu, groups;
  int n, h, w_out, cin, cout, ksize, upsample;
  int tiles_x;
};

__global__ __launch_bounds__(256) void conv_direct_kernel(DirectParams p) {
  __shared__ float s_in[(TH + 2) * HALO][KC + 1];
  __shared__ float s_w[9][KC][TCO];
  __shared__ float s_scale[KC], s_mean[KC], s_beta[KC];

  const int tid = threadIdx.x;
  const int tile = blockIdx.x;
  const int ty0 = (tile / p.tiles_x) * TH, tx0 = (tile % p.tiles_x) * TW;
  const int co0 = blockIdx.y * TCO;
  const int n = blockIdx.z;
  const int pad = p.ksize / 2;
  const int taps = p.ksize * p.ksize;
  const int h_in = p.upsample ? p.h / 2 : p.h, w_in = p.upsample ? p.w_out / 2 : p.w_out;
  const int cpg = p.mean ? p.cin / p.groups : 1;
  const int cinb = packed_cin_blocks(p.cin), coutb = packed_cout_blocks(p.cout);

  // thread -> 4 pixels (one row segment) x 4 output channels
  const int pg = tid & 15, cg = tid >> 4;
  const int py = pg >> 1, px0 = (pg & 1) * 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  const int halo_w = TW + 2 * pad, halo_h = TH + 2 * pad;
  for (int c0 = 0; c0 < p.cin; c0 += KC) {
    __syncthreads();
    if (tid < KC) {
      const int c = c0 + tid;
      float sc = 1.f, mu = 0.f, be = 0.f;
      if (p.mean && c < p.cin) {
        const int g = c / cpg;
        sc = p.gamma[c] * p.rstd[n * p.groups + g];
        mu = p.mean[n * p.groups + g];
        be = p.beta[c];
      }
      s_scale[tid] = sc; s_mean[tid] = mu; s_beta[tid] = be;
    }
    // weights of this channel chunk: s_w[tap][k][co]
    for (int i = tid; i < taps * KC * TCO; i += 256) {
      const int k = i % KC, co = (i / KC) % TCO, tap = i / (KC * TCO);
      float v = 0.f;
      if (co0 + co < p.cout && c0 + k < p.cin)
        v = load_as_float(p.w, p.op_dtype, packed_index(tap, co0 + co, c0 + k, cinb, coutb));
      s_w[tap][k][co] = v;
    }
    __syncthreads();
    // activated input tile with halo; zero outside the (upsampled) image
    for (int i = tid; i < halo_h * halo_w * KC; i += 256) {
      const int k = i % KC, hp = i / KC;
      const int hy = hp / halo_w, hx = hp % halo_w;
      const int gy = ty0 + hy - pad, gx = tx0 + hx - pad;  // position on the output grid
      const int c = c0 + k;
      float v = 0.f;
      if (gy >= 0 && gy < p.h && gx >= 0 && gx < p.w_out && c < p.cin) {
        const int sy = p.upsample ? (gy >> 1) : gy, sx = p.upsample ? (gx >> 1) : gx;
        const size_t idx = p.x_nchw ? (((size_t)n * p.cin + c) * h_in + sy) * w_in + sx
                                    : (((size_t)n * h_in + sy) * w_in + sx) * p.cin + c;
        v = load_as_float(p.x, p.x_dtype, idx);
        if (p.mean) {
          v = fmaf(v - s_mean[k], s_scale[k], s_beta[k]);  // subtract first: no cancellation when |mean| >> std
          if (p.silu) v = silu_f(v);
        }
        v = round_op(v, p.op_dtype);
      }
      s_in[hy * HALO + hx][k] = v;
    }
    __syncthreads();
    for (int tap = 0; tap < taps; ++tap) {
      const int ky = tap / p.ksize, kx = tap % p.ksize;
#pragma unroll
      for (int k = 0; k < KC; ++k) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = s_in[(py + ky) * HALO + px0 + i + kx][k];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = s_w[tap][k][cg * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
    }
  }

  const int oy = ty0 + py;
  if (oy >= p.h) return;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ox = tx0 + px0 + i;
    if (ox >= p.w_out) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int co = co0 + cg * 4 + j;
      if (co >= p.cout) continue;
      float v = acc[i][j];
      if (p.bias) v += p.bias[co];
      const size_t nhwc = (((size_t)n * p.h + oy) * p.w_out + ox) * p.cout + co;
      if (p.res) v += load_as_float(p.res, p.res_dtype, nhwc);
      const size_t oi = p.y_nchw ? (((size_t)n * p.cout + co) * p.h + oy) * p.w_out + ox : nhwc;
      store_from_float(p.y, p.y_dtype, oi, v);
    }
  }
}

// 3x3 convolution with very few input channels (the decoder's conv_in, C_in = 4): far too little contraction for
// the matrix cores, and the general kernel above spends its time staging.  A thread owns one output channel and
// keeps that channel's 9 x CI weights in registers (the packed layout stores the first 8 input channels of a
// (tap, output channel) pair as 16 contiguous bytes); a workgroup walks a row segment of 32 pixels whose
// three-row halo strip sits in LDS (operands rounded to the operand type, zeros outside the image), so every
// input value is one broadcast LDS read for 256 output channels.  Bias in the epilogue, NHWC output.
// With x_step the input of sample n is formed while it is staged: x[0] + (n + 1) * step_scale * x_step (one fp32
// fused multiply-add, then the one rounding to the operand type): n + 1 first-order extrapolation steps of a latent
// along its motion vector (Alg. 2, hit branch), so a batch of extrapolated latents never exists in memory.
constexpr int SP = 48;    // pixels per workgroup: two segments per row of the 90-pixel latent
constexpr int SCO = 64;   // output channels per workgroup: lane = channel
constexpr int SQ = 4;     // the pixels of a segment are dealt to the four wavefronts in runs of SP / SQ

template <int CI, typename TW_, typename TO>
__global__ __launch_bounds__(256) void conv_small_cin_kernel(const void* __restrict__ x, int x_dtype, int x_nchw,
                                                             const void* __restrict__ x_step, float step_scale,
                                                             const TW_* __restrict__ w, const float* __restrict__ bias,
                                                             TO* __restrict__ y, int h, int w_out, int cin, int cout,
                                                             Moments* __restrict__ stats, int stats_cpg, int stats_groups) {
  __shared__ __align__(16) float s_in[3][SP + 2][CI];
  __shared__ Moments s_m[SQ][SCO];
  const int tid = threadIdx.x, lane = tid & 63, q = tid >> 6;
  const int segs = (w_out + SP - 1) / SP;
  const int oy = blockIdx.x / segs, x0 = (blockIdx.x % segs) * SP;
  const int co = blockIdx.y * SCO + lane;
  const int n = blockIdx.z;
  for (int i = tid; i < 3 * (SP + 2) * CI; i += 256) {
    const int c = i % CI, hx = (i / CI) % (SP + 2), hy = i / (CI * (SP + 2));
    const int gy = oy + hy - 1, gx = x0 + hx - 1;
    float v = 0.f;
    if (c < cin && gy >= 0 && gy < h && gx >= 0 && gx < w_out) {
      const size_t xn = x_step ? 0 : n;
      const size_t idx = x_nchw ? ((xn * cin + c) * h + gy) * w_out + gx : ((xn * h + gy) * w_out + gx) * cin + c;
      v = load_as_float(x, x_dtype, idx);
      if (x_step) v = fmaf((float)(n + 1) * step_scale, load_as_float(x_step, x_dtype, idx), v);
      v = round_through<TW_>(v);
    }
    s_in[hy][hx][c] = v;
  }
  float wr[9][CI];
  const int coutb = packed_cout_blocks(cout), cinb = packed_cin_blocks(cin);
  const int cc = min(co, cout - 1);
#pragma unroll
  for (int tap = 0; tap < 9; ++tap) {
    const TW_* src = w + packed_index(tap, cc, 0, cinb, coutb);   // input channels 0..7 of (tap, cc): 16 contiguous bytes
#pragma unroll
    for (int c = 0; c < CI; ++c) wr[tap][c] = to_float(src[c]);
  }
  const float bv = bias ? bias[cc] : 0.f;
  __syncthreads();
  const bool live = co < cout;
  TO* yrow = y + (((size_t)n * h + oy) * w_out + x0) * cout + cc;
  const int npx = min(SP, w_out - x0);
  Moments m = {0.f, 0.f, 0.f};   // of this channel's stored values, one value at a time (Welford)
  const int p0 = q * (SP / SQ), p1 = min(p0 + SP / SQ, npx);
  for (int px = p0; px < p1; ++px) {
    float acc = bv;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
      for (int c = 0; c < CI; ++c) acc = fmaf(s_in[tap / 3][px + tap % 3][c], wr[tap][c], acc);
    const TO stored = from_float<TO>(acc);
    if (live) yrow[(size_t)px * cout] = stored;
    const float v = to_float(stored), d = v - m.mean;
    m.n += 1.f;
    m.mean += d * __builtin_amdgcn_rcpf(m.n);
    m.m2 = fmaf(d, v - m.mean, m.m2);
  }
  // GroupNorm moments of y for the next layer: the channels of a group are stats_cpg consecutive lanes (the launcher
  // checks that groups do not straddle wavefronts or the end of the channels); the four wavefronts' triples of a group
  // are merged in wavefront order: one triple per (sample, group, workgroup)
  if (stats) {
    s_m[q][lane] = merge_to_first(m, lane, stats_cpg);
    __syncthreads();
    if (q == 0 && live && lane % stats_cpg == 0) {
      Moments t = s_m[0][lane];
#pragma unroll
      for (int k = 1; k < SQ; ++k) t = merge(t, s_m[k][lane]);
      stats[((size_t)n * stats_groups + co / stats_cpg) * ((size_t)segs * h) + blockIdx.x] = t;
    }
  }
}

template <int CI, typename TW_>
int launch_small_cin_t(const ConvArgs& a, hipStream_t s) {
  const int segs = (a.w + SP - 1) / SP;
  dim3 grid((unsigned)(segs * a.h), (unsigned)((a.cout + SCO - 1) / SCO), (unsigned)a.n);
  const int cpg = a.stats_ws ? a.cout / a.stats_groups : 1;
  switch (a.y_dtype) {
    case WMDEC_F32: hipLaunchKernelGGL((conv_small_cin_kernel<CI, TW_, float>), grid, dim3(256), 0, s, a.x, a.x_dtype, a.x_nchw, a.x_step, a.step_scale, (const TW_*)a.wt, a.bias, (float*)a.y, a.h, a.w, a.cin, a.cout, (Moments*)a.stats_ws, cpg, a.stats_groups); break;
    case WMDEC_BF16: hipLaunchKernelGGL((conv_small_cin_kernel<CI, TW_, bf16_t>), grid, dim3(256), 0, s, a.x, a.x_dtype, a.x_nchw, a.x_step, a.step_scale, (const TW_*)a.wt, a.bias, (bf16_t*)a.y, a.h, a.w, a.cin, a.cout, (Moments*)a.stats_ws, cpg, a.stats_groups); break;
    default: hipLaunchKernelGGL((conv_small_cin_kernel<CI, TW_, f16_t>), grid, dim3(256), 0, s, a.x, a.x_dtype, a.x_nchw, a.x_step, a.step_scale, (const TW_*)a.wt, a.bias, (f16_t*)a.y, a.h, a.w, a.cin, a.cout, (Moments*)a.stats_ws, cpg, a.stats_groups); break;
  }
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

}  // namespace

// Triples per (sample, group) this kernel emits for its output, 0 if it cannot: a group must be a power-of-two run of
// at most 64 lanes (= channels), so that no group straddles a wavefront, a workgroup or the end of the channels.
int conv_small_cin_stats_slots(const ConvArgs& a) {
  if (a.stats_groups < 1 || a.cout % a.stats_groups != 0) return 0;
  const int cpg = a.cout / a.stats_groups;
  if (cpg > 64 || (cpg & (cpg - 1)) != 0) return 0;
  return (a.w + SP - 1) / SP * a.h;
}

bool conv_small_cin_supported(const ConvArgs& a) {
  return a.ksize == 3 && !a.upsample && a.cin <= 8 && !a.mean && !a.groups_norm && !a.rows_in && !a.res && !a.x2 && !a.y_nchw &&
         is_16bit(a.op_dtype) && !a.rows_out && (a.stats_ws == nullptr || conv_small_cin_stats_slots(a) > 0);
}

int launch_conv_small_cin(const ConvArgs& a, hipStream_t s) {
  if (a.cin <= 4)
    return a.op_dtype == WMDEC_BF16 ? launch_small_cin_t<4, bf16_t>(a, s) : launch_small_cin_t<4, f16_t>(a, s);
  return a.op_dtype == WMDEC_BF16 ? launch_small_cin_t<8, bf16_t>(a, s) : launch_small_cin_t<8, f16_t>(a, s);
}

int launch_conv_direct(const ConvArgs& a, hipStream_t s) {
  DirectParams p;
  p.x = a.x; p.mean = a.mean; p.rstd = a.rstd; p.gamma = a.gamma; p.beta = a.beta;
  p.w = a.wt; p.bias = a.bias; p.res = a.res; p.y = a.y;
  p.x_dtype = a.x_dtype; p.op_dtype = a.op_dtype; p.res_dtype = a.res_dtype; p.y_dtype = a.y_dtype;
  p.x_nchw = a.x_nchw; p.y_nchw = a.y_nchw; p.silu = a.silu; p.groups = a.groups;
  p.n = a.n; p.h = a.h; p.w_out = a.w; p.cin = a.cin; p.cout = a.cout; p.ksize = a.ksize; p.upsample = a.upsample;
  p.tiles_x = (a.w + TW - 1) / TW;
  const int tiles_y = (a.h + TH - 1) / TH;
  dim3 grid((unsigned)(p.tiles_x * tiles_y), (unsigned)((a.cout + TCO - 1) / TCO), (unsigned)a.n);
  hipLaunchKernelGGL(conv_direct_kernel, grid, dim3(256), 0, s, p);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

}  // namespace wmdec
