// Horizontal fusion of the DiT's AdaLN projections (Sec. IV-B-2): the shift, scale and gate vectors of a block are
// three small products of the same conditioning vector; with the three weight matrices stored as one row-concatenated
// matrix they are one product, one launch, one pass over the weights.
//
// With a handful of conditioning vectors per call (one per frame) the product is a matrix-vector product: every weight
// is used `batch` times, far below the ridge point, so the bound is the single read of the weights from HBM and the
// matrix cores have nothing to add.  A wavefront owns eight weight rows at a time: a lane reads 16 contiguous bytes of
// each row per step (a wavefront's load is 1 KiB of one row), the activated conditioning vectors sit in LDS as fp32
// and are read once per step for all eight rows, partial sums stay in registers and are reduced over the 64 lanes at
// the end with a fixed butterfly.
#include "common.hpp"

namespace wmdec {
namespace {

constexpr int kRowsPerWave = 4;
constexpr int kWaves = 4;
constexpr int kMaxBatch = 16;
constexpr int kMaxLdsFloats = 16384;   // batch * d_cond fp32 values of the conditioning vectors (64 KiB)
constexpr int kMaxSteps = 8;           // 16-byte steps of a lane along a row: d_cond <= 8 * 64 * (16 / sizeof(weight))

template <typename T> struct Vec8 { static constexpr int N = 16 / sizeof(T); T v[16 / sizeof(T)]; };

// B: conditioning vectors the accumulators are sized for (batch rounded up); STEPS: 16-byte steps per lane and row.
// All RW x STEPS weight vectors of a wavefront are requested before the first is used: the kernel lives on loads in
// flight, and a loop that waits for one step before it asks for the next would pay the HBM latency STEPS times.
template <typename TW, int B, int STEPS>
__global__ __launch_bounds__(64 * kWaves) void adaln_projection_kernel(const void* __restrict__ c, int c_dtype, const TW* __restrict__ w,
                                                                       const float* __restrict__ bias, float* __restrict__ out,
                                                                       int batch, int d_cond, int rows, int apply_silu) {
  constexpr int V = 16 / sizeof(TW);   // weights per 16-byte load
  extern __shared__ __align__(16) float s_a[];   // [B][d_cond]; vectors past `batch` are zero
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row0 = (blockIdx.x * kWaves + wave) * kRowsPerWave;
  Vec8<TW> wv[kRowsPerWave][STEPS];
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r)   // rows and columns past the end re-read valid elements; they are masked below
#pragma unroll
    for (int st = 0; st < STEPS; ++st)
      wv[r][st] = *reinterpret_cast<const Vec8<TW>*>(w + (size_t)min(row0 + r, rows - 1) * d_cond + min((st * 64 + lane) * V, d_cond - V));
  // conditioning vectors -> LDS as fp32, activated; 16-byte loads, four in flight per thread (a loop that waits for
  // each load would cost more than the pass over the weights)
  {
    const int per = c_dtype == WMDEC_F32 ? 4 : 8;            // elements per 16-byte load
    const int nvec = batch * d_cond / per, total = B * d_cond / per;
    for (int i0 = tid; i0 < total; i0 += 4 * 64 * kWaves) {
      uint4 q[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) q[u] = reinterpret_cast<const uint4*>(c)[min(i0 + u * 64 * kWaves, nvec - 1)];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * 64 * kWaves;
        if (i >= total) continue;
        float t[8];
        if (c_dtype == WMDEC_F32) {
          t[0] = __uint_as_float(q[u].x); t[1] = __uint_as_float(q[u].y); t[2] = __uint_as_float(q[u].z); t[3] = __uint_as_float(q[u].w);
        } else {
          const uint32_t wd[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (c_dtype == WMDEC_BF16) { t[2 * e] = to_float(bf16_t{(uint16_t)(wd[e] & 0xffffu)}); t[2 * e + 1] = to_float(bf16_t{(uint16_t)(wd[e] >> 16)}); }
            else { t[2 * e] = to_float(f16_t{(uint16_t)(wd[e] & 0xffffu)}); t[2 * e + 1] = to_float(f16_t{(uint16_t)(wd[e] >> 16)}); }
          }
        }
        for (int e = 0; e < per; ++e) {
          float v = i < nvec ? t[e] : 0.f;
          if (apply_silu) v = silu_f(v);
          s_a[i * per + e] = v;
        }
      }
    }
  }
  __syncthreads();
  if (row0 >= rows) return;
  float acc[kRowsPerWave][B];
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r)
#pragma unroll
    for (int b = 0; b < B; ++b) acc[r][b] = 0.f;
#pragma unroll
  for (int st = 0; st < STEPS; ++st) {
    const int k0 = (st * 64 + lane) * V;
    if (k0 < d_cond) {
#pragma unroll
      for (int b = 0; b < B; ++b) {
        float a[V];
#pragma unroll
        for (int j = 0; j < V; j += 4) {
          const float4 q = *reinterpret_cast<const float4*>(s_a + b * d_cond + k0 + j);
          a[j] = q.x; a[j + 1] = q.y; a[j + 2] = q.z; a[j + 3] = q.w;
        }
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r)
#pragma unroll
          for (int j = 0; j < V; ++j) acc[r][b] = fmaf(to_float(wv[r][st].v[j]), a[j], acc[r][b]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < kRowsPerWave; ++r)
#pragma unroll
    for (int b = 0; b < B; ++b) {
      float v = acc[r][b];
      for (int mask = 32; mask > 0; mask >>= 1) v += __shfl_xor(v, mask);
      if (lane == 0 && row0 + r < rows && b < batch) out[(size_t)b * rows + row0 + r] = v + (bias ? bias[row0 + r] : 0.f);
    }
}

template <typename TW, int B, int STEPS>
int launch_k(const void* c, int c_dtype, const void* w, const float* bias, float* out, int batch, int d_cond, int rows, int silu, hipStream_t s) {
  const dim3 grid((unsigned)((rows + kWaves * kRowsPerWave - 1) / (kWaves * kRowsPerWave)));
  const size_t smem = (size_t)B * d_cond * sizeof(float);
  auto kern = adaln_projection_kernel<TW, B, STEPS>;
  if (smem > 48 * 1024) WMDEC_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
  hipLaunchKernelGGL(kern, grid, dim3(64 * kWaves), smem, s, c, c_dtype, (const TW*)w, bias, out, batch, d_cond, rows, silu);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

template <typename TW, int B>
int launch_s(const void* c, int c_dtype, const void* w, const float* bias, float* out, int batch, int d_cond, int rows, int silu, hipStream_t s) {
  const int steps = (d_cond + 64 * (16 / (int)sizeof(TW)) - 1) / (64 * (16 / (int)sizeof(TW)));
  if (steps <= 1) return launch_k<TW, B, 1>(c, c_dtype, w, bias, out, batch, d_cond, rows, silu, s);
  if (steps <= 2) return launch_k<TW, B, 2>(c, c_dtype, w, bias, out, batch, d_cond, rows, silu, s);
  if (steps <= 4) return launch_k<TW, B, 4>(c, c_dtype, w, bias, out, batch, d_cond, rows, silu, s);
  return launch_k<TW, B, 8>(c, c_dtype, w, bias, out, batch, d_cond, rows, silu, s);
}

template <typename TW>
int launch_b(const void* c, int c_dtype, const void* w, const float* bias, float* out, int batch, int d_cond, int rows, int silu, hipStream_t s) {
  if (batch <= 1) return launch_s<TW, 1>(c, c_dtype, w, bias, out, batch, d_cond, rows, silu, s);
  if (batch <= 2) return launch_s<TW, 2>(c, c_dtype, w, bias, out, batch, d_cond, rows, silu, s);
  if (batch <= 4) return launch_s<TW, 4>(c, c_dtype, w, bias, out, batch, d_cond, rows, silu, s);
  if (batch <= 8) return launch_s<TW, 8>(c, c_dtype, w, bias, out, batch, d_cond, rows, silu, s);
  return launch_s<TW, 16>(c, c_dtype, w, bias, out, batch, d_cond, rows, silu, s);
}

}  // namespace

// conditioning vectors one launch can take: the accumulators are sized for the batch rounded up to a power of two, and
// that many vectors of d_cond fp32 values must fit the LDS budget
int adaln_max_batch(int d_cond) {
  if (d_cond <= 0) return 0;
  int b = kMaxBatch;
  while (b > 1 && (long)b * d_cond > kMaxLdsFloats) b >>= 1;
  return (long)b * d_cond > kMaxLdsFloats ? 0 : b;
}

int adaln_max_d_cond(int w_dtype) { return kMaxSteps * 64 * (int)(16 / dtype_size(w_dtype)); }

int launch_adaln_projection(const void* c, int c_dtype, const void* w, int w_dtype, const float* bias, float* out, int batch,
                            int d_cond, int rows, int apply_silu, hipStream_t s) {
  switch (w_dtype) {
    case WMDEC_F32: return launch_b<float>(c, c_dtype, w, bias, out, batch, d_cond, rows, apply_silu, s);
    case WMDEC_BF16: return launch_b<bf16_t>(c, c_dtype, w, bias, out, batch, d_cond, rows, apply_silu, s);
    default: return launch_b<f16_t>(c, c_dtype, w, bias, out, batch, d_cond, rows, apply_silu, s);
  }
}

}  // namespace wmdec
