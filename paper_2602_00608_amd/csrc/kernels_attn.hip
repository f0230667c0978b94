// Single-head attention core, flash style: for a block of queries the keys are
// streamed in blocks of 32 through LDS, the scores live only in registers, and a
// running maximum / running sum rescale the output accumulator.
//
// The products are computed transposed so that no register transpose is needed:
//   S^T[key][query] = K * Q^T      (A = K rows from LDS, B = Q rows held in registers)
//   O^T[d][query]  += V^T * P^T    (A = V^T rows from LDS, B = P^T straight from the S^T registers)
// In both, one lane owns one query column (n = lane % 16), so the softmax row
// statistics are per lane plus a reduction over the 4 lanes that share a query.
#include "mfma.hpp"

namespace wmdec {
namespace {

constexpr int D = 512;            // head dimension
constexpr int KB = 32;            // keys per block
constexpr int QW = 16;            // queries per wavefront
constexpr int WAVES = 4;
constexpr int QB = QW * WAVES;    // queries per workgroup
constexpr int K_LD = D + 8;       // LDS row stride of the K tile (elements): +16 B against bank conflicts
constexpr int V_LD = KB + 4;      // LDS row stride of the V^T tile (elements)

template <typename T>
__global__ __launch_bounds__(256) void flash_attn_kernel(const T* __restrict__ q, const T* __restrict__ k, size_t ld,
                                                         size_t batch_stride, const T* __restrict__ vt, int t_pad,
                                                         T* __restrict__ o, int t, float scale_log2e) {
  extern __shared__ __align__(16) unsigned char smem[];
  T* s_k = reinterpret_cast<T*>(smem);                 // [KB][K_LD]
  T* s_v = s_k + KB * K_LD;                            // [D][V_LD]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = blockIdx.y;
  const int q0 = blockIdx.x * QB + wave * QW;
  const int lq = lane & 15, lg = lane >> 4;            // query column, lane group
  q += (size_t)n * batch_stride; k += (size_t)n * batch_stride;
  vt += (size_t)n * D * t_pad; o += (size_t)n * t * D;

  // Q fragment: B[k = d][n = query] = Q[q0 + lq][32*step + 8*lg + j]
  u32x4 qf[D / 32];
  {
    const int qr = min(q0 + lq, t - 1);
    const u32x4* src = reinterpret_cast<const u32x4*>(q + (size_t)qr * ld);
#pragma unroll
    for (int st = 0; st < D / 32; ++st) qf[st] = src[st * 4 + lg];
  }

  f32x4 acc[D / 16];
#pragma unroll
  for (int i = 0; i < D / 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  for (int kb = 0; kb < t; kb += KB) {
    __syncthreads();
    // K tile: KB rows of D elements, 16 B per thread
    for (int i = tid; i < KB * (D / 8); i += 256) {
      const int r = i / (D / 8), c = i % (D / 8);
      u32x4 v = u32x4{0u, 0u, 0u, 0u};
      if (kb + r < t) v = reinterpret_cast<const u32x4*>(k + (size_t)(kb + r) * ld)[c];
      *reinterpret_cast<u32x4*>(s_k + r * K_LD + c * 8) = v;
    }
    // V^T tile: D rows of KB keys; keys >= t are zeroed
    for (int i = tid; i < D * (KB / 8); i += 256) {
      const int r = i / (KB / 8), c = i % (KB / 8);
      const int key = kb + c * 8;
      u32x4 v = u32x4{0u, 0u, 0u, 0u};
      if (key < t_pad) v = reinterpret_cast<const u32x4*>(vt + (size_t)r * t_pad + key)[0];
      if (key + 8 > t) {
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (key + e >= t) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
        v = u32x4{w[0], w[1], w[2], w[3]};
      }
      T* dst = s_v + r * V_LD + c * 8;
      *reinterpret_cast<u32x2*>(dst) = u32x2{v.x, v.y};
      *reinterpret_cast<u32x2*>(dst + 4) = u32x2{v.z, v.w};
    }
    __syncthreads();

    // S^T tiles: keys kb + 16*tile + 4*lg + r, query q0 + lq
    f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
    for (int st = 0; st < D / 32; ++st) {
      const u32x4 a0 = *reinterpret_cast<const u32x4*>(s_k + lq * K_LD + st * 32 + lg * 8);
      const u32x4 a1 = *reinterpret_cast<const u32x4*>(s_k + (16 + lq) * K_LD + st * 32 + lg * 8);
      s0 = Mma<T>::m16(a0, qf[st], s0);
      s1 = Mma<T>::m16(a1, qf[st], s1);
    }
    float sv[8];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      sv[r] = (kb + 4 * lg + r < t) ? s0[r] * scale_log2e : -INFINITY;
      sv[4 + r] = (kb + 16 + 4 * lg + r < t) ? s1[r] * scale_log2e : -INFINITY;
    }
    float bm = sv[0];
#pragma unroll
    for (int r = 1; r < 8; ++r) bm = fmaxf(bm, sv[r]);
    bm = fmaxf(bm, __shfl_xor(bm, 16));
    bm = fmaxf(bm, __shfl_xor(bm, 32));
    const float m_new = fmaxf(m_run, bm);   // finite: every block holds at least one valid key
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    float p[8], ps = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) { p[r] = __builtin_amdgcn_exp2f(sv[r] - m_new); ps += p[r]; }
    l_run = l_run * alpha + ps;
    m_run = m_new;
    // P^T fragment: contraction slots 8*lg + j  <->  keys {4*lg + j (tile 0), 16 + 4*lg + j - 4 (tile 1)}
    const u32x4 pf = u32x4{pack2<T>(p[0], p[1]), pack2<T>(p[2], p[3]), pack2<T>(p[4], p[5]), pack2<T>(p[6], p[7])};
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      const T* row = s_v + (dt * 16 + lq) * V_LD;
      const u32x2 lo = *reinterpret_cast<const u32x2*>(row + 4 * lg);
      const u32x2 hi = *reinterpret_cast<const u32x2*>(row + 16 + 4 * lg);
      f32x4 c = acc[dt];
      c *= alpha;
      acc[dt] = Mma<T>::m16(u32x4{lo.x, lo.y, hi.x, hi.y}, pf, c);
    }
  }

  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  const float inv = 1.0f / l_run;
  const int qr = q0 + lq;
  if (qr < t) {
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      const f32x4 c = acc[dt];
      const u32x2 w = u32x2{pack2<T>(c[0] * inv, c[1] * inv), pack2<T>(c[2] * inv, c[3] * inv)};
      *reinterpret_cast<u32x2*>(o + (size_t)qr * D + dt * 16 + 4 * lg) = w;
    }
  }
}

}  // namespace

int launch_flash_attention(const void* q, const void* k, size_t qk_ld, size_t qk_batch_stride, const void* vt,
                           int t_pad, void* o, int dtype, int n, int t, int d, float scale, hipStream_t s) {
  WMDEC_REQUIRE(d == D, WMDEC_ERR_UNSUPPORTED, "attention: head dimension %d is not supported (only %d)", d, D);
  WMDEC_REQUIRE(is_16bit(dtype), WMDEC_ERR_UNSUPPORTED, "attention: dtype must be BF16 or F16");
  WMDEC_REQUIRE(t_pad % 8 == 0 && t_pad >= t && qk_ld % 8 == 0, WMDEC_ERR_SHAPE, "attention: bad leading dimensions");
  const size_t smem = (size_t)(KB * K_LD + D * V_LD) * 2;
  dim3 grid((unsigned)((t + QB - 1) / QB), (unsigned)n);
  const float sl = scale * 1.4426950408889634f;
  if (dtype == WMDEC_BF16) {
    WMDEC_HIP(hipFuncSetAttribute((const void*)flash_attn_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    hipLaunchKernelGGL(flash_attn_kernel<bf16_t>, grid, dim3(256), smem, s, (const bf16_t*)q, (const bf16_t*)k, qk_ld,
                       qk_batch_stride, (const bf16_t*)vt, t_pad, (bf16_t*)o, t, sl);
  } else {
    WMDEC_HIP(hipFuncSetAttribute((const void*)flash_attn_kernel<f16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    hipLaunchKernelGGL(flash_attn_kernel<f16_t>, grid, dim3(256), smem, s, (const f16_t*)q, (const f16_t*)k, qk_ld,
                       qk_batch_stride, (const f16_t*)vt, t_pad, (f16_t*)o, t, sl);
  }
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

}  // namespace wmdec
