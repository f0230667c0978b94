// Single-head attention core, flash style, for head dimension 512: keys are streamed in blocks of 32 through
// LDS, the scores live only in registers and (as 16-bit probabilities) in a 5 KiB LDS tile, and a running
// maximum / running sum rescale the output accumulator.
//
// A workgroup of 8 wavefronts owns 64 queries.  With d = 512 a wavefront cannot hold both a query fragment and
// an output accumulator for all of d without spilling, so the two products are split differently:
//   scores   S^T[key][query] = K * Q^T : wavefronts 0..3, 16 queries each, all 32 keys, the whole contraction
//            over d (A = K rows from LDS, B = the wavefront's Q rows, held in registers for the whole kernel).
//            One lane owns one query column, so the softmax statistics are per lane plus a reduction over the 4
//            lanes that share a query; the probabilities go to LDS as P[query][key] with the block's rescale
//            factor per query.
//   output   O^T[d][query] += V^T * P^T : all 8 wavefronts, each a 64-wide slice of d for all 64 queries
//            (A = V^T rows from LDS, B = P rows from LDS, 32x32x16 MFMAs); again a lane owns a query column,
//            so the rescale factor and the final 1/sum are one value per lane and query tile.
// Per key block a SIMD thus runs 512 cycles of score MFMAs (one wavefront) and 512 of output MFMAs (two).
// To fill 256 compute units with only T/64 query blocks the keys are split into `splits` ranges handled by
// different workgroups, each writing an unnormalised partial output with its (max, sum); attn_combine merges
// them in a fixed order.  The next K tile is fetched into registers during the score phase and the next V^T
// tile during the output phase (two barriers per key block).
#include "mfma.hpp"

namespace wmdec {
namespace {

constexpr int D = 512;            // head dimension
constexpr int KB = 32;            // keys per block
constexpr int QW = 16;            // queries per score wavefront
constexpr int SW = 4;             // score wavefronts
constexpr int WAVES = 8;
constexpr int NT = WAVES * 64;    // threads per workgroup
constexpr int QB = QW * SW;       // queries per workgroup
constexpr int DS = D / WAVES;     // slice of d per wavefront in the output product
constexpr int K_LD = D + 8;       // LDS row stride of the K tile (elements): +16 B against bank conflicts
constexpr int V_LD = KB + 8;      // LDS row stride of the V^T tile
constexpr int P_LD = KB + 8;      // LDS row stride of the probability tile
constexpr int KV = KB * (D / 8) / NT;   // 16-byte vectors of a tile per thread (= 4)
constexpr size_t kSmemBytes = (size_t)(KB * K_LD + D * V_LD + QB * P_LD) * 2 + 2 * QB * sizeof(float);

template <typename T>
__global__ __launch_bounds__(NT) void flash_attn_kernel(const T* __restrict__ q, const T* __restrict__ k, size_t ld,
                                                        size_t batch_stride, const T* __restrict__ vt, int t_pad,
                                                        T* __restrict__ o, float* __restrict__ opart,
                                                        float* __restrict__ ml, int t, int splits, float scale_log2e) {
  extern __shared__ __align__(16) unsigned char smem[];
  T* s_k = reinterpret_cast<T*>(smem);                 // [KB][K_LD]
  T* s_v = s_k + KB * K_LD;                            // [D][V_LD]
  T* s_p = s_v + D * V_LD;                             // [QB][P_LD]
  float* s_alpha = reinterpret_cast<float*>(s_p + QB * P_LD);   // [QB] rescale factor of the block, later 1/sum
  float* s_l = s_alpha + QB;                           // [QB] final sums

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = blockIdx.z, split = blockIdx.y;
  const int qb0 = blockIdx.x * QB;
  const int lq = lane & 15, lg = lane >> 4;            // score phase: query column, lane group
  const int l32 = lane & 31, lh = lane >> 5;           // output phase: query column within a tile, contraction half
  q += (size_t)n * batch_stride; k += (size_t)n * batch_stride;
  vt += (size_t)n * D * t_pad;
  // key blocks of this split
  const int nkb = (t + KB - 1) / KB;
  const int kb_begin = (int)((long)split * nkb / splits) * KB, kb_end = (int)((long)(split + 1) * nkb / splits) * KB;

  // Q fragment of a score wavefront: B[k = d][n = query] = Q[qb0 + 16*wave + lq][32*step + 8*lg + j]
  u32x4 qf[D / 32];
  if (wave < SW) {
    const int qr = min(qb0 + wave * QW + lq, t - 1);
    const u32x4* src = reinterpret_cast<const u32x4*>(q + (size_t)qr * ld);
#pragma unroll
    for (int st = 0; st < D / 32; ++st) qf[st] = src[st * 4 + lg];
  }
  f32x16 acc[2][2];   // [d tile][query tile] of O^T
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // staging: thread -> KV vectors of the K tile (row r, 16-byte column c) and of the V^T tile (row d, 8 keys)
  u32x4 pre[KV], prev[KV];   // next K tile, next V^T tile: both fetched at the start of a key block
  auto load_k = [&](int kb) {
#pragma unroll
    for (int i = 0; i < KV; ++i) {
      const int v = tid + i * NT, r = v / (D / 8), c = v % (D / 8);
      pre[i] = reinterpret_cast<const u32x4*>(k + (size_t)min(kb + r, t - 1) * ld)[c];   // rows past t are masked later
    }
  };
  auto store_k = [&]() {
#pragma unroll
    for (int i = 0; i < KV; ++i) {
      const int v = tid + i * NT, r = v / (D / 8), c = v % (D / 8);
      *reinterpret_cast<u32x4*>(s_k + r * K_LD + c * 8) = pre[i];
    }
  };
  auto load_v = [&](int kb) {
#pragma unroll
    for (int i = 0; i < KV; ++i) {
      const int v = tid + i * NT, r = v / (KB / 8), c = v % (KB / 8);
      prev[i] = reinterpret_cast<const u32x4*>(vt + (size_t)r * t_pad + min(kb, t_pad - KB) + c * 8)[0];
    }
  };
  auto store_v = [&](int kb) {   // keys >= t are zeroed: their probability is 0 but 0 * garbage could be NaN
#pragma unroll
    for (int i = 0; i < KV; ++i) {
      const int v = tid + i * NT, r = v / (KB / 8), c = v % (KB / 8);
      const int key = kb + c * 8;
      uint32_t w[4] = {prev[i].x, prev[i].y, prev[i].z, prev[i].w};
      if (key + 8 > t) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (key + e >= t) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
      }
      *reinterpret_cast<u32x4*>(s_v + r * V_LD + c * 8) = u32x4{w[0], w[1], w[2], w[3]};
    }
  };

  if (kb_begin < kb_end) {
    load_k(kb_begin); store_k();
    load_v(kb_begin); store_v(kb_begin);
  }
  __syncthreads();

  for (int kb = kb_begin; kb < kb_end; kb += KB) {
    const int kn = min(kb + KB, kb_end - KB);   // next block (the last iteration reloads its own: harmless)
    load_k(kn);
    load_v(kn);
    if (wave < SW) {
      // S^T tiles: keys kb + 16*tile + 4*lg + r, query qb0 + 16*wave + lq
      // K fragments are read from LDS PF contraction steps ahead of the MFMAs that consume them; the scheduling
      // barriers keep that distance (left alone, the compiler sinks each read to its use and every step pays
      // the LDS latency)
      f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
      constexpr int PF = 3;
      u32x4 ka[PF][2];
      const T* krow0 = s_k + lq * K_LD + lg * 8;
      const T* krow1 = krow0 + 16 * K_LD;
#pragma unroll
      for (int st = 0; st < PF; ++st) {
        ka[st][0] = *reinterpret_cast<const u32x4*>(krow0 + st * 32);
        ka[st][1] = *reinterpret_cast<const u32x4*>(krow1 + st * 32);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int st = 0; st < D / 32; ++st) {
        s0 = Mma<T>::m16(ka[st % PF][0], qf[st], s0);
        s1 = Mma<T>::m16(ka[st % PF][1], qf[st], s1);
        if (st + PF < D / 32) {
          ka[st % PF][0] = *reinterpret_cast<const u32x4*>(krow0 + (st + PF) * 32);
          ka[st % PF][1] = *reinterpret_cast<const u32x4*>(krow1 + (st + PF) * 32);
        }
        __builtin_amdgcn_sched_barrier(0);
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
      float pr[8], ps = 0.f;
#pragma unroll
      for (int r = 0; r < 8; ++r) { pr[r] = __builtin_amdgcn_exp2f(sv[r] - m_new); ps += pr[r]; }
      l_run = l_run * alpha + ps;
      m_run = m_new;
      T* prow = s_p + (wave * QW + lq) * P_LD;
      *reinterpret_cast<u32x2*>(prow + 4 * lg) = u32x2{pack2<T>(pr[0], pr[1]), pack2<T>(pr[2], pr[3])};
      *reinterpret_cast<u32x2*>(prow + 16 + 4 * lg) = u32x2{pack2<T>(pr[4], pr[5]), pack2<T>(pr[6], pr[7])};
      if (lg == 0) s_alpha[wave * QW + lq] = alpha;
    }
    __syncthreads();            // probabilities and rescale factors visible; every wavefront is done with the K tile
    store_k();                  // next K tile
    {
      const float al0 = s_alpha[l32], al1 = s_alpha[32 + l32];
      if (__any(al0 != 1.0f || al1 != 1.0f)) {
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) { acc[dt][0] *= al0; acc[dt][1] *= al1; }
      }
#pragma unroll
      for (int ks = 0; ks < KB / 16; ++ks) {
        u32x4 pf[2], vf[2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) pf[qt] = *reinterpret_cast<const u32x4*>(s_p + (qt * 32 + l32) * P_LD + ks * 16 + lh * 8);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) vf[dt] = *reinterpret_cast<const u32x4*>(s_v + (wave * DS + dt * 32 + l32) * V_LD + ks * 16 + lh * 8);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int qt = 0; qt < 2; ++qt) acc[dt][qt] = Mma<T>::m32(vf[dt], pf[qt], acc[dt][qt]);
      }
    }
    __syncthreads();            // every wavefront is done with the V^T and probability tiles; next K tile visible
    store_v(kn);
  }

  // final sums per query (and, for split keys, the running maxima) from the score wavefronts
  if (wave < SW) {
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    const int ql = wave * QW + lq, qr = qb0 + ql;
    if (lg == 0) {
      s_l[ql] = l_run;
      if (splits > 1 && qr < t) {
        const size_t row = ((size_t)n * splits + split) * t + qr;
        ml[row * 2] = m_run; ml[row * 2 + 1] = l_run;
      }
    }
  }
  __syncthreads();
  // O^T tile element r of lane: d = wave*DS + dt*32 + 8*(r/4) + 4*lh + r%4, query = qb0 + qt*32 + l32
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const int qr = qb0 + qt * 32 + l32;
    if (qr >= t) continue;
    if (splits == 1) {
      const float inv = 1.0f / s_l[qt * 32 + l32];
      T* orow = o + ((size_t)n * t + qr) * D + wave * DS + 4 * lh;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x16& c = acc[dt][qt];
          *reinterpret_cast<u32x2*>(orow + dt * 32 + g * 8) =
              u32x2{pack2<T>(c[4 * g] * inv, c[4 * g + 1] * inv), pack2<T>(c[4 * g + 2] * inv, c[4 * g + 3] * inv)};
        }
    } else {
      float* prow = opart + (((size_t)n * splits + split) * t + qr) * D + wave * DS + 4 * lh;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x16& c = acc[dt][qt];
          *reinterpret_cast<f32x4*>(prow + dt * 32 + g * 8) = f32x4{c[4 * g], c[4 * g + 1], c[4 * g + 2], c[4 * g + 3]};
        }
    }
  }
}

// o[n][q][:] = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M), splits merged in index order.
// One workgroup of 128 threads per query, 4 consecutive d per thread.
template <typename T>
__global__ __launch_bounds__(128) void attn_combine_kernel(const float* __restrict__ opart, const float* __restrict__ ml,
                                                           T* __restrict__ o, int t, int splits) {
  const int qr = blockIdx.x, n = blockIdx.y, d0 = threadIdx.x * 4;
  float mx = -INFINITY;
  for (int s = 0; s < splits; ++s) mx = fmaxf(mx, ml[(((size_t)n * splits + s) * t + qr) * 2]);
  float den = 0.f;
  f32x4 num = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    const size_t row = ((size_t)n * splits + s) * t + qr;
    const float w = __builtin_amdgcn_exp2f(ml[row * 2] - mx);
    den += w * ml[row * 2 + 1];
    num += w * *reinterpret_cast<const f32x4*>(opart + row * D + d0);
  }
  const float inv = 1.0f / den;
  *reinterpret_cast<u32x2*>(o + ((size_t)n * t + qr) * D + d0) =
      u32x2{pack2<T>(num[0] * inv, num[1] * inv), pack2<T>(num[2] * inv, num[3] * inv)};
}

}  // namespace

int flash_attention_splits(int n, int t) {
  const int qblocks = (t + QB - 1) / QB, nkb = (t + KB - 1) / KB;
  (void)n;   // independent of the batch, so that a frame's bits do not depend on what it is batched with
  int s = 256 / qblocks;   // about one workgroup per compute unit
  if (s > 8) s = 8;
  if (s > nkb) s = nkb;
  return s < 1 ? 1 : s;
}

size_t flash_attention_scratch_bytes(int n, int t, int d) {
  const int s = flash_attention_splits(n, t);
  if (s == 1) return 0;
  return (size_t)n * s * t * (d + 2) * sizeof(float);
}

int launch_flash_attention(const void* q, const void* k, size_t qk_ld, size_t qk_batch_stride, const void* vt,
                           int t_pad, void* o, void* scratch, int dtype, int n, int t, int d, float scale, hipStream_t s) {
  WMDEC_REQUIRE(d == D, WMDEC_ERR_UNSUPPORTED, "attention: head dimension %d is not supported (only %d)", d, D);
  WMDEC_REQUIRE(is_16bit(dtype), WMDEC_ERR_UNSUPPORTED, "attention: dtype must be BF16 or F16");
  WMDEC_REQUIRE(t_pad % KB == 0 && t_pad >= t && qk_ld % 8 == 0, WMDEC_ERR_SHAPE, "attention: bad leading dimensions");
  const int splits = flash_attention_splits(n, t);
  WMDEC_REQUIRE(splits == 1 || scratch, WMDEC_ERR_WORKSPACE, "attention: scratch for %d key splits missing", splits);
  float* opart = (float*)scratch;
  float* ml = opart ? opart + (size_t)n * splits * t * D : nullptr;
  const size_t smem = kSmemBytes;
  dim3 grid((unsigned)((t + QB - 1) / QB), (unsigned)splits, (unsigned)n);
  const float sl = scale * 1.4426950408889634f;
  static bool attr_set = false;
  if (!attr_set) {
    WMDEC_HIP(hipFuncSetAttribute((const void*)flash_attn_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    WMDEC_HIP(hipFuncSetAttribute((const void*)flash_attn_kernel<f16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_set = true;
  }
  if (dtype == WMDEC_BF16) {
    hipLaunchKernelGGL(flash_attn_kernel<bf16_t>, grid, dim3(NT), smem, s, (const bf16_t*)q, (const bf16_t*)k, qk_ld,
                       qk_batch_stride, (const bf16_t*)vt, t_pad, (bf16_t*)o, opart, ml, t, splits, sl);
    WMDEC_HIP(hipGetLastError());
    if (splits > 1) hipLaunchKernelGGL(attn_combine_kernel<bf16_t>, dim3((unsigned)t, (unsigned)n), dim3(128), 0, s, opart, ml, (bf16_t*)o, t, splits);
  } else {
    hipLaunchKernelGGL(flash_attn_kernel<f16_t>, grid, dim3(NT), smem, s, (const f16_t*)q, (const f16_t*)k, qk_ld,
                       qk_batch_stride, (const f16_t*)vt, t_pad, (f16_t*)o, opart, ml, t, splits, sl);
    WMDEC_HIP(hipGetLastError());
    if (splits > 1) hipLaunchKernelGGL(attn_combine_kernel<f16_t>, dim3((unsigned)t, (unsigned)n), dim3(128), 0, s, opart, ml, (f16_t*)o, t, splits);
  }
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

}  // namespace wmdec
