// Single-head attention core, flash style, for head dimension 512: keys are streamed in blocks of 32 through
// LDS, the scores live only in registers and (as 16-bit probabilities) in a 5 KiB LDS tile, and a running
// maximum / running sum rescale the output accumulator.
//
// A workgroup of 8 wavefronts owns 64 queries.  With d = 512 a wavefront cannot hold both a query fragment and
// an output accumulator for all of d, so the two products belong to different wavefronts, which run them
// concurrently, one key block apart (each SIMD hosts one wavefront of each kind):
//   scores   wavefronts 0..3: S^T[key][query] = K * Q^T for 16 queries each and all 32 keys of block j + 1, the
//            whole contraction over d (A = K rows from LDS, B = the wavefront's Q rows, held in registers for the
//            whole kernel).  One lane owns one query column, so the softmax statistics are per lane plus a
//            reduction over the 4 lanes that share a query; the probabilities go to LDS as P[query][key] with the
//            block's rescale factor per query.
//   output   wavefronts 4..7: O^T[d][query] += V^T * P^T of block j, each a 128-wide slice of d for all 64 queries
//            (A = V^T rows, B = P rows, both from LDS, 32x32x16 MFMAs); again a lane owns a query column, so the
//            rescale factor and the final 1/sum are one value per lane and query tile.
// K, V^T, P and the rescale factors are double-buffered in LDS (157 KiB), and one barrier per key block separates
// the iterations.  The tiles travel from global memory straight into LDS (global_load_lds, 16 bytes per lane: the
// 64 lanes of a wavefront fill 1 KiB of consecutive LDS from one base address): K two blocks ahead, V^T one.  Staged
// through registers, the 64 KiB per key block cost the issuing wavefronts 16 cycles per LDS store (a SIMD moves
// 64 B per cycle to the LDS: 550 to 1000 cycles per block, measured, as much as the block's MFMAs), besides the
// registers.  A K row is 1 KiB in memory and goes to an LDS row of K_LD elements; V^T is kept in memory in the very
// layout of its LDS tile (blocks of 32 keys, rows padded to V_LD elements, keys past the end zero), so that a tile
// is one run of 40 KiB.  The output wavefronts issue the loads behind their first MFMAs and wait for them before
// the barrier; the score wavefronts, whose MFMA loop and softmax are the longer chain, issue none.
// To fill 256 compute units with only T/64 query blocks the keys are split into `splits` ranges handled by
// different workgroups, each writing an unnormalised partial output with its (max, sum); attn_combine merges
// them in a fixed order.
#include <mutex>

#include "mfma.hpp"

namespace wmdec {
namespace {

constexpr int D = 512;            // head dimension
constexpr int KB = 32;            // keys per block
constexpr int QW = 16;            // queries per score wavefront
constexpr int SW = 4;             // score wavefronts
constexpr int OW = 4;             // output wavefronts
constexpr int WAVES = SW + OW;
constexpr int NT = WAVES * 64;    // threads per workgroup
constexpr int QB = QW * SW;       // queries per workgroup
constexpr int DS = D / OW;        // slice of d per output wavefront
constexpr int K_LD = D + 16;      // LDS row stride of the K tile (elements).  +32 B: the stride at which the score reads (a
                                  // wavefront reads 16 rows x 4 column groups of 16 B) run at the full LDS rate; with
                                  // +16 B they take 60 % more cycles (measured)
constexpr int V_LD = KB + 8;      // LDS row stride of the V^T tile
constexpr int P_LD = KB + 8;      // LDS row stride of the probability tile
constexpr int K_LOADS = KB / WAVES;                    // 1 KiB loads per wavefront and tile: its rows of K ...
constexpr int V_LOADS = D * V_LD * 2 / 1024 / WAVES;   // ... and its share of the 40 KiB of V^T
constexpr int T_LOADS = K_LOADS + V_LOADS;
static_assert(KB % WAVES == 0 && (D * V_LD * 2) % (1024 * WAVES) == 0, "the tiles divide among the wavefronts");
constexpr float kSlack = 8.0f;    // log2 of how far a block's maximum may exceed the running reference before it moves
constexpr size_t kSmemBytes = (size_t)2 * (KB * K_LD + D * V_LD + QB * P_LD) * 2 + 3 * QB * sizeof(float);

// max over lanes l and l ^ W (W = 16 or 32) with the row-swap instructions of this chip: no trip through LDS, which
// the score wavefronts keep busy (a bpermute there costs a few hundred cycles on the softmax's dependent chain)
template <int W> __device__ __forceinline__ float xor_max(float v) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  u32x2 r;
  if constexpr (W == 16) r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  else r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // (the results are made opaque: this compiler otherwise takes both for the first one and drops the maximum)
  unsigned a = r.x, b = r.y;
  asm volatile("" : "+v"(a), "+v"(b));
  return fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
}

template <typename T>
__global__ __launch_bounds__(NT) void flash_attn_kernel(const T* __restrict__ q, const T* __restrict__ k, size_t ld,
                                                        size_t batch_stride, const T* __restrict__ vt, int t_pad,
                                                        T* __restrict__ o, float* __restrict__ opart,
                                                        float* __restrict__ ml, int t, int splits, float scale_log2e) {
  extern __shared__ __align__(16) unsigned char smem[];
  T* s_k = reinterpret_cast<T*>(smem);                 // [2][KB][K_LD]
  T* s_v = s_k + 2 * KB * K_LD;                        // [2][D][V_LD]
  T* s_p = s_v + 2 * D * V_LD;                         // [2][QB][P_LD]
  float* s_alpha = reinterpret_cast<float*>(s_p + 2 * QB * P_LD);   // [2][QB] rescale factor of a block
  float* s_l = s_alpha + 2 * QB;                       // [QB] final sums

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = blockIdx.z, split = blockIdx.y;
  const int qb0 = blockIdx.x * QB;
  q += (size_t)n * batch_stride; k += (size_t)n * batch_stride;
  vt += (size_t)n * (t_pad / KB) * D * V_LD;
  // key blocks of this split
  const int nkb = (t + KB - 1) / KB;
  const int kb_begin = (int)((long)split * nkb / splits) * KB, kb_end = (int)((long)(split + 1) * nkb / splits) * KB;
  const int nb = (kb_end - kb_begin) / KB;
  auto block_key = [&](int j) { return kb_begin + min(j, nb - 1) * KB; };   // past the last block: a harmless reload of the last

  // tile loads of this wavefront: load i < K_LOADS is row wave * K_LOADS + i of the K tile, the others are
  // consecutive 1 KiB pieces of the V^T tile; each lane names its 16 bytes, the LDS base is wave-uniform
  typedef const __attribute__((address_space(1))) void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  auto load_k_row = [&](int i, int kb, T* dst) {
    const int r = wave * K_LOADS + i;
    __builtin_amdgcn_global_load_lds((gptr_t)(k + (size_t)min(kb + r, t - 1) * ld + lane * 8),   // rows past t are masked later
                                     (lptr_t)(dst + r * K_LD), 16, 0, 0);
  };
  auto load_v_piece = [&](int i, int kb, T* dst) {
    const int piece = wave * V_LOADS + i;
    __builtin_amdgcn_global_load_lds((gptr_t)(vt + (size_t)(min(kb, t_pad - KB) / KB) * (D * V_LD) + piece * 512 + lane * 8),
                                     (lptr_t)(dst + piece * 512), 16, 0, 0);
  };
  // tile request i of iteration j: K of block j + 2 into the buffer block j used (the score wavefronts are on block
  // j + 1), V^T of block j + 1 into the buffer the output wavefronts do not read in this iteration
  auto tile_request = [&](int i, int j) {
    if (i < K_LOADS) load_k_row(i, block_key(j + 2), s_k + (j & 1) * KB * K_LD);
    else if (i < T_LOADS) load_v_piece(i - K_LOADS, block_key(j + 1), s_v + ((j + 1) & 1) * D * V_LD);
  };
  // every load this wavefront issued has landed in LDS
  auto wait_tiles = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0);   // vmcnt(0) expcnt(0) lgkmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
  };

  // prologue: K of blocks 0 and 1, V^T of block 0
  if (nb > 0) {
#pragma unroll
    for (int i = 0; i < K_LOADS; ++i) { load_k_row(i, block_key(0), s_k); load_k_row(i, block_key(1), s_k + KB * K_LD); }
#pragma unroll
    for (int i = 0; i < V_LOADS; ++i) load_v_piece(i, block_key(0), s_v);
    wait_tiles();
  }
  __syncthreads();

  if (wave < SW) {
    // ------------------------------------------------------------------ score wavefronts
    const int lq = lane & 15, lg = lane >> 4;            // query column, lane group
    // Q fragment: B[k = d][n = query] = Q[qb0 + 16*wave + lq][32*step + 8*lg + j]
    u32x4 qf[D / 32];
    {
      const int qr = min(qb0 + wave * QW + lq, t - 1);
      const u32x4* src = reinterpret_cast<const u32x4*>(q + (size_t)qr * ld);
#pragma unroll
      for (int st = 0; st < D / 32; ++st) qf[st] = src[st * 4 + lg];
      // keep the fragment in registers: left alone, the compiler re-reads it from memory in every key block
#pragma unroll
      for (int st = 0; st < D / 32; ++st) asm volatile("" : "+v"(qf[st]));
    }
    float m_run = -INFINITY, l_run = 0.f;
    // scores and probabilities of key block j (tile in K buffer j & 1) -> P buffer j & 1; with LOADS the tile requests
    // of iteration j - 1 ride behind the MFMA pairs, one per contraction step from the second on: the memory pipeline
    // takes a 16-byte-per-lane load every 16 cycles and holds up a wavefront that issues into a full queue, so the
    // requests are spread over all eight wavefronts and over their loops
    auto score = [&](int j, auto loads_c) {
      constexpr bool LOADS = decltype(loads_c)::value;
      const int kb = kb_begin + j * KB;
      const T* sk = s_k + (j & 1) * KB * K_LD;
      // S^T tiles: keys kb + 16*tile + 4*lg + r, query qb0 + 16*wave + lq
      // K fragments are read from LDS PF contraction steps ahead of the MFMAs that consume them; the scheduling
      // barriers keep that distance (left alone, the compiler sinks each read to its use and every step pays
      // the LDS latency)
      f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
      constexpr int PF = 4;
      u32x4 ka[PF][2];
      const T* krow0 = sk + lq * K_LD + lg * 8;
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
        if constexpr (LOADS) {
          if (st >= 1 && st - 1 < T_LOADS) tile_request(st - 1, j - 1);
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
      bm = xor_max<16>(bm);   // over the four lane groups that share a query: lanes lq, lq + 16, lq + 32, lq + 48
      bm = xor_max<32>(bm);
      // The reference maximum only moves when the block's maximum exceeds it by more than 2^kSlack: until then the
      // probabilities are taken against the old reference (they may reach 2^kSlack, well inside both 16-bit types)
      // and the output accumulator needs no rescaling, which for the output wavefronts is as much vector work as
      // the block's MFMAs.  Sums and outputs share the reference, so the normalised result is the same.
      const float m_new = bm > m_run + kSlack ? bm : m_run;   // finite after the first block: it holds a valid key
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      float pr[8], ps = 0.f;
#pragma unroll
      for (int r = 0; r < 8; ++r) { pr[r] = __builtin_amdgcn_exp2f(sv[r] - m_new); ps += pr[r]; }
      l_run = l_run * alpha + ps;
      m_run = m_new;
      T* prow = s_p + (j & 1) * QB * P_LD + (wave * QW + lq) * P_LD;
      *reinterpret_cast<u32x2*>(prow + 4 * lg) = u32x2{pack2<T>(pr[0], pr[1]), pack2<T>(pr[2], pr[3])};
      *reinterpret_cast<u32x2*>(prow + 16 + 4 * lg) = u32x2{pack2<T>(pr[4], pr[5]), pack2<T>(pr[6], pr[7])};
      if (lg == 0) s_alpha[(j & 1) * QB + wave * QW + lq] = alpha;
    };
    if (nb > 0) score(0, std::false_type{});
    __syncthreads();
    for (int j = 0; j < nb; ++j) {
      // iteration j: scores of block j + 1 while the output wavefronts take block j
      if (j + 1 < nb) score(j + 1, std::true_type{});
      wait_tiles();
      __syncthreads();
    }
    // final sums per query (and, for split keys, the running maxima)
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
    __syncthreads();
  } else {
    // ------------------------------------------------------------------ output wavefronts
    const int ow = wave - SW;
    const int l32 = lane & 31, lh = lane >> 5;           // query column within a tile, contraction half
    f32x16 acc[DS / 32][2];   // [d tile][query tile] of O^T
#pragma unroll
    for (int i = 0; i < DS / 32; ++i)
#pragma unroll
      for (int jq = 0; jq < 2; ++jq)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][jq][r] = 0.f;
    __syncthreads();
    for (int j = 0; j < nb; ++j) {
      const T* sp = s_p + (j & 1) * QB * P_LD;
      const T* sv = s_v + (j & 1) * D * V_LD;
      // everything this iteration reads from LDS is requested up front (one latency instead of one per contraction
      // half: the LDS is the busiest unit of this kernel and answers slowly)
      const float al0 = s_alpha[(j & 1) * QB + l32], al1 = s_alpha[(j & 1) * QB + 32 + l32];
      u32x4 pf[KB / 16][2], vf[KB / 16][DS / 32];
#pragma unroll
      for (int ks = 0; ks < KB / 16; ++ks) {
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) pf[ks][qt] = *reinterpret_cast<const u32x4*>(sp + (qt * 32 + l32) * P_LD + ks * 16 + lh * 8);
#pragma unroll
        for (int dt = 0; dt < DS / 32; ++dt) vf[ks][dt] = *reinterpret_cast<const u32x4*>(sv + (ow * DS + dt * 32 + l32) * V_LD + ks * 16 + lh * 8);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (__any(al0 != 1.0f || al1 != 1.0f)) {
#pragma unroll
        for (int dt = 0; dt < DS / 32; ++dt) { acc[dt][0] *= al0; acc[dt][1] *= al1; }
      }
#pragma unroll
      for (int ks = 0; ks < KB / 16; ++ks) {
#pragma unroll
        for (int dt = 0; dt < DS / 32; ++dt) {
#pragma unroll
          for (int qt = 0; qt < 2; ++qt) acc[dt][qt] = Mma<T>::m32(vf[ks][dt], pf[ks][qt], acc[dt][qt]);
          // this wavefront's tile requests, one (the last slot: two) behind each MFMA pair
          const int li = ks * (DS / 32) + dt;
          tile_request(li, j);
          if (li == KB / 16 * (DS / 32) - 1) tile_request(li + 1, j);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      wait_tiles();
      __syncthreads();
    }
    __syncthreads();
    // O^T tile element r of lane: d = ow*DS + dt*32 + 8*(r/4) + 4*lh + r%4, query = qb0 + qt*32 + l32
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      const int qr = qb0 + qt * 32 + l32;
      if (qr >= t) continue;
      if (splits == 1) {
        const float inv = 1.0f / s_l[qt * 32 + l32];
        T* orow = o + ((size_t)n * t + qr) * D + ow * DS + 4 * lh;
#pragma unroll
        for (int dt = 0; dt < DS / 32; ++dt)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x16& c = acc[dt][qt];
            *reinterpret_cast<u32x2*>(orow + dt * 32 + g * 8) =
                u32x2{pack2<T>(c[4 * g] * inv, c[4 * g + 1] * inv), pack2<T>(c[4 * g + 2] * inv, c[4 * g + 3] * inv)};
          }
      } else {
        float* prow = opart + (((size_t)n * splits + split) * t + qr) * D + ow * DS + 4 * lh;
#pragma unroll
        for (int dt = 0; dt < DS / 32; ++dt)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x16& c = acc[dt][qt];
            *reinterpret_cast<f32x4*>(prow + dt * 32 + g * 8) = f32x4{c[4 * g], c[4 * g + 1], c[4 * g + 2], c[4 * g + 3]};
          }
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

size_t flash_attention_vt_elems(int t, int d) { return (size_t)((t + KB - 1) / KB) * d * V_LD; }

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
  static std::once_flag attr_once;
  hipError_t attr_err = hipSuccess;
  std::call_once(attr_once, [&] {
    attr_err = hipFuncSetAttribute((const void*)flash_attn_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (attr_err == hipSuccess)
      attr_err = hipFuncSetAttribute((const void*)flash_attn_kernel<f16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  });
  WMDEC_HIP(attr_err);
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
