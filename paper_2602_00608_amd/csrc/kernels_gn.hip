// GroupNorm statistics: a streaming read of an NHWC tensor producing, per
// (sample, group), the mean and 1/sqrt(biased variance + eps).
//
// Stage 1 (gn_partial_*): the pixels of a sample are cut into `chunks` slabs;
// one workgroup reads a slab with 16-byte vector loads (every thread keeps a
// fixed set of channels), accumulates shifted sums in fp32 (shift = the first
// value a thread sees per channel, so that E[x^2]-E[x]^2 never cancels), and
// writes one (count, mean, M2) triple per group.  Stage 2 (gn_finalize) merges
// the triples of a group with the pairwise update of Chan et al. in a fixed
// order, so the result does not depend on scheduling.
#include "moments.hpp"

namespace wmdec {
namespace {

template <typename T> struct Vec16;  // 16-byte vector of T
template <> struct alignas(16) Vec16<float> { static constexpr int N = 4; float v[4]; };
template <> struct alignas(16) Vec16<bf16_t> { static constexpr int N = 8; bf16_t v[8]; };
template <> struct alignas(16) Vec16<f16_t> { static constexpr int N = 8; f16_t v[8]; };

// Fast path: c % V == 0, VP = c / V divides 256.  grid = (chunks, n).
// ws: [n][groups][chunks] Moments.
template <typename T>
__global__ __launch_bounds__(256) void gn_partial_vec(const T* __restrict__ x, int pixels, int c, int groups,
                                                      int chunk_pixels, Moments* __restrict__ ws) {
  constexpr int V = Vec16<T>::N;
  __shared__ Moments s_m[256];
  const int tid = threadIdx.x;
  const int vp = c / V;           // vectors per pixel
  const int cv = tid % vp;        // this thread's channel vector
  const int ppi = 256 / vp;       // pixels per sweep of the workgroup
  const int chunk = blockIdx.x, n = blockIdx.y, chunks = gridDim.x;
  const int p0 = chunk * chunk_pixels;
  const int p1 = min(p0 + chunk_pixels, pixels);
  const Vec16<T>* base = reinterpret_cast<const Vec16<T>*>(x + (size_t)n * pixels * c) + cv;

  float shift[V], s[V], q[V];
  float cnt = 0.f;
  int p = p0 + tid / vp;
  if (p < p1) {
    const Vec16<T> v = base[(size_t)p * vp];
#pragma unroll
    for (int j = 0; j < V; ++j) { shift[j] = to_float(v.v[j]); s[j] = 0.f; q[j] = 0.f; }
    cnt = 1.f;
    p += ppi;
  } else {
#pragma unroll
    for (int j = 0; j < V; ++j) { shift[j] = 0.f; s[j] = 0.f; q[j] = 0.f; }
  }
  // four loads in flight per thread
  for (; p + 3 * ppi < p1; p += 4 * ppi) {
    Vec16<T> v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = base[(size_t)(p + u * ppi) * vp];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < V; ++j) { const float d = to_float(v[u].v[j]) - shift[j]; s[j] += d; q[j] = fmaf(d, d, q[j]); }
    cnt += 4.f;
  }
  for (; p < p1; p += ppi) {
    const Vec16<T> v = base[(size_t)p * vp];
#pragma unroll
    for (int j = 0; j < V; ++j) { const float d = to_float(v.v[j]) - shift[j]; s[j] += d; q[j] = fmaf(d, d, q[j]); }
    cnt += 1.f;
  }

  // per-thread moments of its V channels, merged per group.  A vector of V
  // channels covers V/cpg groups when cpg < V, else lies inside one group.
  const int cpg = c / groups;
  const int sub = (cpg < V) ? cpg : V;   // channels of one group inside this vector
  const int nsub = V / sub;              // groups touched by this vector (1, 2 or 4 ...)
  // Reduce one sub-vector at a time through LDS: all threads of the workgroup
  // that hold channels of the same group are merged in a fixed tree.
  for (int sv = 0; sv < nsub; ++sv) {
    Moments m{0.f, 0.f, 0.f};
    if (cnt > 0.f) {
#pragma unroll
      for (int j = 0; j < V; ++j) {
        if (j / sub == sv) {
          Moments e;
          e.n = cnt;
          const float ds = s[j] / cnt;
          e.mean = shift[j] + ds;
          e.m2 = fmaxf(q[j] - s[j] * ds, 0.f);
          m = merge(m, e);
        }
      }
    }
    __syncthreads();
    s_m[tid] = m;
    __syncthreads();
    // group of this thread's sub-vector: g = (cv*V + sv*sub) / cpg.  Threads with equal g:
    // vectors_per_group = max(cpg / V, 1) consecutive cv values, times ppi pixel lanes.
    const int vpg = (cpg >= V) ? cpg / V : 1;
    const int g = (cv * V + sv * sub) / cpg;
    // one leader thread per group does a fixed-order merge of its ppi*vpg members
    if (tid / vp == 0 && (cv % vpg) == 0) {
      Moments r{0.f, 0.f, 0.f};
      for (int pl = 0; pl < ppi; ++pl)
        for (int k = 0; k < vpg; ++k) r = merge(r, s_m[pl * vp + cv + k]);
      ws[((size_t)n * groups + g) * chunks + chunk] = r;
    }
  }
}

// General path (any c, groups): grid = (chunks, groups, n); one workgroup walks
// the (pixel, channel-in-group) pairs of its slab.
template <typename T>
__global__ __launch_bounds__(256) void gn_partial_any(const T* __restrict__ x, int pixels, int c, int groups,
                                                      int chunk_pixels, Moments* __restrict__ ws) {
  __shared__ Moments s_m[256];
  const int tid = threadIdx.x;
  const int chunk = blockIdx.x, g = blockIdx.y, n = blockIdx.z, chunks = gridDim.x;
  const int cpg = c / groups;
  const int p0 = chunk * chunk_pixels, p1 = min(p0 + chunk_pixels, pixels);
  const long total = (long)(p1 - p0) * cpg;
  const T* base = x + ((size_t)n * pixels + p0) * c + (size_t)g * cpg;
  float shift = 0.f, s = 0.f, q = 0.f, cnt = 0.f;
  for (long i = tid; i < total; i += 256) {
    const float v = to_float(base[(size_t)(i / cpg) * c + (i % cpg)]);
    if (cnt == 0.f) shift = v;
    const float d = v - shift;
    s += d; q = fmaf(d, d, q); cnt += 1.f;
  }
  Moments m{0.f, 0.f, 0.f};
  if (cnt > 0.f) { m.n = cnt; const float ds = s / cnt; m.mean = shift + ds; m.m2 = fmaxf(q - s * ds, 0.f); }
  s_m[tid] = m;
  __syncthreads();
  for (int step = 128; step > 0; step >>= 1) {
    if (tid < step) s_m[tid] = merge(s_m[tid], s_m[tid + step]);
    __syncthreads();
  }
  if (tid == 0) ws[((size_t)n * groups + g) * chunks + chunk] = s_m[0];
}

// grid = n*groups workgroups of 256 threads: thread t merges slots t, t+256, ... in order, then a fixed
// butterfly over each wavefront, then wavefronts 0..3 in order.
__global__ __launch_bounds__(256) void gn_finalize(const Moments* __restrict__ ws, int chunks, float eps,
                                                   float* __restrict__ mean, float* __restrict__ rstd) {
  __shared__ Moments s_w[4];
  const int ng = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  Moments m{0.f, 0.f, 0.f};
  for (int i = tid; i < chunks; i += 256) m = merge(m, ws[(size_t)ng * chunks + i]);
  for (int mask = 1; mask < 64; mask <<= 1) m = butterfly(m, lane, mask);   // lane-independent order
  if (lane == 0) s_w[tid >> 6] = m;
  __syncthreads();
  if (tid == 0) {
    m = merge(merge(s_w[0], s_w[1]), merge(s_w[2], s_w[3]));
    mean[ng] = m.mean;
    rstd[ng] = 1.0f / sqrtf(m.m2 / m.n + eps);
  }
}

int pick_chunks(int pixels, int c, int V, bool vec) {
  // aim at <= 2048 workgroups per sample, each sweeping its slab at least 8 times
  const int ppi = vec ? 256 / (c / V) : 1;
  const int min_chunk = vec ? 8 * ppi : 1024;
  int chunks = (pixels + min_chunk - 1) / min_chunk;
  if (chunks > 2048) chunks = 2048;
  if (chunks < 1) chunks = 1;
  return chunks;
}

struct Plan { bool vec; int chunks; int chunk_pixels; };

Plan make_plan(int x_dtype, int n, int h, int w, int c, int groups) {
  const int V = x_dtype == WMDEC_F32 ? 4 : 8;
  const int pixels = h * w;
  const int cpg = c / groups;
  Plan p;
  const bool divisible = (c % V == 0) && (256 % (c / V) == 0) && (c / V <= 256);
  // a vector must not straddle a group boundary unevenly: cpg | V or V | cpg
  p.vec = divisible && ((cpg % V == 0) || (V % cpg == 0));
  p.chunks = pick_chunks(pixels, c, V, p.vec);
  p.chunk_pixels = (pixels + p.chunks - 1) / p.chunks;
  if (p.vec) {
    const int ppi = 256 / (c / V);
    p.chunk_pixels = ((p.chunk_pixels + ppi - 1) / ppi) * ppi;
  }
  p.chunks = (pixels + p.chunk_pixels - 1) / p.chunk_pixels;
  return p;
}

}  // namespace

int launch_gn_finalize(const void* ws, int n_groups, int slots, float eps, float* mean, float* rstd, hipStream_t s) {
  hipLaunchKernelGGL(gn_finalize, dim3((unsigned)n_groups), dim3(256), 0, s, (const Moments*)ws, slots, eps, mean, rstd);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

size_t gn_stats_workspace_bytes(int n, int h, int w, int c, int groups) {
  // upper bound over dtypes: 2048 chunks per (sample, group)
  (void)h; (void)w; (void)c;
  return (size_t)n * groups * 2048 * sizeof(Moments);
}

int launch_gn_stats(const void* x, int x_dtype, int n, int h, int w, int c, int groups, float eps,
                    float* mean, float* rstd, void* ws, size_t ws_bytes, hipStream_t s) {
  const Plan p = make_plan(x_dtype, n, h, w, c, groups);
  WMDEC_REQUIRE(ws && ws_bytes >= (size_t)n * groups * p.chunks * sizeof(Moments), WMDEC_ERR_WORKSPACE,
                "gn_stats: workspace of %zu bytes is too small", ws_bytes);
  Moments* wsm = (Moments*)ws;
  const int pixels = h * w;
  if (p.vec) {
    dim3 grid((unsigned)p.chunks, (unsigned)n);
    switch (x_dtype) {
      case WMDEC_F32: hipLaunchKernelGGL(gn_partial_vec<float>, grid, dim3(256), 0, s, (const float*)x, pixels, c, groups, p.chunk_pixels, wsm); break;
      case WMDEC_BF16: hipLaunchKernelGGL(gn_partial_vec<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)x, pixels, c, groups, p.chunk_pixels, wsm); break;
      default: hipLaunchKernelGGL(gn_partial_vec<f16_t>, grid, dim3(256), 0, s, (const f16_t*)x, pixels, c, groups, p.chunk_pixels, wsm); break;
    }
  } else {
    dim3 grid((unsigned)p.chunks, (unsigned)groups, (unsigned)n);
    switch (x_dtype) {
      case WMDEC_F32: hipLaunchKernelGGL(gn_partial_any<float>, grid, dim3(256), 0, s, (const float*)x, pixels, c, groups, p.chunk_pixels, wsm); break;
      case WMDEC_BF16: hipLaunchKernelGGL(gn_partial_any<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)x, pixels, c, groups, p.chunk_pixels, wsm); break;
      default: hipLaunchKernelGGL(gn_partial_any<f16_t>, grid, dim3(256), 0, s, (const f16_t*)x, pixels, c, groups, p.chunk_pixels, wsm); break;
    }
  }
  WMDEC_HIP(hipGetLastError());
  hipLaunchKernelGGL(gn_finalize, dim3((unsigned)(n * groups)), dim3(256), 0, s, wsm, p.chunks, eps, mean, rstd);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

}  // namespace wmdec
