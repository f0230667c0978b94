// GroupNorm statistics: a streaming read of an NHWC tensor producing, per
// (sample, group), the mean and 1/sqrt(biased variance + eps).
//
// The pixels of a sample are cut into slabs; a workgroup reads its slab with
// 16-byte vector loads (every thread keeps a fixed set of channels), accumulates
// shifted sums in fp32 (so that E[d^2]-E[d]^2 never cancels) and produces one
// (count, mean, M2) triple per group.  Triples are merged with the pairwise
// update of Chan et al. in a fixed order, so the result does not depend on
// scheduling.  Channel counts that fit the vector layout take the single-launch
// kernel gn_stats_vec, whose last workgroup per sample does the merge; everything
// else takes gn_partial_any followed by gn_finalize, which also merges the
// moments a convolution emitted from its epilogue.
//
// Hardware assumption of the single-launch kernel (gfx950 only, checked below): its cross-workgroup hand-over uses
// no release / acquire fence, because an agent-scope fence on this chip writes back or invalidates the whole L2
// of the XCD (microseconds per wavefront).  Instead every shared word is itself accessed with agent-scope atomic
// stores and loads, which gfx950 executes as write-through stores / L2-bypassing loads of memory that is coherent
// across the XCDs; the publishing wavefront waits until the memory system has acknowledged its stores (vmcnt = 0)
// before it takes the ticket, and only the workgroup that draws the last ticket reads.  Under the language memory
// model the relaxed accesses alone would not order the stores before the ticket; the wait does, on this hardware.
#include <mutex>

#include "moments.hpp"

#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "kernels_gn.hip relies on gfx950 memory behaviour (see the note on the single-launch kernel)"
#endif

namespace wmdec {
namespace {

struct alignas(16) f32x4s { float x, y, z, w; };

template <typename T> struct Vec16;  // 16-byte vector of T
template <> struct alignas(16) Vec16<float> { static constexpr int N = 4; float v[4]; };
template <> struct alignas(16) Vec16<bf16_t> { static constexpr int N = 8; bf16_t v[8]; };
template <> struct alignas(16) Vec16<f16_t> { static constexpr int N = 8; f16_t v[8]; };

// Fast path: c % V == 0, vp = c / V divides 1024, channels per group a power of two <= 64.
// grid = (chunks, n), 1024 threads.  ws: [n][groups][chunks] Moments.  One launch does everything: a workgroup
// streams its slab (8 loads of 16 bytes in flight per thread, the ragged end as one masked batch), sums
// x - shift and its square per thread (shift = the slab's first pixel, shared by all threads of a channel),
// adds the threads of a channel in a fixed order through LDS, the channels of a group with a butterfly, and
// writes one triple per group.  The workgroup of a sample that finishes last (one wrapping ticket counter per
// sample, which returns to zero by itself) merges the sample's triples in a fixed order into mean / rstd.
constexpr int kVecThreads = 1024;
constexpr int kVecMaxChunks = 256;
constexpr int kVecMaxGroups = 256;

template <typename T, int V, bool MASKED>
__device__ __forceinline__ void gn_accumulate(const Vec16<T>* base, int p, int p1, int ppi, int vp, const float* shift,
                                              float* s, float* q) {
  constexpr int U = 8;
  Vec16<T> v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int pp = p + u * ppi;
    v[u] = base[(size_t)((MASKED && pp >= p1) ? p : pp) * vp];   // always a pixel of this slab: no branch around the load
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const bool live = !MASKED || p + u * ppi < p1;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const float d = live ? to_float(v[u].v[j]) - shift[j] : 0.f;
      s[j] += d;
      q[j] = fmaf(d, d, q[j]);
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kVecThreads) void gn_stats_vec(const T* __restrict__ x, int pixels, int c, int groups,
                                                            int chunk_pixels, Moments* ws, unsigned* ticket, float eps,
                                                            float* __restrict__ mean, float* __restrict__ rstd) {
  constexpr int V = Vec16<T>::N;
  constexpr int U = 8;
  __shared__ float2 s_e[kVecThreads * V];   // (sum, sum of squares) per (pixel lane, channel)
  __shared__ Moments s_g[kVecMaxGroups];    // the slab's moments per group
  __shared__ unsigned s_last;
  const int tid = threadIdx.x;
  const int vp = c / V;           // vectors per pixel
  const int cv = tid % vp;        // this thread's channel vector
  const int ppi = kVecThreads / vp;   // pixels per sweep of the workgroup
  const int chunk = blockIdx.x, n = blockIdx.y, chunks = gridDim.x;
  const int p0 = chunk * chunk_pixels;
  const int p1 = min(p0 + chunk_pixels, pixels);
  const Vec16<T>* base = reinterpret_cast<const Vec16<T>*>(x + (size_t)n * pixels * c) + cv;

  float shift[V], s[V], q[V];
  {
    const Vec16<T> v = base[(size_t)p0 * vp];
#pragma unroll
    for (int j = 0; j < V; ++j) { shift[j] = to_float(v.v[j]); s[j] = 0.f; q[j] = 0.f; }
  }
  int p = p0 + tid / vp;
  for (; p + (U - 1) * ppi < p1; p += U * ppi) gn_accumulate<T, V, false>(base, p, p1, ppi, vp, shift, s, q);
  if (p < p1) gn_accumulate<T, V, true>(base, p, p1, ppi, vp, shift, s, q);

#pragma unroll
  for (int j = 0; j < V; ++j) s_e[(tid / vp) * c + cv * V + j] = float2{s[j], q[j]};
  __syncthreads();
  const int cpg = c / groups;
  const float cnt = (float)(p1 - p0);
  for (int ch = tid; ch < c; ch += kVecThreads) {
    float s0 = 0.f, q0 = 0.f;
#pragma unroll 8
    for (int r = 0; r < ppi; ++r) { const float2 e = s_e[r * c + ch]; s0 += e.x; q0 += e.y; }
    // every thread of a channel used the same shift: the slab's first pixel
    const float a0 = to_float(x[((size_t)n * pixels + p0) * c + ch]);
    const float ds = s0 / cnt;
    Moments m{cnt, a0 + ds, fmaxf(q0 - s0 * ds, 0.f)};
    for (int mask = 1; mask < cpg; mask <<= 1) m = butterfly(m, tid, mask);   // cpg consecutive lanes = one group
    if ((ch & (cpg - 1)) == 0) s_g[ch / cpg] = m;
  }
  __syncthreads();

  // One wavefront publishes the slab's triples and takes the sample's ticket.  No fences (a fence walks the whole
  // L2 and costs microseconds per workgroup): the triples are written with device-scope stores, which go through
  // to memory, the wavefront waits for them to complete before it takes the ticket, and the sample's last
  // workgroup reads all triples with device-scope loads, which do not hit stale lines of its own L2.
  if (tid < 64) {
    for (int g = tid; g < groups; g += 64) store_device(ws + ((size_t)n * groups + g) * chunks + chunk, s_g[g]);
    wait_stores();
    if (tid == 0) s_last = atomicInc(ticket + n, chunks - 1) == (unsigned)(chunks - 1);
  }
  __syncthreads();
  if (!s_last) return;
  // half a wavefront per group, 8 slots per lane, merged in a fixed order
  const int sub = tid & 31, half = tid >> 5;
  for (int g = half; g < groups; g += kVecThreads / 32) {
    const Moments* row = ws + ((size_t)n * groups + g) * chunks;
    Moments t[kVecMaxChunks / 32];
#pragma unroll
    for (int k = 0; k < kVecMaxChunks / 32; ++k) {
      const int i = sub + 32 * k;
      t[k] = load_device(row + min(i, chunks - 1));
      if (i >= chunks) t[k].n = 0.f;
    }
    Moments m = t[0];
#pragma unroll
    for (int k = 1; k < kVecMaxChunks / 32; ++k) m = merge(m, t[k]);
    for (int mask = 1; mask < 32; mask <<= 1) m = butterfly(m, sub, mask);
    if (sub == 0) {
      mean[n * groups + g] = m.mean;
      rstd[n * groups + g] = 1.0f / sqrtf(m.m2 / m.n + eps);
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

// grid = n*groups workgroups of 1024 threads: thread t merges slots t, t+1024, ... in order (loaded four at a
// time: a row of up to 4096 slots costs one memory round trip), then a fixed merge tree over each wavefront, then
// over the 16 wavefronts.
constexpr int kFinThreads = 1024;
__global__ __launch_bounds__(kFinThreads) void gn_finalize(const Moments* __restrict__ ws, int chunks, float eps,
                                                           float* __restrict__ mean, float* __restrict__ rstd) {
  __shared__ Moments s_w[kFinThreads / 64];
  const int ng = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const Moments* row = ws + (size_t)ng * chunks;
  Moments m{0.f, 0.f, 0.f};
  for (int i0 = tid; i0 < chunks; i0 += kFinThreads * 4) {
    Moments t[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + kFinThreads * k;
      t[k] = row[min(i, chunks - 1)];
      if (i >= chunks) t[k].n = 0.f;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) m = merge(m, t[k]);
  }
  m = merge_to_first(m, lane, 64);   // fixed order
  if (lane == 0) s_w[tid >> 6] = m;
  __syncthreads();
  if (tid < 64) {   // the 16 wavefront results: four merge levels inside one row of lanes instead of a chain of 15
    static_assert(kFinThreads / 64 == 16, "one row of 16 lanes");
    m = tid < kFinThreads / 64 ? s_w[tid] : Moments{0.f, 0.f, 0.f};
    m = merge_to_first(m, lane, 16);
    if (tid == 0) {
      mean[ng] = m.mean;
      rstd[ng] = 1.0f / sqrtf(m.m2 / m.n + eps);
    }
  }
}

int pick_chunks(int pixels, int c, int V, bool vec) {
  // vector path: <= 256 workgroups of 1024 threads per sample (one per compute unit, 128 KiB of loads in flight),
  // every one sweeping its slab at least 4 times; general path: <= 2048 slabs of >= 1024 pixels.
  // Never a function of the batch size: a sample's result must not depend on its neighbours.
  const int ppi = vec ? kVecThreads / (c / V) : 1;
  const int min_chunk = vec ? 4 * ppi : 1024;
  int chunks = (pixels + min_chunk - 1) / min_chunk;
  const int cap = vec ? kVecMaxChunks : 2048;
  if (chunks > cap) chunks = cap;
  if (chunks < 1) chunks = 1;
  return chunks;
}

struct Plan { bool vec; int chunks; int chunk_pixels; };

Plan make_plan(int x_dtype, int n, int h, int w, int c, int groups) {
  (void)n;
  const int V = x_dtype == WMDEC_F32 ? 4 : 8;
  const int pixels = h * w;
  const int cpg = c / groups;
  Plan p;
  const bool divisible = (c % V == 0) && (kVecThreads % (c / V) == 0) && c <= kVecThreads;
  p.vec = divisible && (cpg & (cpg - 1)) == 0 && cpg <= 64 && groups <= kVecMaxGroups;   // groups are runs of 2^k lanes in the channel reduction
  p.chunks = pick_chunks(pixels, c, V, p.vec);
  p.chunk_pixels = (pixels + p.chunks - 1) / p.chunks;
  if (p.vec) {
    const int ppi = kVecThreads / (c / V);
    p.chunk_pixels = ((p.chunk_pixels + ppi - 1) / ppi) * ppi;
  }
  p.chunks = (pixels + p.chunk_pixels - 1) / p.chunk_pixels;
  return p;
}

}  // namespace

int launch_gn_finalize(const void* ws, int n_groups, int slots, float eps, float* mean, float* rstd, hipStream_t s) {
  hipLaunchKernelGGL(gn_finalize, dim3((unsigned)n_groups), dim3(kFinThreads), 0, s, (const Moments*)ws, slots, eps, mean, rstd);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

// one ticket counter per sample for the single-launch path
size_t gn_stats_ticket_bytes(int n) { return ((size_t)n * sizeof(unsigned) + 255) / 256 * 256; }

size_t gn_stats_moments_bytes(int n, int groups) {
  // upper bound over shapes and dtypes: 2048 chunks per (sample, group)
  return (size_t)n * groups * 2048 * sizeof(Moments);
}

int gn_stats_num_launches(int x_dtype, int h, int w, int c, int groups) {
  return make_plan(x_dtype, 1, h, w, c, groups).vec ? 1 : 2;
}

int launch_gn_stats(const void* x, int x_dtype, int n, int h, int w, int c, int groups, float eps,
                    float* mean, float* rstd, unsigned* ticket, void* moments, size_t moments_bytes, hipStream_t s) {
  const Plan p = make_plan(x_dtype, n, h, w, c, groups);
  WMDEC_REQUIRE(ticket && moments && moments_bytes >= (size_t)n * groups * p.chunks * sizeof(Moments), WMDEC_ERR_WORKSPACE,
                "gn_stats: workspace of %zu bytes is too small", moments_bytes);
  Moments* wsm = (Moments*)moments;
  const int pixels = h * w;
  if (p.vec) {
    dim3 grid((unsigned)p.chunks, (unsigned)n);
    switch (x_dtype) {
      case WMDEC_F32: hipLaunchKernelGGL(gn_stats_vec<float>, grid, dim3(kVecThreads), 0, s, (const float*)x, pixels, c, groups, p.chunk_pixels, wsm, ticket, eps, mean, rstd); break;
      case WMDEC_BF16: hipLaunchKernelGGL(gn_stats_vec<bf16_t>, grid, dim3(kVecThreads), 0, s, (const bf16_t*)x, pixels, c, groups, p.chunk_pixels, wsm, ticket, eps, mean, rstd); break;
      default: hipLaunchKernelGGL(gn_stats_vec<f16_t>, grid, dim3(kVecThreads), 0, s, (const f16_t*)x, pixels, c, groups, p.chunk_pixels, wsm, ticket, eps, mean, rstd); break;
    }
    WMDEC_HIP(hipGetLastError());
    return WMDEC_OK;
  } else {
    dim3 grid((unsigned)p.chunks, (unsigned)groups, (unsigned)n);
    switch (x_dtype) {
      case WMDEC_F32: hipLaunchKernelGGL(gn_partial_any<float>, grid, dim3(256), 0, s, (const float*)x, pixels, c, groups, p.chunk_pixels, wsm); break;
      case WMDEC_BF16: hipLaunchKernelGGL(gn_partial_any<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)x, pixels, c, groups, p.chunk_pixels, wsm); break;
      default: hipLaunchKernelGGL(gn_partial_any<f16_t>, grid, dim3(256), 0, s, (const f16_t*)x, pixels, c, groups, p.chunk_pixels, wsm); break;
    }
  }
  WMDEC_HIP(hipGetLastError());
  hipLaunchKernelGGL(gn_finalize, dim3((unsigned)(n * groups)), dim3(kFinThreads), 0, s, wsm, p.chunks, eps, mean, rstd);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

// ---- the variant for callers that cannot allocate: the workspace is a file-scope device array
constexpr size_t kStaticTicketBytes = 256;                 // 64 ticket counters
constexpr size_t kStaticMomentsBytes = (size_t)1 << 20;    // 87381 moment triples
static __device__ __align__(256) unsigned char scratch[kStaticTicketBytes + kStaticMomentsBytes];

size_t gn_stats_static_capacity_bytes() { return kStaticMomentsBytes; }

int launch_gn_stats_static(const void* x, int x_dtype, int n, int h, int w, int c, int groups, float eps,
                           float* mean, float* rstd, hipStream_t s) {
  const Plan p = make_plan(x_dtype, n, h, w, c, groups);
  const size_t need = (size_t)n * groups * p.chunks * sizeof(Moments);
  WMDEC_REQUIRE((size_t)n * sizeof(unsigned) <= kStaticTicketBytes && need <= kStaticMomentsBytes, WMDEC_ERR_WORKSPACE,
                "gn_stats_noalloc: %d samples x %d groups x %d slabs need %zu bytes of built-in scratch, the limit is %zu "
                "(and 64 samples); use wmdec_gn_stats with a workspace", n, groups, p.chunks, need, kStaticMomentsBytes);
  // every device holds its own copy of the array at its own address: resolve it once per device, with that device current
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static unsigned char* dev_scratch[kMaxDevices] = {};
  int dev = -1;
  WMDEC_HIP(hipGetDevice(&dev));
  WMDEC_REQUIRE(dev >= 0 && dev < kMaxDevices, WMDEC_ERR_UNSUPPORTED, "gn_stats_noalloc: device index %d not supported", dev);
  unsigned char* ptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!dev_scratch[dev]) {
      void* sym = nullptr;
      WMDEC_HIP(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
      dev_scratch[dev] = (unsigned char*)sym;
    }
    ptr = dev_scratch[dev];
  }
  // the array keeps what the last call left: the counters are put back to zero by a fill kernel (not a memset
  // node: the call may be captured in a graph); the moment slots are all written before they are read
  const int rc = launch_zero_u32(ptr, (int)(kStaticTicketBytes / sizeof(unsigned)), s);
  if (rc != WMDEC_OK) return rc;
  return launch_gn_stats(x, x_dtype, n, h, w, c, groups, eps, mean, rstd, (unsigned*)ptr, ptr + kStaticTicketBytes,
                         kStaticMomentsBytes, s);
}

}  // namespace wmdec
