// Running moments (count, mean, sum of squared deviations) and their pairwise merge
// (Chan, Golub, LeVeque).  Shared by the GroupNorm statistics kernels and by the convolution
// epilogue that emits statistics of its own output.
#pragma once
#include "common.hpp"

namespace wmdec {

struct Moments { float n, mean, m2; };

__device__ __forceinline__ Moments merge(Moments a, Moments b) {
  if (b.n == 0.f) return a;
  if (a.n == 0.f) return b;
  const float n = a.n + b.n;
  const float d = b.mean - a.mean;
  const float fb = b.n * __builtin_amdgcn_rcpf(n);   // 1 ulp is ample for a weight
  Moments r;
  r.n = n;
  r.mean = a.mean + d * fb;
  r.m2 = a.m2 + b.m2 + d * d * a.n * fb;
  return r;
}

__device__ __forceinline__ Moments shfl_xor(Moments m, int mask) {
  Moments r;
  r.n = __shfl_xor(m.n, mask); r.mean = __shfl_xor(m.mean, mask); r.m2 = __shfl_xor(m.m2, mask);
  return r;
}

// both lanes of a pair end with the same bits: merge(lower lane, upper lane)
__device__ __forceinline__ Moments butterfly(Moments m, int lane, int mask) {
  const Moments o = shfl_xor(m, mask);
  return (lane & mask) ? merge(o, m) : merge(m, o);
}

// Lane i takes the triple of lane i + N of its row of 16 lanes (N = 1, 2, 4, 8), an empty triple if that lane lies
// outside the row: a data-parallel-primitive move in the vector ALU, where the xor shuffle above is a trip through LDS.
template <int N> __device__ __forceinline__ Moments row_down(Moments m) {
  Moments r;
  r.n = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, m.n), 0x100 + N, 0xf, 0xf, true));
  r.mean = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, m.mean), 0x100 + N, 0xf, 0xf, true));
  r.m2 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, m.m2), 0x100 + N, 0xf, 0xf, true));
  return r;
}
// Merge of the `width` consecutive lanes (a power of two up to 64) that start at a lane whose index is a multiple of
// `width`, left in that first lane, in a fixed order; the other lanes end with partial merges.
__device__ __forceinline__ Moments merge_to_first(Moments m, int lane, int width) {
  if (width > 1) m = merge(m, row_down<1>(m));
  if (width > 2) m = merge(m, row_down<2>(m));
  if (width > 4) m = merge(m, row_down<4>(m));
  if (width > 8) m = merge(m, row_down<8>(m));
  if (width > 16) m = butterfly(m, lane, 16);
  if (width > 32) m = butterfly(m, lane, 32);
  return m;
}

// Device-scope (write-through / L2-bypassing) accesses of a triple and the wait that orders a wavefront's stores before
// a ticket it takes afterwards: the hand-over between workgroups of one launch that both the single-launch statistics
// kernel and the convolution epilogue use (gfx950; see the note at the top of kernels_gn.hip).
__device__ __forceinline__ void store_device(Moments* p, Moments m) {
  __hip_atomic_store(&p->n, m.n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(&p->mean, m.mean, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(&p->m2, m.m2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ Moments load_device(const Moments* p) {
  Moments m;
  m.n = __hip_atomic_load(&p->n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  m.mean = __hip_atomic_load(&p->mean, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  m.m2 = __hip_atomic_load(&p->m2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return m;
}
__device__ __forceinline__ void wait_stores() {
  __builtin_amdgcn_sched_barrier(0);
  // s_waitcnt immediate of gfx9-family chips: vmcnt in bits 3:0 and 15:14, expcnt in 6:4, lgkmcnt in 11:8
  constexpr int kVmcnt0 = 0, kExpcntAny = 7 << 4, kLgkmcntAny = 0xF << 8;
  __builtin_amdgcn_s_waitcnt(kVmcnt0 | kExpcntAny | kLgkmcntAny);   // every store of this wavefront has been acknowledged
  __builtin_amdgcn_sched_barrier(0);
}

}  // namespace wmdec
