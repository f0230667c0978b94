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
