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

}  // namespace wmdec
