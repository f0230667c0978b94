// Diagnostic (not on the product path): what the gfx950 matrix pipe sustains on this machine.
//
// The published dense f16/bf16 figure (2516.6 TFLOP/s) assumes 2.4 GHz on all 256 compute units; under a
// matrix-heavy kernel the power limit lowers the clock, and by how much depends on how many operand bits
// toggle.  This program times, on every compute unit at once,
//   mode 0: a loop of nothing but 32x32x16 f16 MFMAs on register operands,
//   mode 1: the inner loop of the convolution kernel: A fragments read from LDS at tap offsets, B fragments
//           (1 KiB each) loaded from an L2-resident weight blob three k-steps ahead, one barrier per 18 k-steps,
// each with constant operands (zeros / ones) and with random f16 operands, at one and two workgroups per
// compute unit, and prints TFLOP/s and the shader clock seen by clock64() against the 100 MHz wall clock.
// Build: python -m paper_2602_00608_amd.build --diag      Run: paper_2602_00608_amd/mfma_ceiling
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <type_traits>
#include <utility>

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

#define CHECK(expr)                                                                      \
  do {                                                                                   \
    hipError_t e__ = (expr);                                                             \
    if (e__ != hipSuccess) { fprintf(stderr, "%s: %s\n", #expr, hipGetErrorString(e__)); exit(1); } \
  } while (0)

template <int N, typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl<N>(f, std::make_integer_sequence<int, N>{}); }

__device__ __forceinline__ f32x16 mma(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

constexpr int MI = 4, NI = 2, D = 3, KK = 2, STEPS = 18, HW_ = 34, PS = 40, TILE_PX = 340;

// LOOP: false = registers only, true = operands from LDS / L2
template <bool LOOP>
__global__ __launch_bounds__(256, 2) void kernel(const u32x4* __restrict__ w, float* out, long long* clk, int chunks,
                                                 int tap_stride, int kk_stride) {
  extern __shared__ __align__(16) unsigned char smem[];
  _Float16* buf = reinterpret_cast<_Float16*>(smem);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / 2, wn = wave % 2;
  // the LDS tile takes its bits from the weight blob: zeros or random, like the B operand
  for (int i = tid; i < TILE_PX * PS / 2; i += 256)
    reinterpret_cast<unsigned*>(smem)[i] = reinterpret_cast<const unsigned*>(w)[(i * 7 + blockIdx.x * 131) & 0xffff];
  __syncthreads();
  const int lm = lane & 31, lk = lane >> 5;
  int a_off[MI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) a_off[mi] = ((wm * MI + mi) * HW_ + lm) * PS + 8 * lk;
  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const u32x4* wcol = w + (size_t)(wn * NI + (blockIdx.x & 1) * 4) * 64;
  const int rot = blockIdx.x * 5;   // workgroups walk the blob out of step, as in a real launch
  u32x4 bq[D][NI];
#pragma unroll
  for (int sp = 0; sp < D; ++sp)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) bq[sp][ni] = (wcol + ((sp / KK) * tap_stride + (sp % KK) * kk_stride + ni * 64))[lane];
  u32x4 af[MI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) af[mi] = *reinterpret_cast<const u32x4*>(buf + a_off[mi]);
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int c = 0; c < chunks; ++c) {
    const u32x4* bcur = wcol + (size_t)(((c + rot) & 7) * KK) * kk_stride;
    const u32x4* bnext = wcol + (size_t)(((c + 1 + rot) & 7) * KK) * kk_stride;
    auto step = [&](auto s_c) {
      constexpr int s = decltype(s_c)::value;
      if constexpr (LOOP) {
        constexpr int sp = s + D - 1;
        const u32x4* src = sp < STEPS ? bcur : bnext;
        constexpr int spp = sp < STEPS ? sp : sp - STEPS;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) bq[sp % D][ni] = (src + ((spp / KK) * tap_stride + (spp % KK) * kk_stride + ni * 64))[lane];
        __builtin_amdgcn_sched_barrier(0);
      }
      auto tile = [&](auto mi_c) {
        constexpr int mi = decltype(mi_c)::value;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = mma(af[mi], bq[s % D][ni], acc[mi][ni]);
        if constexpr (LOOP) {
          constexpr int s1 = (s + 1) % STEPS, tap = s1 / KK, kk = s1 % KK;
          af[mi] = *reinterpret_cast<const u32x4*>(buf + a_off[mi] + ((tap / 3) * HW_ + tap % 3) * PS + kk * 16);
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      static_for<MI>(tile);
    };
    static_for<STEPS>(step);
    if constexpr (LOOP) __syncthreads();
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[i][j][r];
  out[blockIdx.x * 256 + tid] = s;
  if (tid == 0 && blockIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}

template <bool LOOP>
void run(const char* what, const u32x4* w, float* out, long long* clk, int wgs_per_cu) {
  const int chunks = 64, grid = 256 * wgs_per_cu;
  const int cout_blocks = 8, cin_blocks = 16;   // the packed weights of a 256 -> 256 layer
  const int tap_stride = cin_blocks * cout_blocks * 64, kk_stride = cout_blocks * 64;
  auto kern = kernel<LOOP>;
  CHECK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024));
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  kern<<<grid, 256, 60 * 1024>>>(w, out, clk, 4, tap_stride, kk_stride);
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0));
  kern<<<grid, 256, 60 * 1024>>>(w, out, clk, chunks, tap_stride, kk_stride);
  CHECK(hipEventRecord(e1));
  CHECK(hipDeviceSynchronize());
  float ms;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  long long h[2];
  CHECK(hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost));
  const double flops = (double)grid * 4 * chunks * STEPS * MI * NI * 32768.0;
  printf("%-34s %d workgroup(s)/CU: %8.1f TFLOP/s (%4.1f%% of 2516.6), shader clock %4.0f MHz\n", what, wgs_per_cu,
         flops / ms / 1e9, flops / ms / 1e9 / 25.166, (double)h[0] / (double)h[1] * 100.0);
  fflush(stdout);
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
}

int main() {
  const size_t wb = 9 * 256 * 256 * 2 + (1 << 20);
  u32x4* w; float* out; long long* clk;
  CHECK(hipMalloc(&w, wb));
  CHECK(hipMalloc(&out, 512 * 256 * sizeof(float)));
  CHECK(hipMalloc(&clk, 2 * sizeof(long long)));
  unsigned short* h = (unsigned short*)malloc(wb);
  for (int random = 0; random < 2; ++random) {
    unsigned x = 12345u;
    for (size_t i = 0; i < wb / 2; ++i) {   // random f16 in about [-2, 2): random sign, exponent 12..15, random mantissa
      x = x * 1664525u + 1013904223u;
      h[i] = random ? (unsigned short)(((x >> 16) & 0x8000u) | ((12u + ((x >> 8) & 3u)) << 10) | ((x >> 18) & 0x3ffu)) : 0;
    }
    CHECK(hipMemcpy(w, h, wb, hipMemcpyHostToDevice));
    for (int wg = 1; wg <= 2; ++wg) {
      run<false>(random ? "MFMA only, random f16 operands" : "MFMA only, constant operands", w, out, clk, wg);
      run<true>(random ? "conv inner loop, random operands" : "conv inner loop, constant operands", w, out, clk, wg);
    }
  }
  free(h);
  return 0;
}
