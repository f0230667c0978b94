// 3x3 convolution with very few output channels (the decoder's last layer, 128 -> 3) whose output is the planar
// fp32 frame: normalise + SiLU on the load path like the other convolutions, but the contraction is turned round.
//
// y[p][co] = sum_tap sum_ci a[p + tap][ci] * W[co][ci][tap] is evaluated as
//   u[q][j]  = sum_ci a[q][ci] * W[co][ci][tap],  j = tap * C_out + co   (a 1x1 contraction with 9 * C_out <= 32 outputs)
//   y[p][co] = bias[co] + sum_tap u[p + tap][tap * C_out + co]           (nine shifted reads per output)
// so a pixel's channels are contracted once instead of nine times, the whole weight tensor (32 x C_in) sits in the
// registers of every wavefront as MFMA B operands, and an input vector goes from memory straight into the A operand
// layout of the 32x32x16 MFMA (lane = pixel, 8 consecutive channels per k-step) with no LDS staging.  What is left is
// the work on the load path: the kernel is bound by the read of x and the normalise + SiLU arithmetic, not by the
// matrix pipe.  A workgroup of 4 wavefronts owns 8 x 32 output pixels, computes u for the 10 x 34 halo patch in 11
// M tiles of 32 pixels into LDS (fp32, pixel stride 27 floats: odd, so neighbouring pixels fall on different banks)
// and then sums the nine taps per output in a fixed order.  Pixels outside the image contribute u = 0 (zero padding in
// the activated domain).  The weights are read from the ordinary 3x3 pack.
#include "mfma.hpp"
#include "pack_layout.hpp"

namespace wmdec {
namespace {

struct TapsParams {
  const void* x; const float* mean; const float* rstd; const float* gamma; const float* beta;
  const void* w; const float* bias; float* y;
  int n, h, w_out, cout, groups, silu, tiles_x, tiles_y, cin_blocks;
};

constexpr int kTH = 8, kTW = 32, kHW = kTW + 2, kHH = kTH + 2, kHP = kHW * kHH;   // halo patch: 340 pixels
constexpr int kMT = (kHP + 31) / 32;                                              // M tiles of 32 pixels
constexpr int kNJ = 27;                                                           // floats of u per pixel

__device__ __forceinline__ float silu_scaled(float u) {   // silu(t) from u = -log2(e) * t
  constexpr float k = -1.4426950408889634f;
  return u * __builtin_amdgcn_rcpf(fmaf(__builtin_amdgcn_exp2f(u), k, k));
}

// KSTEPS = C_in / 16.  ACT: 0 plain, 1 scale/shift, 2 scale/shift + SiLU.
template <typename T, int KSTEPS, int ACT>
__global__ __launch_bounds__(256, 4) void conv_taps_kernel(TapsParams p) {
  constexpr int CIN = KSTEPS * 16;
  __shared__ __align__(16) float2 s_ab[CIN];
  __shared__ float s_u[kMT * 32 * kNJ];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int tiles = p.tiles_x * p.tiles_y;
  const int n = blockIdx.x / tiles, tile = blockIdx.x % tiles;
  const int ty0 = (tile / p.tiles_x) * kTH, tx0 = (tile % p.tiles_x) * kTW;
  const T* xin = reinterpret_cast<const T*>(p.x) + (size_t)n * p.h * p.w_out * CIN;

  // the lane's pixel of M tile mt, as a byte offset of its 8-channel run (0 outside the image: loaded, then zeroed)
  auto pixel = [&](int mt, bool* inside) -> int {
    const int hp = mt * 32 + l32;
    const int hy = hp / kHW, hx = hp % kHW;
    const int gy = ty0 + hy - 1, gx = tx0 + hx - 1;
    *inside = hp < kHP && gy >= 0 && gy < p.h && gx >= 0 && gx < p.w_out;
    return *inside ? ((gy * p.w_out + gx) * CIN + half * 8) * (int)sizeof(T) : half * 8 * (int)sizeof(T);
  };
  u32x4 a[KSTEPS];
  auto load_tile = [&](int off) {
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) a[s] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(xin) + (unsigned)(off + s * 32));
  };
  bool inside;
  int off = pixel(wave, &inside);
  load_tile(off);

  // B operands: column j = l32 of k-step s is W[co][16 s + 8 half ..][tap], which the 3x3 pack keeps in fragment
  // (tap, s) at lane co + 32 half
  u32x4 bw[KSTEPS];
  {
    const int tap = l32 / p.cout, co = l32 % p.cout;
    const bool used = l32 < 9 * p.cout;
    const T* wp = reinterpret_cast<const T*>(p.w);
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
      const size_t e = ((size_t)(used ? tap : 0) * p.cin_blocks + s) * 512 + (size_t)((used ? co : 0) + 32 * half) * 8;
      bw[s] = *reinterpret_cast<const u32x4*>(wp + e);
      if (!used) bw[s] = u32x4{0u, 0u, 0u, 0u};
    }
  }
  if constexpr (ACT > 0) {
    const int cpg = CIN / p.groups;
    const float k = ACT == 2 ? -1.4426950408889634f : 1.0f;
    for (int c = tid; c < CIN; c += 256) {
      const int g = c / cpg;
      const float sc = p.gamma[c] * p.rstd[n * p.groups + g];
      s_ab[c] = make_float2(k * sc, k * (p.beta[c] - p.mean[n * p.groups + g] * sc));
    }
    __syncthreads();
  }

  for (int mt = wave; mt < kMT; mt += 4) {
    if constexpr (ACT > 0) {
      // The table entries do not depend on the tile, and the compiler would keep all of them (4 * KSTEPS four-float
      // registers) across the loop and spill; the opaque offset makes it read them again per tile (the two halves of
      // a wavefront read two addresses: a broadcast, a few cycles per read).
      int toff = half * 8;
      asm volatile("" : "+v"(toff));
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) {
        const f32x4* tab = reinterpret_cast<const f32x4*>(s_ab + s * 16 + toff);
        uint32_t wv[4] = {a[s].x, a[s].y, a[s].z, a[s].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 ab = tab[q];
          float f0 = fmaf(unpack_lo<T>(wv[q]), ab[0], ab[1]), f1 = fmaf(unpack_hi<T>(wv[q]), ab[2], ab[3]);
          if constexpr (ACT == 2) { f0 = silu_scaled(f0); f1 = silu_scaled(f1); }
          wv[q] = pack2<T>(f0, f1);
        }
        a[s] = u32x4{wv[0], wv[1], wv[2], wv[3]};
      }
    }
    if (!inside) {
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) a[s] = u32x4{0u, 0u, 0u, 0u};
    }
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) acc = Mma<T>::m32(a[s], bw[s], acc);
    // the next tile's vectors travel while this one's results go to LDS
    if (mt + 4 < kMT) {
      off = pixel(mt + 4, &inside);
      load_tile(off);
    }
    if (l32 < kNJ) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s_u[(mt * 32 + 8 * (r / 4) + 4 * half + (r % 4)) * kNJ + l32] = acc[r];
    }
  }
  __syncthreads();

  const int ty = tid / kTW, tx = tid % kTW;
  const int gy = ty0 + ty, gx = tx0 + tx;
  if (gy < p.h && gx < p.w_out) {
    for (int co = 0; co < p.cout; ++co) {
      float sum = p.bias ? p.bias[co] : 0.f;
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) sum += s_u[((ty + tap / 3) * kHW + tx + tap % 3) * kNJ + tap * p.cout + co];
      p.y[(((size_t)n * p.cout + co) * p.h + gy) * p.w_out + gx] = sum;
    }
  }
}

template <typename T, int KSTEPS>
int launch_k(const TapsParams& p, bool norm, hipStream_t s) {
  void (*kern)(TapsParams) = !norm ? conv_taps_kernel<T, KSTEPS, 0> : (p.silu ? conv_taps_kernel<T, KSTEPS, 2> : conv_taps_kernel<T, KSTEPS, 1>);
  hipLaunchKernelGGL(kern, dim3((unsigned)(p.tiles_x * p.tiles_y * p.n)), dim3(256), 0, s, p);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

}  // namespace

bool conv_taps_supported(const ConvArgs& a) {
  if (!is_16bit(a.op_dtype) || a.x_dtype != a.op_dtype || a.x_nchw) return false;
  if (!a.y_nchw || a.y_dtype != WMDEC_F32 || a.ksize != 3 || a.upsample) return false;
  if (a.res || a.x2 || a.stats_ws || a.rows_in || a.rows_out) return false;
  if (a.cout < 1 || a.cout > 3 || (a.cin != 64 && a.cin != 128)) return false;
  if (a.groups < 1 || a.cin % a.groups != 0) return false;
  if ((long)a.h * a.w * a.cin >= (1L << 29)) return false;   // 32-bit byte offsets per sample
  return true;
}

const char* conv_taps_label(const ConvArgs& a) {
  static thread_local char buf[96];
  const int act = a.mean == nullptr && !a.groups_norm ? 0 : (a.silu ? 2 : 1);
  snprintf(buf, sizeof(buf), "conv_taps_kernel<%s, %d, %d>", a.op_dtype == WMDEC_BF16 ? "wmdec::bf16_t" : "wmdec::f16_t", a.cin / 16, act);
  return buf;
}

int launch_conv_taps(const ConvArgs& a, hipStream_t s) {
  WMDEC_REQUIRE(conv_taps_supported(a), WMDEC_ERR_UNSUPPORTED, "conv_taps: unsupported shape");
  TapsParams p;
  p.x = a.x; p.mean = a.mean; p.rstd = a.rstd; p.gamma = a.gamma; p.beta = a.beta; p.w = a.wt; p.bias = a.bias;
  p.y = (float*)a.y; p.n = a.n; p.h = a.h; p.w_out = a.w; p.cout = a.cout; p.groups = a.groups; p.silu = a.silu;
  p.tiles_x = (a.w + kTW - 1) / kTW; p.tiles_y = (a.h + kTH - 1) / kTH; p.cin_blocks = packed_cin_blocks(a.cin);
  const bool norm = a.mean != nullptr;
  if (a.op_dtype == WMDEC_BF16) return a.cin == 128 ? launch_k<bf16_t, 8>(p, norm, s) : launch_k<bf16_t, 4>(p, norm, s);
  return a.cin == 128 ? launch_k<f16_t, 8>(p, norm, s) : launch_k<f16_t, 4>(p, norm, s);
}

}  // namespace wmdec
