// Implicit-GEMM convolution on the gfx950 matrix cores.
//
// GEMM view: M = output pixels, N = output channels, K = taps * C_in.
// One workgroup (4 wavefronts) owns a TH x TW patch of output pixels and TN
// output channels.  Per chunk of KC input channels it stages the patch plus its
// one-pixel halo into LDS -- GroupNorm scale/shift and SiLU are applied there,
// once per element, positions outside the image become zeros, and a folded
// nearest-2x upsample is just a different source address -- and then sweeps the
// nine taps over that tile: the A operand of every MFMA is a 16-byte LDS read
// at a tap-dependent constant offset, the B operand (weights) comes straight
// from global memory, where the packed layout stores every 32(co) x 16(ci)
// fragment as 1 KiB in lane order, so a wavefront's load is one contiguous KiB.
// Accumulators stay in registers for the whole K loop; bias, residual and the
// single rounding to the storage type happen in the epilogue.
// Two workgroups fit on a compute unit (registers <= 256, LDS < 80 KiB), so one
// stages while the other multiplies.
#include "mfma.hpp"
#include "pack_layout.hpp"

namespace wmdec {
namespace {

struct MfmaParams {
  const void* x; const float* mean; const float* rstd; const float* gamma; const float* beta;
  const void* w; const float* bias; const void* res; void* y;
  int silu, groups, norm;
  int n, h, w_out, cin, cout, upsample;
  int tiles_x, tiles_y, ntiles, total;
  int cin_blocks, cout_blocks;   // packed-layout extents: ceil(cin/16), ceil(cout/32)
};

template <typename T> __device__ __forceinline__ void unpack8(const u32x4& v, float* f) {
  f[0] = unpack_lo<T>(v.x); f[1] = unpack_hi<T>(v.x); f[2] = unpack_lo<T>(v.y); f[3] = unpack_hi<T>(v.y);
  f[4] = unpack_lo<T>(v.z); f[5] = unpack_hi<T>(v.z); f[6] = unpack_lo<T>(v.w); f[7] = unpack_hi<T>(v.w);
}

template <typename T, typename TO, int TH, int TW, int WM, int WN, int NI, int KS, int KC>
__global__ __launch_bounds__(256, 2) void conv_mfma_kernel(MfmaParams p) {
  static_assert(WM * WN == 4, "four wavefronts");
  constexpr int MI = TH * TW / 32 / WM;          // 32-pixel M tiles per wavefront
  constexpr int PAD = KS / 2;
  constexpr int HW_ = TW + 2 * PAD, HH_ = TH + 2 * PAD, HP = HW_ * HH_;
  constexpr int PS = KC + 8;                     // LDS pixel stride in elements (+16 B: conflict-free 16-byte reads)
  constexpr int MTW = TW < 32 ? TW : 32, MTH = 32 / MTW, MT_PER_ROW = TW / MTW;
  constexpr int TN = WN * NI * 32;
  constexpr int VPP = KC / 8;                    // 16-byte vectors per pixel per chunk
  static_assert(256 % VPP == 0, "a thread keeps one channel octet");

  extern __shared__ __align__(16) unsigned char smem[];
  T* s_a = reinterpret_cast<T*>(smem);                                   // [HP][PS]
  float2* s_ab = reinterpret_cast<float2*>(smem + ((HP * PS * 2 + 15) & ~15));  // [cin] (scale, shift)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int lm = lane & 31, lk = lane >> 5;

  // workgroup id -> (channel tile, sample, spatial tile); consecutive ids of one XCD (id % 8) are neighbours
  int L;
  {
    const int i = blockIdx.x, per = p.total / 8, rem = p.total % 8;
    const int x = i % 8, j = i / 8;
    L = x * per + (x < rem ? x : rem) + j;
  }
  const int tiles = p.tiles_x * p.tiles_y;
  const int nt = L / (tiles * p.n);
  const int n = (L / tiles) % p.n;
  const int tile = L % tiles;
  const int ty0 = (tile / p.tiles_x) * TH, tx0 = (tile % p.tiles_x) * TW;
  const int co0 = nt * TN;
  const int h_in = p.upsample ? p.h >> 1 : p.h, w_in = p.upsample ? p.w_out >> 1 : p.w_out;

  // per-channel scale/shift table: a = gamma*rstd, b = beta - mean*a
  if (p.norm) {
    const int cpg = p.cin / p.groups;
    for (int c = tid; c < p.cin; c += 256) {
      const int g = c / cpg;
      const float a = p.gamma[c] * p.rstd[n * p.groups + g];
      s_ab[c] = make_float2(a, p.beta[c] - p.mean[n * p.groups + g] * a);
    }
  }

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // LDS element offset of this lane's pixel in each of its M tiles (tap (0,0), k offset of the lane half)
  int a_off[MI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int mt = wm * MI + mi;
    const int ty = (mt / MT_PER_ROW) * MTH + lm / MTW, tx = (mt % MT_PER_ROW) * MTW + lm % MTW;
    a_off[mi] = (ty * HW_ + tx) * PS + 8 * lk;
  }
  const T* xin = reinterpret_cast<const T*>(p.x) + (size_t)n * h_in * w_in * p.cin;
  const u32x4* wfrag = reinterpret_cast<const u32x4*>(p.w) + lane;   // + block * 64
  const int cvec = tid % VPP;

  for (int c0 = 0; c0 < p.cin; c0 += KC) {
    __syncthreads();   // previous chunk's MFMA reads are done (also orders the s_ab writes)
    // ---- stage the activated halo tile of channels [c0, c0+KC)
    {
      float sc[8], sh[8];
      if (p.norm) {
#pragma unroll
        for (int j = 0; j < 8; ++j) { const float2 ab = s_ab[c0 + cvec * 8 + j]; sc[j] = ab.x; sh[j] = ab.y; }
      }
      for (int v = tid; v < HP * VPP; v += 256) {
        const int hp = v / VPP;
        const int hy = hp / HW_, hx = hp % HW_;
        const int gy = ty0 + hy - PAD, gx = tx0 + hx - PAD;
        u32x4 out = u32x4{0u, 0u, 0u, 0u};
        if (gy >= 0 && gy < p.h && gx >= 0 && gx < p.w_out) {
          const int sy = p.upsample ? gy >> 1 : gy, sx = p.upsample ? gx >> 1 : gx;
          const u32x4 raw = *reinterpret_cast<const u32x4*>(xin + ((size_t)sy * w_in + sx) * p.cin + c0 + cvec * 8);
          if (p.norm) {
            float f[8];
            unpack8<T>(raw, f);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              f[j] = fmaf(f[j], sc[j], sh[j]);
              if (p.silu) f[j] = silu_f(f[j]);
            }
            out = u32x4{pack2<T>(f[0], f[1]), pack2<T>(f[2], f[3]), pack2<T>(f[4], f[5]), pack2<T>(f[6], f[7])};
          } else {
            out = raw;
          }
        }
        *reinterpret_cast<u32x4*>(s_a + hp * PS + cvec * 8) = out;
      }
    }
    __syncthreads();
    // ---- nine taps x KC/16 k-steps of MFMAs
    const int cb0 = c0 / 16;
#pragma unroll
    for (int tap = 0; tap < KS * KS; ++tap) {
      const int ky = tap / KS, kx = tap % KS;
#pragma unroll
      for (int kk = 0; kk < KC / 16; ++kk) {
        u32x4 bf[NI];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
          const int blk = (tap * p.cin_blocks + cb0 + kk) * p.cout_blocks + (co0 >> 5) + wn * NI + ni;
          bf[ni] = wfrag[(size_t)blk * 64];
        }
        u32x4 af[MI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          af[mi] = *reinterpret_cast<const u32x4*>(s_a + a_off[mi] + (ky * HW_ + kx) * PS + kk * 16);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = Mma<T>::m32(af[mi], bf[ni], acc[mi][ni]);
      }
    }
  }

  // ---- epilogue: bias, residual, one rounding, store
  TO* yout = reinterpret_cast<TO*>(p.y) + (size_t)n * p.h * p.w_out * p.cout;
  const T* rin = p.res ? reinterpret_cast<const T*>(p.res) + (size_t)n * p.h * p.w_out * p.cout : nullptr;
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int co = co0 + (wn * NI + ni) * 32 + lm;
    const float bv = p.bias ? p.bias[co] : 0.f;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int mt = wm * MI + mi;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = 8 * (r / 4) + 4 * lk + (r % 4);     // row of the 32x32 tile = pixel of the M tile
        const int oy = ty0 + (mt / MT_PER_ROW) * MTH + i / MTW, ox = tx0 + (mt % MT_PER_ROW) * MTW + i % MTW;
        if (oy < p.h && ox < p.w_out) {
          const size_t idx = ((size_t)oy * p.w_out + ox) * p.cout + co;
          float v = acc[mi][ni][r] + bv;
          if (rin) v += to_float(rin[idx]);
          yout[idx] = from_float<TO>(v);
        }
      }
    }
  }
}

template <typename T, typename TO, int TH, int TW, int WM, int WN, int NI, int KS, int KC>
int launch_cfg(const ConvArgs& a, hipStream_t s) {
  constexpr int PAD = KS / 2;
  constexpr int HP = (TW + 2 * PAD) * (TH + 2 * PAD);
  constexpr int TN = WN * NI * 32;
  MfmaParams p;
  p.x = a.x; p.mean = a.mean; p.rstd = a.rstd; p.gamma = a.gamma; p.beta = a.beta;
  p.w = a.wt; p.bias = a.bias; p.res = a.res; p.y = a.y;
  p.silu = a.silu; p.groups = a.groups; p.norm = a.mean != nullptr;
  p.n = a.n; p.h = a.h; p.w_out = a.w; p.cin = a.cin; p.cout = a.cout; p.upsample = a.upsample;
  p.tiles_x = (a.w + TW - 1) / TW; p.tiles_y = (a.h + TH - 1) / TH; p.ntiles = a.cout / TN;
  p.total = p.tiles_x * p.tiles_y * p.ntiles * a.n;
  p.cin_blocks = packed_cin_blocks(a.cin); p.cout_blocks = packed_cout_blocks(a.cout);
  const size_t smem = (((size_t)HP * (KC + 8) * 2 + 15) & ~(size_t)15) + (size_t)a.cin * sizeof(float2);
  auto kern = conv_mfma_kernel<T, TO, TH, TW, WM, WN, NI, KS, KC>;
  static bool attr_set = false;   // per instantiation
  if (!attr_set) {
    WMDEC_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024));
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)p.total), dim3(256), smem, s, p);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

template <typename T, typename TO, int KS>
int launch_shape(const ConvArgs& a, hipStream_t s) {
  // tile choice: 256 pixels x 128 channels when that still gives every compute unit work, else smaller
  const long px = (long)a.n * a.h * a.w;
  if (a.cout % 128 == 0 && px * (a.cout / 128) >= 256L * 256 * 3) return launch_cfg<T, TO, 8, 32, 2, 2, 2, KS, 32>(a, s);
  if (a.cout % 128 == 0 && px * (a.cout / 128) >= 128L * 256 * 3) return launch_cfg<T, TO, 4, 32, 2, 2, 2, KS, 32>(a, s);
  return launch_cfg<T, TO, 4, 32, 4, 1, 2, KS, 32>(a, s);   // 128 pixels x 64 channels
}

template <typename T>
int launch_type(const ConvArgs& a, hipStream_t s) {
  if (a.y_dtype == WMDEC_F32)
    return a.ksize == 3 ? launch_shape<T, float, 3>(a, s) : launch_shape<T, float, 1>(a, s);
  return a.ksize == 3 ? launch_shape<T, T, 3>(a, s) : launch_shape<T, T, 1>(a, s);
}

}  // namespace

bool conv_mfma_supported(const ConvArgs& a) {
  if (!is_16bit(a.op_dtype) || a.x_dtype != a.op_dtype) return false;
  if (a.res && a.res_dtype != a.op_dtype) return false;
  if (a.y_dtype != a.op_dtype && a.y_dtype != WMDEC_F32) return false;
  if (a.x_nchw || a.y_nchw) return false;
  if (a.cin % 32 != 0 || a.cout % 64 != 0) return false;
  if (a.cin > 4096) return false;   // scale/shift table lives in LDS
  if (a.ksize != 1 && a.ksize != 3) return false;
  return true;
}

int launch_conv_mfma(const ConvArgs& a, hipStream_t s) {
  return a.op_dtype == WMDEC_BF16 ? launch_type<bf16_t>(a, s) : launch_type<f16_t>(a, s);
}

}  // namespace wmdec
