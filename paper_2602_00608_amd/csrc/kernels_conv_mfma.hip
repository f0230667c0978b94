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
#include <stdlib.h>

#include "mfma.hpp"
#include "pack_layout.hpp"

namespace wmdec {
namespace {

int g_dbg = 0;
int g_tile = -1;
int g_variant = 0;   // kernel variant under evaluation (set from WMDEC_CONV_VARIANT at first launch)

struct MfmaParams {
  const void* x; const float* mean; const float* rstd; const float* gamma; const float* beta;
  const void* w; const float* bias; const void* res; void* y;
  int silu, groups, norm;
  int n, h, w_out, cin, cout, upsample;
  int tiles_x, tiles_y, ntiles, total;
  int cin_blocks, cout_blocks;   // packed-layout extents: ceil(cin/16), ceil(cout/32)
  int y_nchw;                    // 1: y is planar [n][cout][h][w] (the frame), else NHWC
  int dbg;                       // ablation switches for timing experiments (0 in production)
};

template <typename T> __device__ __forceinline__ void unpack8(const u32x4& v, float* f) {
  f[0] = unpack_lo<T>(v.x); f[1] = unpack_hi<T>(v.x); f[2] = unpack_lo<T>(v.y); f[3] = unpack_hi<T>(v.y);
  f[4] = unpack_lo<T>(v.z); f[5] = unpack_hi<T>(v.z); f[6] = unpack_lo<T>(v.w); f[7] = unpack_hi<T>(v.w);
}



// Epilogue of one wavefront: its MI x NI accumulator tiles (32 pixels x 32 channels each, a lane
// holding one channel column) go through a wavefront-private LDS patch, one 32-pixel M tile at a
// time, and come back as rows of 8 consecutive channels per lane, so that bias, residual and the
// output move as 16-byte vectors and every pixel's channel run is written contiguously.
// lds: 32 x (NI*32 + 4) floats owned by this wavefront.  LDS operations of one wavefront execute
// in order, so the patch needs no barrier between its write and read phases.
template <typename T, typename TO, int MI, int NI, int MTW, int MTH, int MT_PER_ROW>
__device__ __forceinline__ void epilogue_store(const f32x16 (&acc)[MI][NI], float* lds, int lane, int mt0, int ty0,
                                               int tx0, int co_w, const float* bias, const T* rin, TO* yout, int h,
                                               int w_out, int cout, bool skip, bool nchw) {
  constexpr int RW = NI * 32 + 4;       // padded row of the patch, floats
  if (nchw) {
    // planar output with few channels (the frame): a lane owns one pixel of the M tile and walks the
    // channels, so that 32 lanes write 32 consecutive pixels of one plane
    const int lm = lane & 31, lk = lane >> 5;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int mt = mt0 + mi;
      const int oy = ty0 + (mt / MT_PER_ROW) * MTH + lm / MTW, ox = tx0 + (mt % MT_PER_ROW) * MTW + lm % MTW;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r) lds[(8 * (r / 4) + 4 * lk + (r % 4)) * RW + ni * 32 + lm] = acc[mi][ni][r];
      if (oy < h && ox < w_out && !skip) {
        for (int c = lk; c < NI * 32 && co_w + c < cout; c += 2) {
          const float v = lds[lm * RW + c] + (bias ? bias[co_w + c] : 0.f);
          yout[((size_t)(co_w + c) * h + oy) * w_out + ox] = from_float<TO>(v);
        }
      }
    }
    return;
  }
  constexpr int VPL = 2 * NI;           // 8-channel vectors per lane per M tile (32 pixels x NI*4 vectors / 64 lanes)
  const int lm = lane & 31, lk = lane >> 5;
  const int cvec = lane % (NI * 4);     // which 8-channel vector of the row this lane reads back
  const int prow = lane / (NI * 4);     // first pixel row it reads; the others are prow + j * (64 / (NI*4))
  float bv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) bv[e] = bias ? bias[co_w + cvec * 8 + e] : 0.f;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int mt = mt0 + mi;
    const int py0 = ty0 + (mt / MT_PER_ROW) * MTH, px0 = tx0 + (mt % MT_PER_ROW) * MTW;
    // residual vectors first: their latency hides behind the LDS round trip
    u32x4 rv[VPL];
    bool ok[VPL];
    size_t idx[VPL];
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int pi = prow + j * (64 / (NI * 4));
      const int oy = py0 + pi / MTW, ox = px0 + pi % MTW;
      ok[j] = oy < h && ox < w_out && !skip;
      idx[j] = ((size_t)oy * w_out + ox) * cout + co_w + cvec * 8;
      rv[j] = u32x4{0u, 0u, 0u, 0u};
      if (rin && ok[j]) rv[j] = *reinterpret_cast<const u32x4*>(rin + idx[j]);
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) lds[(8 * (r / 4) + 4 * lk + (r % 4)) * RW + ni * 32 + lm] = acc[mi][ni][r];
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int pi = prow + j * (64 / (NI * 4));
      const f32x4 lo = *reinterpret_cast<const f32x4*>(lds + pi * RW + cvec * 8);
      const f32x4 hi = *reinterpret_cast<const f32x4*>(lds + pi * RW + cvec * 8 + 4);
      float v[8] = {lo[0] + bv[0], lo[1] + bv[1], lo[2] + bv[2], lo[3] + bv[3],
                    hi[0] + bv[4], hi[1] + bv[5], hi[2] + bv[6], hi[3] + bv[7]};
      if (rin) {
        float rf[8];
        unpack8<T>(rv[j], rf);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += rf[e];
      }
      if (ok[j]) {
        if constexpr (sizeof(TO) == 4) {
          f32x4* dst = reinterpret_cast<f32x4*>(yout + idx[j]);
          dst[0] = f32x4{v[0], v[1], v[2], v[3]};
          dst[1] = f32x4{v[4], v[5], v[6], v[7]};
        } else {
          *reinterpret_cast<u32x4*>(yout + idx[j]) =
              u32x4{pack2<T>(v[0], v[1]), pack2<T>(v[2], v[3]), pack2<T>(v[4], v[5]), pack2<T>(v[6], v[7])};
        }
      }
    }
  }
}

// Ring length of the weight-fragment prefetch: it must divide the k-steps of a chunk so that the ring
// position is the same at every chunk start.
constexpr int prefetch_ring(int steps) { return steps % 3 == 0 ? 3 : (steps % 4 == 0 ? 4 : 2); }

// MFMA work of one staged chunk: STEPS = taps * KC/16 k-steps, each MI x NI 32x32x16 MFMAs.
// Weight fragments are fetched D-1 steps ahead (bq is a ring that persists across chunks: on
// entry it holds steps 0..D-2 of this chunk, on exit steps 0..D-2 of the chunk at `bnext`),
// A fragments one step ahead.  The scheduling barriers pin that order: without them the
// compiler sinks every load to just before its use and each k-step pays a full memory latency.
template <typename T, int MI, int NI, int KS, int KC, int HW_, int PS, int D>
__device__ __forceinline__ void mfma_chunk(const T* buf, const int (&a_off)[MI], const u32x4* bcur, const u32x4* bnext,
                                           int tap_stride, int kk_stride, int lane, u32x4 (&bq)[D][NI],
                                           f32x16 (&acc)[MI][NI], int dbg = 0) {
  if (dbg & 2) { tap_stride = 0; kk_stride = 0; bnext = bcur; }   // ablation: every fragment load hits the same KiB
  constexpr int KK = KC / 16, STEPS = KS * KS * KK;
  u32x4 af[2][MI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) af[0][mi] = *reinterpret_cast<const u32x4*>(buf + a_off[mi]);
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    if (!(dbg & 16)) {
      const int sp = s + D - 1;
      const u32x4* src = sp < STEPS ? bcur : bnext;
      const int spp = sp < STEPS ? sp : sp - STEPS;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        bq[sp % D][ni] = (src + ((spp / KK) * tap_stride + (spp % KK) * kk_stride + ni * 64))[lane];
    }
    if (s + 1 < STEPS && !(dbg & 8)) {
      const int tap = (s + 1) / KK, kk = (s + 1) % KK;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        af[(s + 1) & 1][mi] = *reinterpret_cast<const u32x4*>(buf + a_off[mi] + ((tap / KS) * HW_ + tap % KS) * PS + kk * 16);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = Mma<T>::m32(af[s & 1][mi], bq[s % D][ni], acc[mi][ni]);
    __builtin_amdgcn_sched_barrier(0);
  }
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
  constexpr int KK = KC / 16;
  constexpr int D = prefetch_ring(KS * KS * KK);   // weight fragments are fetched D-1 k-steps ahead
  const int tap_stride = p.cin_blocks * p.cout_blocks * 64, kk_stride = p.cout_blocks * 64;   // in 16-byte units
  // fragment column of this wavefront (uniform pointer; the lane index is added at the load)
  const u32x4* wcol = reinterpret_cast<const u32x4*>(p.w) + (size_t)((co0 >> 5) + wn * NI) * 64;
  const int cvec = tid % VPP;
  u32x4 bq[D][NI];
#pragma unroll
  for (int sp = 0; sp < D - 1; ++sp)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) bq[sp][ni] = (wcol + ((sp / KK) * tap_stride + (sp % KK) * kk_stride + ni * 64))[lane];

  for (int c0 = 0; c0 < p.cin; c0 += KC) {
    __syncthreads();   // previous chunk's MFMA reads are done (also orders the s_ab writes)
    // ---- stage the activated halo tile of channels [c0, c0+KC)
    {
      float sc[8], sh[8];
      if (p.norm) {
#pragma unroll
        for (int j = 0; j < 8; ++j) { const float2 ab = s_ab[c0 + cvec * 8 + j]; sc[j] = ab.x; sh[j] = ab.y; }
      }
      for (int v = tid; v < ((p.dbg & 1) ? 0 : HP * VPP); v += 256) {
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
    const u32x4* bcur = wcol + (size_t)(c0 / 16) * kk_stride;
    const u32x4* bnext = c0 + KC < p.cin ? bcur + (size_t)(KC / 16) * kk_stride : bcur;
    mfma_chunk<T, MI, NI, KS, KC, HW_, PS, D>(s_a, a_off, bcur, bnext, tap_stride, kk_stride, lane, bq, acc, p.dbg);
  }

  // ---- epilogue: bias, residual, one rounding, store (through a wavefront-private LDS patch)
  __syncthreads();   // every wavefront is done with the staged tile; its LDS is reused
  TO* yout = reinterpret_cast<TO*>(p.y) + (size_t)n * p.h * p.w_out * p.cout;
  const T* rin = p.res ? reinterpret_cast<const T*>(p.res) + (size_t)n * p.h * p.w_out * p.cout : nullptr;
  float* patch = reinterpret_cast<float*>(smem) + wave * (32 * (NI * 32 + 4));
  epilogue_store<T, TO, MI, NI, MTW, MTH, MT_PER_ROW>(acc, patch, lane, wm * MI, ty0, tx0, co0 + wn * NI * 32, p.bias, rin,
                                                      yout, p.h, p.w_out, p.cout, (p.dbg & 4) != 0, p.y_nchw != 0);
}

// ---------------------------------------------------------------------------
// Wavefront-specialised, persistent variant: 8 wavefronts per workgroup, one
// workgroup per compute unit.  Wavefronts 0-3 (consumers) only read LDS, load
// weight fragments and issue MFMAs; wavefronts 4-7 (producers) only stage: they
// fetch the next chunk's halo tile from global memory one chunk ahead, apply
// scale/shift + SiLU and write the other half of a double-buffered LDS tile.
// One workgroup barrier per chunk hands a buffer over.  A workgroup walks a
// strided list of tiles, so the producers already stage the next tile while
// the consumers run the epilogue of the current one.
template <typename T, typename TO, int TH, int TW, int WM, int WN, int NI, int KS, int KC>
__global__ __launch_bounds__(512, 1) void conv_ws_kernel(MfmaParams p) {
  static_assert(WM * WN == 4, "four consumer wavefronts");
  constexpr int MI = TH * TW / 32 / WM;
  constexpr int PAD = KS / 2;
  constexpr int HW_ = TW + 2 * PAD, HH_ = TH + 2 * PAD, HP = HW_ * HH_;
  constexpr int PS = KC + 8;
  constexpr int MTW = TW < 32 ? TW : 32, MTH = 32 / MTW, MT_PER_ROW = TW / MTW;
  constexpr int TN = WN * NI * 32;
  constexpr int VPP = KC / 8;
  constexpr int NV = (HP * VPP + 255) / 256;     // 16-byte vectors a producer thread stages per chunk
  constexpr int STEPS = KS * KS * (KC / 16);     // MFMA k-steps per chunk
  constexpr int D = prefetch_ring(STEPS);        // weight fragments are fetched D-1 steps ahead
  static_assert(256 % VPP == 0, "shape assumptions");

  extern __shared__ __align__(16) unsigned char smem[];
  T* s_a = reinterpret_cast<T*>(smem);           // [2][HP][PS]

  const int tid = threadIdx.x;
  const int tiles = p.tiles_x * p.tiles_y;
  const int nchunks = p.cin / KC;
  // this workgroup's tiles: first + k*gridDim.x; workgroups of one XCD (blockIdx % 8) get neighbouring tiles
  const int nwg = gridDim.x;
  const int first = (blockIdx.x % 8) * (nwg / 8) + blockIdx.x / 8;
  const int my_tiles = first < p.total ? (p.total - first + nwg - 1) / nwg : 0;
  const int G = my_tiles * nchunks;
  const int h_in = p.upsample ? p.h >> 1 : p.h, w_in = p.upsample ? p.w_out >> 1 : p.w_out;

  if (tid < 256) {
    // ------------------------------------------------------------ consumers
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lm = lane & 31, lk = lane >> 5;
    int a_off[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int mt = wm * MI + mi;
      const int ty = (mt / MT_PER_ROW) * MTH + lm / MTW, tx = (mt % MT_PER_ROW) * MTW + lm % MTW;
      a_off[mi] = (ty * HW_ + tx) * PS + 8 * lk;
    }
    const int tap_stride = p.cin_blocks * p.cout_blocks * 64, kk_stride = p.cout_blocks * 64;   // 16-byte units
    constexpr int KK = KC / 16;
    // fragment base (uniform) of (tile sequence number, chunk): channel-tile column of this wavefront, first ci block
    auto frag_base = [&](int k, int c) -> const u32x4* {
      const int L = first + k * nwg;
      const int nt = L / (tiles * p.n);
      return reinterpret_cast<const u32x4*>(p.w) + ((size_t)(c * KK) * p.cout_blocks + (nt * TN >> 5) + wn * NI) * 64;
    };
    u32x4 bq[D][NI];
    if (G > 0) {
      const u32x4* b0 = frag_base(0, 0);
#pragma unroll
      for (int sp = 0; sp < D - 1; ++sp)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) bq[sp][ni] = (b0 + ((sp / KK) * tap_stride + (sp % KK) * kk_stride + ni * 64))[lane];
    }
    __syncthreads();   // first buffer staged
    int g = 0;
    for (int k = 0; k < my_tiles; ++k) {
      const int L = first + k * nwg;
      const int nt = L / (tiles * p.n);
      const int n = (L / tiles) % p.n;
      const int tile = L % tiles;
      const int ty0 = (tile / p.tiles_x) * TH, tx0 = (tile % p.tiles_x) * TW;
      const int co0 = nt * TN;
      f32x16 acc[MI][NI];
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
      for (int c = 0; c < nchunks; ++c, ++g) {
        const T* buf = s_a + (g & 1) * (HP * PS);
        const u32x4* bcur = frag_base(k, c);
        // where the fragments after this chunk come from: next chunk, next tile, or (at the very end) here again
        const u32x4* bnext = (c + 1 < nchunks) ? frag_base(k, c + 1) : (k + 1 < my_tiles ? frag_base(k + 1, 0) : bcur);
        mfma_chunk<T, MI, NI, KS, KC, HW_, PS, D>(buf, a_off, bcur, bnext, tap_stride, kk_stride, lane, bq, acc, p.dbg);
        __syncthreads();   // this buffer may be refilled, the other one is ready
      }
      // epilogue: bias, residual, one rounding, store (wavefront-private LDS patch behind the two tile buffers)
      TO* yout = reinterpret_cast<TO*>(p.y) + (size_t)n * p.h * p.w_out * p.cout;
      const T* rin = p.res ? reinterpret_cast<const T*>(p.res) + (size_t)n * p.h * p.w_out * p.cout : nullptr;
      float* patch = reinterpret_cast<float*>(smem + 2 * HP * PS * 2) + wave * (32 * (NI * 32 + 4));
      epilogue_store<T, TO, MI, NI, MTW, MTH, MT_PER_ROW>(acc, patch, lane, wm * MI, ty0, tx0, co0 + wn * NI * 32, p.bias,
                                                          rin, yout, p.h, p.w_out, p.cout, (p.dbg & 4) != 0, p.y_nchw != 0);
    }
  } else {
    // ------------------------------------------------------------ producers
    const int ptid = tid - 256;
    const int cvec = ptid % VPP;
    const int cpg = p.norm ? p.cin / p.groups : 1;
    u32x4 raw[NV];
    unsigned valid = 0;
    float sc[8], sh[8];
    auto issue = [&](int gg) {
      const int k = gg / nchunks, c0 = (gg % nchunks) * KC;
      const int L = first + k * nwg;
      const int n = (L / tiles) % p.n;
      const int tile = L % tiles;
      const int ty0 = (tile / p.tiles_x) * TH, tx0 = (tile % p.tiles_x) * TW;
      const T* xin = reinterpret_cast<const T*>(p.x) + (size_t)n * h_in * w_in * p.cin + c0 + cvec * 8;
      valid = 0;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int v = ptid + i * 256;
        const int hp = v / VPP;
        const int hy = hp / HW_, hx = hp % HW_;
        const int gy = ty0 + hy - PAD, gx = tx0 + hx - PAD;
        raw[i] = u32x4{0u, 0u, 0u, 0u};
        if (v < HP * VPP && gy >= 0 && gy < p.h && gx >= 0 && gx < p.w_out) {
          const int sy = p.upsample ? gy >> 1 : gy, sx = p.upsample ? gx >> 1 : gx;
          raw[i] = *reinterpret_cast<const u32x4*>(xin + ((size_t)sy * w_in + sx) * p.cin);
          valid |= 1u << i;
        }
      }
      if (p.norm) {
        const int cb = c0 + cvec * 8;
        const float4 g0 = *reinterpret_cast<const float4*>(p.gamma + cb), g1 = *reinterpret_cast<const float4*>(p.gamma + cb + 4);
        const float4 b0 = *reinterpret_cast<const float4*>(p.beta + cb), b1 = *reinterpret_cast<const float4*>(p.beta + cb + 4);
        const float ga[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        const float be[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int grp = n * p.groups + (cb + j) / cpg;
          sc[j] = ga[j] * p.rstd[grp];
          sh[j] = be[j] - p.mean[grp] * sc[j];
        }
      }
    };
    auto process = [&](int gg) {
      T* buf = s_a + (gg & 1) * (HP * PS);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int v = ptid + i * 256;
        if (v < HP * VPP) {
          u32x4 out = raw[i];
          if (p.norm && (valid >> i & 1u)) {
            float f[8];
            unpack8<T>(out, f);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              f[j] = fmaf(f[j], sc[j], sh[j]);
              if (p.silu) f[j] = silu_f(f[j]);
            }
            out = u32x4{pack2<T>(f[0], f[1]), pack2<T>(f[2], f[3]), pack2<T>(f[4], f[5]), pack2<T>(f[6], f[7])};
          }
          *reinterpret_cast<u32x4*>(buf + (v / VPP) * PS + cvec * 8) = out;
        }
      }
    };
    if (G > 0) {
      issue(0);
      process(0);
      if (G > 1) issue(1);
    }
    __syncthreads();   // first buffer staged
    for (int g = 0; g < G; ++g) {
      if (g + 1 < G) {
        process(g + 1);
        if (g + 2 < G) issue(g + 2);
      }
      __syncthreads();
    }
  }
}

template <typename T, typename TO, int TH, int TW, int WM, int WN, int NI, int KS, int KC>
int launch_ws(const ConvArgs& a, hipStream_t s) {
  constexpr int PAD = KS / 2;
  constexpr int HP = (TW + 2 * PAD) * (TH + 2 * PAD);
  constexpr int TN = WN * NI * 32;
  MfmaParams p;
  p.x = a.x; p.mean = a.mean; p.rstd = a.rstd; p.gamma = a.gamma; p.beta = a.beta;
  p.w = a.wt; p.bias = a.bias; p.res = a.res; p.y = a.y;
  p.silu = a.silu; p.groups = a.groups; p.norm = a.mean != nullptr;
  p.n = a.n; p.h = a.h; p.w_out = a.w; p.cin = a.cin; p.cout = a.cout; p.upsample = a.upsample;
  p.tiles_x = (a.w + TW - 1) / TW; p.tiles_y = (a.h + TH - 1) / TH; p.ntiles = (a.cout + TN - 1) / TN;
  p.total = p.tiles_x * p.tiles_y * p.ntiles * a.n;
  p.cin_blocks = packed_cin_blocks(a.cin); p.cout_blocks = packed_cout_blocks(a.cout); p.dbg = g_dbg; p.y_nchw = a.y_nchw;
  const size_t smem = (size_t)2 * HP * (KC + 8) * 2 + (size_t)4 * 32 * (NI * 32 + 4) * sizeof(float);
  auto kern = conv_ws_kernel<T, TO, TH, TW, WM, WN, NI, KS, KC>;
  static bool attr_set = false;
  if (!attr_set) {
    WMDEC_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    attr_set = true;
  }
  int nwg = p.total < 256 ? (p.total + 7) / 8 * 8 : 256;
  hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(512), smem, s, p);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
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
  p.tiles_x = (a.w + TW - 1) / TW; p.tiles_y = (a.h + TH - 1) / TH; p.ntiles = (a.cout + TN - 1) / TN;
  p.total = p.tiles_x * p.tiles_y * p.ntiles * a.n;
  p.cin_blocks = packed_cin_blocks(a.cin); p.cout_blocks = packed_cout_blocks(a.cout); p.dbg = g_dbg; p.y_nchw = a.y_nchw;
  size_t smem = (((size_t)HP * (KC + 8) * 2 + 15) & ~(size_t)15) + (size_t)a.cin * sizeof(float2);
  const size_t patch = (size_t)4 * 32 * (NI * 32 + 4) * sizeof(float);   // epilogue patches of the four wavefronts
  if (smem < patch) smem = patch;
  auto kern = conv_mfma_kernel<T, TO, TH, TW, WM, WN, NI, KS, KC>;
  static bool attr_set = false;   // per instantiation
  if (!attr_set) {
    WMDEC_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024));   // two workgroups per compute unit
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)p.total), dim3(256), smem, s, p);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

template <typename T, typename TO, int KS>
int launch_shape(const ConvArgs& a, hipStream_t s) {
  if constexpr (KS == 3) {
    if (g_variant == 1 && a.cout % 128 == 0) return launch_ws<T, TO, 8, 32, 2, 2, 2, KS, 32>(a, s);
  }
  // tile choice: 256 pixels x 128 channels when that still gives every compute unit work, else smaller
  const long px = (long)a.n * a.h * a.w;
  if (a.cout <= 32) return launch_cfg<T, TO, 8, 32, 4, 1, 1, KS, 32>(a, s);   // few output channels (the frame): one 32-wide tile
  if (g_tile >= 0) {   // tile sweep
    const bool n128 = a.cout % 128 == 0;
    switch (g_tile) {
      case 0: if (n128) return launch_cfg<T, TO, 8, 32, 2, 2, 2, KS, 32>(a, s); break;   // 256 x 128
      case 1: if (n128) return launch_cfg<T, TO, 4, 32, 2, 2, 2, KS, 32>(a, s); break;   // 128 x 128
      case 2: return launch_cfg<T, TO, 4, 32, 4, 1, 2, KS, 32>(a, s);                    // 128 x 64
      case 3: return launch_cfg<T, TO, 8, 32, 4, 1, 2, KS, 32>(a, s);                    // 256 x 64
      case 4: if (n128) return launch_cfg<T, TO, 8, 16, 2, 2, 2, KS, 32>(a, s); break;   // 128 x 128, 8x16 patch
      case 5: if (n128) return launch_cfg<T, TO, 16, 16, 2, 2, 2, KS, 32>(a, s); break;  // 256 x 128, 16x16 patch
      case 6: return launch_cfg<T, TO, 8, 16, 4, 1, 2, KS, 32>(a, s);                    // 128 x 64, 8x16 patch
      case 7: if (n128) return launch_cfg<T, TO, 8, 32, 2, 2, 2, KS, 64>(a, s); break;   // 256 x 128, 64-channel chunks
      default: break;
    }
  }
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
  if (a.x_nchw) return false;
  if (a.y_nchw && !(a.cout <= 32 && a.y_dtype == WMDEC_F32 && !a.res)) return false;
  if (a.cin % 32 != 0) return false;
  if (a.cout % 64 != 0 && !(a.y_nchw && a.cout <= 32)) return false;
  if (a.cin > 4096) return false;   // scale/shift table lives in LDS
  if (a.ksize != 1 && a.ksize != 3) return false;
  return true;
}

int launch_conv_mfma(const ConvArgs& a, hipStream_t s) {
  static bool init = false;
  if (!init) { const char* e = getenv("WMDEC_CONV_VARIANT"); g_variant = e ? atoi(e) : 0; const char* d = getenv("WMDEC_CONV_DBG"); g_dbg = d ? atoi(d) : 0; const char* t = getenv("WMDEC_CONV_TILE"); g_tile = t ? atoi(t) : -1; init = true; }
  return a.op_dtype == WMDEC_BF16 ? launch_type<bf16_t>(a, s) : launch_type<f16_t>(a, s);
}

}  // namespace wmdec
