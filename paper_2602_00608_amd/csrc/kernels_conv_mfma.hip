// Implicit-GEMM convolution on the gfx950 matrix cores.
//
// GEMM view: M = output pixels, N = output channels, K = taps * C_in.
// One workgroup (4 wavefronts) owns a TH x TW patch of output pixels and TN
// output channels.  Per chunk of KC input channels it stages the patch plus its
// one-pixel halo into LDS -- GroupNorm scale/shift and SiLU are applied there,
// once per element, and positions outside the image are zeros -- and then sweeps
// the nine taps over that tile: the A operand of every MFMA is a 16-byte LDS read
// at a tap-dependent constant offset, the B operand (weights) is loaded straight
// from the L2-resident packed weights, where every 32(co) x 16(ci) fragment is
// 1 KiB in lane order, so a wavefront's load is one contiguous KiB.
// Accumulators stay in registers for the whole K loop; bias, residual, the single
// rounding to the storage type and the GroupNorm moments of the output happen in
// the epilogue.
// The staged tile is double-buffered: the raw vectors of chunk c+2 are loaded
// right after the sweep of chunk c, and chunk c+1 is activated and stored into
// the other buffer in compile-time slots inside the sweep of chunk c, with one
// workgroup barrier per chunk.  Two or three workgroups fit on a compute unit, so
// the prologue and epilogue of one overlap the sweeps of the others.
// A nearest-2x upsample in front of the convolution is either folded into the
// staging address (bf16) or, in f16, removed algebraically: the phase mode
// computes each of the four output phases as a 2x2 convolution on the input grid.
#include <stdio.h>

#include <mutex>
#include <type_traits>
#include <utility>

#include "mfma.hpp"
#include "moments.hpp"
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
  int w_bytes;                   // size of the packed weights the kernel may read
  int y_nchw;                    // 1: y is planar [n][cout][h][w] (the frame), else NHWC
  Moments* stats;                // non-null: moments of y per (sample, group, slot); slot = spatial tile * WM + wave row
  int stats_cpg, stats_groups, stats_slots;
  // Statistics hand-over without a merge launch.  rows_out: the last workgroup of every (sample, tile row, channel
  // tile) merges that row's triples into one triple per group, [n][stats_groups][tiles_y]; tickets: one counter per
  // (sample, tile row, channel tile), zero before the launch and zero again after it.  rows_in: the statistics of x
  // arrive as such row triples, [n][groups][rows_in_count], and are merged while the scale/shift table is built.
  Moments* rows_out; unsigned* tickets;
  const Moments* rows_in; int rows_in_count; float eps;
  // 1x1 shortcut folded into the contraction (3x3 only): y += W2 * x2 + bias2, x2 [n,h,w,cin2] taken as stored
  const void* x2; const void* w2; const float* bias2;
  int cin2, w2_bytes;
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
// floats of the wavefront-private epilogue patch: 32 padded rows, and at least the 64 x 8 four-float entries
// that the statistics reduction parks there
constexpr int patch_floats(int ni) { return 32 * (ni * 32 + 4) > 2048 ? 32 * (ni * 32 + 4) : 2048; }

template <typename T, typename TO, int MI, int NI, int MTW, int MTH, int MT_PER_ROW, bool RES>
__device__ __forceinline__ void epilogue_store(const f32x16 (&acc)[MI][NI], float* lds, int lane, int mt0, int ty0,
                                               int tx0, int co_w, const float* bias, const float* bias2, const T* rin, TO* yout, int h,
                                               int w_out, int cout, bool nchw, Moments* stats, int cpg, int stats_stride,
                                               int osc = 1, int oy_off = 0, int ox_off = 0) {
  // tile pixel (ty, tx) is output pixel (ty * osc + oy_off, tx * osc + ox_off): osc = 2 when the tile lives on the
  // low-resolution grid of a phase-decomposed upsampling convolution
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
      if (oy < h && ox < w_out) {
        for (int c = lk; c < NI * 32 && co_w + c < cout; c += 2) {
          const float v = lds[lm * RW + c] + (bias ? bias[co_w + c] : 0.f) + (bias2 ? bias2[co_w + c] : 0.f);
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
  for (int e = 0; e < 8; ++e) bv[e] = (bias ? bias[co_w + cvec * 8 + e] : 0.f) + (bias2 ? bias2[co_w + cvec * 8 + e] : 0.f);
  // 32-bit element offset of this lane's vector in M tile mi, row j (or -1 outside the image)
  auto vec_off = [&](int mi, int j) -> int {
    const int mt = mt0 + mi;
    const int pi = prow + j * (64 / (NI * 4));
    const int oy = (ty0 + (mt / MT_PER_ROW) * MTH + pi / MTW) * osc + oy_off;
    const int ox = (tx0 + (mt % MT_PER_ROW) * MTW + pi % MTW) * osc + ox_off;
    return (oy < h && ox < w_out) ? (oy * w_out + ox) * cout + co_w + cvec * 8 : -1;   // < 2^30 elements (checked on the host)
  };
  // residual vectors are fetched two M tiles ahead (unconditional loads, clamped to element 0 outside the
  // image) so that their latency hides behind the LDS round trips of the tiles before
  constexpr int RD = 2;
  u32x4 rv[RD][VPL];
  if constexpr (RES) {
#pragma unroll
    for (int mi = 0; mi < RD && mi < MI; ++mi)
#pragma unroll
      for (int j = 0; j < VPL; ++j) rv[mi][j] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(rin) + (unsigned)(max(vec_off(mi, j), 0) * (int)sizeof(T)));
  }
  // moments of the values this lane stores, per channel of its octet (shifted sums: the shift is the first value)
  float st_shift[8], st_s[8], st_q[8], st_n = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) { st_shift[e] = 0.f; st_s[e] = 0.f; st_q[e] = 0.f; }
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) lds[(8 * (r / 4) + 4 * lk + (r % 4)) * RW + ni * 32 + lm] = acc[mi][ni][r];
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int pi = prow + j * (64 / (NI * 4));
      const int off = vec_off(mi, j);
      const f32x4 lo = *reinterpret_cast<const f32x4*>(lds + pi * RW + cvec * 8);
      const f32x4 hi = *reinterpret_cast<const f32x4*>(lds + pi * RW + cvec * 8 + 4);
      float v[8] = {lo[0] + bv[0], lo[1] + bv[1], lo[2] + bv[2], lo[3] + bv[3],
                    hi[0] + bv[4], hi[1] + bv[5], hi[2] + bv[6], hi[3] + bv[7]};
      if constexpr (RES) {
        float rf[8];
        unpack8<T>(rv[mi % RD][j], rf);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += rf[e];
        if (mi + RD < MI)
          rv[mi % RD][j] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(rin) + (unsigned)(max(vec_off(mi + RD, j), 0) * (int)sizeof(T)));
      }
      // the stored vector; the moments are those of the values as stored (after the rounding to the storage
      // type), which is what the consumer of the tensor normalises
      u32x4 packed;
      if constexpr (sizeof(TO) == 2) {
        packed = u32x4{pack2<T>(v[0], v[1]), pack2<T>(v[2], v[3]), pack2<T>(v[4], v[5]), pack2<T>(v[6], v[7])};
      }
      if (stats && off >= 0) {
        float sv[8];
        if constexpr (sizeof(TO) == 2) {
          unpack8<T>(packed, sv);
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) sv[e] = v[e];
        }
        if (st_n == 0.f) {
#pragma unroll
          for (int e = 0; e < 8; ++e) st_shift[e] = sv[e];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float dv = sv[e] - st_shift[e]; st_s[e] += dv; st_q[e] = fmaf(dv, dv, st_q[e]); }
        st_n += 1.f;
      }
      if (off >= 0) {
        TO* dst = reinterpret_cast<TO*>(reinterpret_cast<char*>(yout) + (unsigned)(off * (int)sizeof(TO)));
        if constexpr (sizeof(TO) == 4) {
          reinterpret_cast<f32x4*>(dst)[0] = f32x4{v[0], v[1], v[2], v[3]};
          reinterpret_cast<f32x4*>(dst)[1] = f32x4{v[4], v[5], v[6], v[7]};
        } else {
          *reinterpret_cast<u32x4*>(dst) = packed;
        }
      }
    }
  }
  if (stats) {
    // lane -> wavefront: every lane parks its 8 channels' (count, shift, sum, sum of squares) in the LDS patch;
    // lane L then owns channel L of the wavefront's run, re-centres the entries of the lanes that held that
    // channel (they differ in the pixel rows they read back) on one shift and adds them in a fixed order.
    constexpr int CV = NI * 4;                 // octets per row of the patch
    constexpr int ROWS = 64 / CV;              // lanes per octet
    f32x4* park = reinterpret_cast<f32x4*>(lds);
#pragma unroll
    for (int e = 0; e < 8; ++e) park[lane * 8 + e] = f32x4{st_n, st_shift[e], st_s[e], st_q[e]};
    Moments m{0.f, 0.f, 0.f};
    if (lane < CV * 8) {
      float n0 = 0.f, a0 = 0.f, s0 = 0.f, q0 = 0.f;
#pragma unroll
      for (int r = 0; r < ROWS; ++r) {
        const f32x4 en = park[r * (CV * 8) + lane];     // (row r, octet lane / 8, channel lane % 8)
        if (en[0] > 0.f) {
          if (n0 == 0.f) a0 = en[1];
          const float d = en[1] - a0;
          s0 += en[2] + en[0] * d;
          q0 += en[3] + 2.f * d * en[2] + en[0] * d * d;
          n0 += en[0];
        }
      }
      if (n0 > 0.f) { const float ds = s0 / n0; m.n = n0; m.mean = a0 + ds; m.m2 = fmaxf(q0 - s0 * ds, 0.f); }
    }
    // channels of one group are cpg consecutive lanes
    m = merge_to_first(m, lane, cpg);
    // (device-scope stores: another workgroup of this launch may merge them, see the row hand-over in the kernel)
    if (lane < CV * 8 && (lane & (cpg - 1)) == 0) store_device(stats + (size_t)((co_w + lane) / cpg) * stats_stride, m);
  }
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <int N, typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl<N>(f, std::make_integer_sequence<int, N>{}); }

// Ring length of the weight-fragment prefetch: it must divide the k-steps of a chunk so that the ring
// position is the same at every chunk start.
// It is as long as the register budget of the tile allows (`room`: accumulator tiles per wavefront): the fragments
// come from the L2, whose latency is several k-steps.  The 256-pixel tiles, at the 256-register limit, take the
// short ring and spend the registers on the activation-table prefetch instead (measured: +1.5 to 2 %).
constexpr int prefetch_ring(int steps, int room) {
  if (room > 4 && steps % 3 == 0) return 3;
  if (steps % 6 == 0) return 6;
  return steps % 3 == 0 ? 3 : (steps % 4 == 0 ? 4 : 2);
}

// silu(t) from u = -log2(e) * t (see the scale/shift table)
__device__ __forceinline__ float silu_from_scaled(float u) {
  constexpr float k = -1.4426950408889634f;
  return u * __builtin_amdgcn_rcpf(fmaf(__builtin_amdgcn_exp2f(u), k, k));
}

// One weight fragment (1 KiB, a lane's 16 bytes at lane16 = 16 * lane) at byte offset `off` of the packed weights.
// A buffer load takes the wave-uniform offset in a scalar register, so the address costs no vector-ALU work
// (a global load would add the 64-bit base per fragment), and offsets past the blob read zeros instead of faulting.
__device__ __forceinline__ u32x4 load_fragment(__amdgpu_buffer_rsrc_t rsrc, int lane16, int off) {
  return __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane16, off, 0);
}

// MFMA work of one staged chunk: STEPS = taps * KC/16 k-steps, each MI x NI 32x32x16 MFMAs.
// Weight fragments are fetched D-1 steps ahead (bq is a ring that persists across chunks: on
// entry it holds steps 0..D-2 of this chunk, on exit steps 0..D-2 of the chunk at `bnext`).
// The A fragment of an M tile is refreshed in place for the next step right after the MFMAs
// that consumed it, which gives the LDS read the rest of the step to land.  The scheduling
// barriers pin that order: without them the compiler sinks every load to just before its use
// and each k-step pays a full memory latency.
// VALU_PER_MFMA: -1 pins the order as written (slot hook after the MFMAs of an M tile); >= 0 asks the scheduler to
// interleave that many vector-ALU instructions behind every MFMA of a k-step.
// AD: how many k-steps ahead the A fragments are read (1 or 2).  One step is MI - 1 MFMAs of slack, about the LDS
// latency: enough where other wavefronts of the SIMD fill the gaps, too little for a wavefront that is alone on it.
template <typename T, int MI, int NI, int KS, int KC, int ROW, int PS, int D, bool SLICED, int VALU_PER_MFMA, typename Slice, int AD = 1>
__device__ __forceinline__ void mfma_chunk(const T* buf, const int (&a_off)[MI], __amdgpu_buffer_rsrc_t wrsrc, int bcur, int bnext,
                                           int tap_stride, int kk_stride, int lane16, u32x4 (&bq)[D][NI],
                                           f32x16 (&acc)[MI][NI], Slice&& slice) {
  constexpr int KK = KC / 16, STEPS = KS * KS * KK;
  static_assert(AD == 1 || AD == 2, "A fragments one or two k-steps ahead");
  u32x4 af[AD][MI];   // af[s % AD]: fragments of k-step s
#pragma unroll
  for (int a = 0; a < AD && a < STEPS; ++a) {
    const int tap = a / KK, kk = a % KK;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) af[a][mi] = *reinterpret_cast<const u32x4*>(buf + a_off[mi] + (tap / KS) * ROW + (tap % KS) * PS + kk * 16);
  }
  // one k-step; the slot hook runs after the MFMAs of every M tile so that its vector-ALU work issues
  // while those MFMAs occupy the matrix pipe
  auto step = [&](auto s_c) {
    constexpr int s = decltype(s_c)::value;
    {
      constexpr int sp = s + D - 1;
      const int src = sp < STEPS ? bcur : bnext;
      constexpr int spp = sp < STEPS ? sp : sp - STEPS;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        bq[sp % D][ni] = load_fragment(wrsrc, lane16, src + (spp / KK) * tap_stride + (spp % KK) * kk_stride + ni * 1024);
    }
    __builtin_amdgcn_sched_barrier(0);
    auto tile = [&](auto mi_c) {
      constexpr int mi = decltype(mi_c)::value;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = Mma<T>::m32(af[s % AD][mi], bq[s % D][ni], acc[mi][ni]);
      if constexpr (s + AD < STEPS) {
        constexpr int tap = (s + AD) / KK, kk = (s + AD) % KK;
        af[s % AD][mi] = *reinterpret_cast<const u32x4*>(buf + a_off[mi] + (tap / KS) * ROW + (tap % KS) * PS + kk * 16);
      }
      if constexpr (SLICED) slice(std::integral_constant<int, s * MI + mi>{});
      if constexpr (VALU_PER_MFMA < 0) __builtin_amdgcn_sched_barrier(0);
    };
    static_for<MI>(tile);
    if constexpr (VALU_PER_MFMA >= 0) {
      // The whole k-step is one scheduling region; spell out the issue order inside it: after every MFMA the A
      // refresh that belongs to it (one LDS read per NI MFMAs) and an equal share of the step's activation work,
      // so that each MFMA's 32 cycles in the matrix pipe cover vector-ALU work instead of the next MFMA's wait.
      static_for<MI * NI>([&](auto j_c) {
        constexpr int j = decltype(j_c)::value;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one MFMA
        if constexpr (j % NI == NI - 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
        if constexpr (VALU_PER_MFMA > 0) __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER_MFMA, 0);
      });
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  static_for<STEPS>(step);
}

// ACT: what happens to an input element on its way into LDS: 0 nothing, 1 scale/shift, 2 scale/shift + SiLU
// PH: phase-decomposed nearest-2x upsampling convolution.  The tile lives on the low-resolution input grid; wavefront
// w computes output phase (py, px) = (w >> 1, w & 1) of all its pixels, i.e. output pixels (2i + py, 2j + px), as a
// 2x2 convolution over input rows i + py - 1 .. i + py and columns j + px - 1 .. j + px with the phase's pre-summed
// weights (taps 4 * w .. 4 * w + 3 of the 16-tap phase pack): 4/9 of the multiplications of the 3x3 form.
constexpr int wave_m_tiles(int th, int tw, int wm, bool ph) { return ph ? th * tw / 32 : th * tw / 32 / wm; }
// Workgroups per compute unit the register budget is sized for: three for the small accumulator tiles, except the
// 2x2-wavefront 128x128 shape, which is only picked for layers with at most two workgroups per compute unit and
// uses the registers for a longer prefetch instead.
constexpr int resident_workgroups(int acc_tiles, int wm, int wn) {
  return wm * wn == 8 ? 1 : (acc_tiles <= 4 && !(wm == 2 && wn == 2) ? 3 : 2);
}

// LDS layout of a staged tile (elements of the 16-bit type): pixel (hy, hx) of the halo patch sits at hy * ROW + hx * PS.
// PS = KC + 8: the 16-byte pad makes the 16 lanes that the LDS serves per cycle (consecutive pixels of a row, 16 bytes
// each) fall on 64 distinct banks.  A 32-pixel M tile that spans two patch rows (16-pixel-wide patches) has lanes i and
// i + 16 one row apart; the LDS only runs at full rate when such lane pairs are a multiple of 256 bytes apart (measured:
// any other row stride costs a second pass per read), so for those patches the row stride is rounded up to 256 bytes.
// One pixel slot behind the patch is spare: vectors that lie outside the image (or past the patch) are stored there,
// where no MFMA reads them.
constexpr int tile_row_elems(int tw, int pad, int kc) {
  const int raw = (tw + 2 * pad) * (kc + 8);
  return tw < 32 ? (raw * 2 + 255) / 256 * 128 : raw;
}
constexpr int tile_buf_elems(int th, int tw, int pad, int kc) { return (th + 2 * pad) * tile_row_elems(tw, pad, kc) + (kc + 8); }

// RING: 0 = weight-fragment ring sized by prefetch_ring; otherwise its length in k-steps (a divisor of the k-steps of
// a chunk).  The whole-chunk ring is for launches that leave a compute unit at most two workgroups: there a wavefront
// is alone on its SIMD, nothing else hides the latency of weights that come from beyond the L2 (every layer's weights
// are new to the L2 inside a decoder run), and the registers of the third workgroup are free for it.
template <typename T, typename TO, int TH, int TW, int WM, int WN, int NI, int KS, int KC, int ACT, bool PH = false, int RING = 0>
__global__ __launch_bounds__(64 * WM * WN, RING > 6 ? 2 : resident_workgroups(wave_m_tiles(TH, TW, WM, PH) * NI, WM, WN))
void conv_mfma_kernel(MfmaParams p) {
  static_assert(WM * WN == 4 || WM * WN == 8, "four or eight wavefronts");
  constexpr int NT = 64 * WM * WN;               // threads of the workgroup
  static_assert(!PH || (KS == 3 && WM == 4 && WN == 1), "phase mode: one wavefront per phase");
  constexpr int MI = wave_m_tiles(TH, TW, WM, PH);   // 32-pixel M tiles per wavefront
  constexpr int KT = PH ? 2 : KS;                // taps per dimension a wavefront sweeps
  constexpr int PAD = PH ? 1 : KS / 2;
  constexpr int HW_ = TW + 2 * PAD, HH_ = TH + 2 * PAD, HP = HW_ * HH_;
  constexpr int PS = KC + 8;                     // LDS pixel stride in elements (+16 B: conflict-free 16-byte reads)
  constexpr int MTW = TW < 32 ? TW : 32, MTH = 32 / MTW, MT_PER_ROW = TW / MTW;
  constexpr int TN = WN * NI * 32;
  constexpr int VPP = KC / 8;                    // 16-byte vectors per pixel per chunk
  constexpr int NV = (HP * VPP + NT - 1) / NT;   // vectors a thread stages per chunk
  constexpr int ROW = tile_row_elems(TW, PAD, KC);       // LDS row stride of the staged tile, elements
  constexpr int BUF = tile_buf_elems(TH, TW, PAD, KC);   // elements of one staged tile: the halo patch plus the spare slot
  constexpr int SPARE = HH_ * ROW;                       // element offset of the spare pixel slot
  constexpr int STEPS = KT * KT * (KC / 16), SLOTS = STEPS * MI;
  constexpr bool SLICED = KS == 3;               // activation of the next chunk is sliced into the MFMA sweep
  static_assert(NT % VPP == 0, "a thread keeps one channel octet");

  extern __shared__ __align__(16) unsigned char smem[];
  T* s_a = reinterpret_cast<T*>(smem);                                          // [2][BUF]
  float2* s_ab = reinterpret_cast<float2*>(smem + ((2 * BUF * 2 + 15) & ~15));  // [cin] (scale, shift)

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform: keeps the per-wave addresses scalar
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
  const int h_t = PH ? h_in : p.h, w_t = PH ? w_in : p.w_out;   // the grid the tiles live on

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
    const int mt = PH ? mi : wm * MI + mi;
    const int ty = (mt / MT_PER_ROW) * MTH + lm / MTW, tx = (mt % MT_PER_ROW) * MTW + lm % MTW;
    a_off[mi] = ty * ROW + tx * PS + 8 * lk + (PH ? (wave >> 1) * ROW + (wave & 1) * PS : 0);
  }
  constexpr int KK = KC / 16;
  constexpr int D = RING > 0 ? RING : prefetch_ring(KT * KT * KK, MI * NI);   // weight fragments are fetched D-1 k-steps ahead
  static_assert((KT * KT * KK) % D == 0, "the ring position must be the same at every chunk start");
  const int tap_stride = p.cin_blocks * p.cout_blocks * 1024, kk_stride = p.cout_blocks * 1024;   // bytes
  // byte offset of this wavefront's fragment column (wave-uniform; the lane's 16 bytes are added by the load)
  const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w), 0, p.w_bytes, 0x00020000);
  const int wcol = ((co0 >> 5) + wn * NI) * 1024 + (PH ? wave * 4 * tap_stride : 0);
  const int lane16 = lane * 16;
  u32x4 bq[D][NI];
#pragma unroll
  for (int sp = 0; sp < D - 1; ++sp)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) bq[sp][ni] = load_fragment(wrsrc, lane16, wcol + (sp / KK) * tap_stride + (sp % KK) * kk_stride + ni * 1024);

  // ---- staging: a thread owns NV (pixel, channel-octet) vectors of the halo tile; the octet is the same for all
  const int cvec = tid % VPP;
  const char* xin = reinterpret_cast<const char*>(p.x) + (size_t)n * h_in * w_in * p.cin * sizeof(T);   // uniform base
  // Zero padding without per-element work: a vector outside the image is loaded from pixel 0 (a load under a lane
  // mask would make the compiler wait for it at the end of the branch), activated like any other, and stored to
  // the spare pixel slot behind the patch; its real slot is zeroed once, here, in both buffers.  A 1x1 convolution
  // has no halo: what its out-of-image pixels hold only reaches outputs that are never stored.
  int src_off[NV];          // byte offset of the vector in x (chunk 0)
  int dst_off[NV];          // element offset of its slot in a staged tile
  int src_pix[NV];          // index of its source pixel in the sample (0 outside the image); only the shortcut phase reads it
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int v = tid + i * NT;
    const int hp = v / VPP;
    const int hy = hp / HW_, hx = hp % HW_;
    const int gy = ty0 + hy - PAD, gx = tx0 + hx - PAD;
    const bool in_patch = v < HP * VPP;
    const bool inside = in_patch && gy >= 0 && gy < h_t && gx >= 0 && gx < w_t;
    src_off[i] = 0;
    src_pix[i] = 0;
    if (inside) {
      const int sy = (!PH && p.upsample) ? gy >> 1 : gy, sx = (!PH && p.upsample) ? gx >> 1 : gx;
      src_pix[i] = sy * w_in + sx;
      src_off[i] = (src_pix[i] * p.cin + cvec * 8) * (int)sizeof(T);
    }
    const bool keep = KS == 1 ? in_patch : inside;
    dst_off[i] = (keep ? hy * ROW + hx * PS : SPARE) + cvec * 8;
    if (KS != 1 && in_patch && !inside) {
      *reinterpret_cast<u32x4*>(s_a + hy * ROW + hx * PS + cvec * 8) = u32x4{0u, 0u, 0u, 0u};
      *reinterpret_cast<u32x4*>(s_a + BUF + hy * ROW + hx * PS + cvec * 8) = u32x4{0u, 0u, 0u, 0u};
    }
  }
  // One register set of raw vectors.  The loads of chunk k+1 are issued right after the MFMA sweep of chunk
  // k-1 (vector-memory loads return in order, so weight-fragment loads issued behind them cannot be consumed
  // before they have landed: the workgroup barrier and the first third of the next sweep cover that), and the
  // vectors are activated and stored into the other LDS buffer in the last two thirds of the sweep of chunk k,
  // a few elements after every M tile's MFMAs, so that this vector-ALU work overlaps the matrix pipe instead of
  // forming a phase of its own.
  u32x4 raw[NV];
  auto issue = [&](int chunk) {
    const int cb = min(chunk, p.cin / KC - 1) * KC * (int)sizeof(T);   // past the last chunk: a harmless reload
#pragma unroll
    for (int i = 0; i < NV; ++i) raw[i] = *reinterpret_cast<const u32x4*>(xin + (unsigned)(src_off[i] + cb));
  };
  // word (two channels) of a staged vector: scale/shift (+ SiLU) with the table entries ab = (a0, b0, a1, b1)
  auto activate_with = [&](uint32_t wv, const f32x4& ab) -> uint32_t {
    if constexpr (ACT > 0) {
      float f0 = fmaf(unpack_lo<T>(wv), ab[0], ab[1]), f1 = fmaf(unpack_hi<T>(wv), ab[2], ab[3]);
      if constexpr (ACT == 2) { f0 = silu_from_scaled(f0); f1 = silu_from_scaled(f1); }
      wv = pack2<T>(f0, f1);
    }
    return wv;
  };
  // table entries of word `part` of this thread's channel octet in the chunk that starts at channel c0
  auto table_entry = [&](int part, int c0) -> f32x4 {
    if constexpr (ACT > 0) return *reinterpret_cast<const f32x4*>(s_ab + c0 + cvec * 8 + 2 * part);
    else return f32x4{0.f, 0.f, 0.f, 0.f};
  };
  auto activate_word = [&](uint32_t wv, int i, int part, int c0) -> uint32_t {
    (void)i;
    return activate_with(wv, table_entry(part, c0));
  };
  auto store_vec = [&](int i, T* buf) { *reinterpret_cast<u32x4*>(buf + dst_off[i]) = raw[i]; };
  auto activate_all = [&](int c0, T* buf) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      raw[i] = u32x4{activate_word(raw[i].x, i, 0, c0), activate_word(raw[i].y, i, 1, c0),
                     activate_word(raw[i].z, i, 2, c0), activate_word(raw[i].w, i, 3, c0)};
      store_vec(i, buf);
    }
  };
  const int nchunks = p.cin / KC;
  // vector-ALU instructions of the activation per MFMA of an active k-step (8 per element with SiLU, 3 without),
  // one less than the average so that the tail of a word does not delay the next k-step; the 256-pixel tiles keep
  // the order as written (spreading measured 0 to -4 % there, +1 to +2 % on the small tiles)
  constexpr int SPREAD_AVG = (NV * 8 * (ACT == 2 ? 8 : 3) + (SLOTS - SLOTS / 3) * NI - 1) / ((SLOTS - SLOTS / 3) * NI);
  constexpr int SPREAD = (ACT == 0 || MI * NI > 4) ? -1 : (SPREAD_AVG > 1 ? SPREAD_AVG - 1 : 1);
  f32x4 abv[2];   // table entries of the part being activated and of the next one (sliced activation)

  // ---- shortcut phase (3x3 kernels with a second input): acc = W2 * x2 over the tile's own pixels, a 1x1
  // contraction over cin2 channels taken as stored (no normalisation).  Chunks of KC channels go through the same
  // two LDS buffers with the tile's halo layout (only the centre tap is read), loads two chunks ahead; the main
  // loop below then adds the 3x3 contraction to the same accumulators, so the shortcut tensor never exists in
  // memory and the epilogue adds both biases.
  if constexpr (KS == 3 && !PH) {
    if (p.x2) {
      const char* xin2 = reinterpret_cast<const char*>(p.x2) + (size_t)n * p.h * p.w_out * p.cin2 * sizeof(T);
      const int nch2 = p.cin2 / KC;
      auto issue2 = [&](int chunk) {
        const int cb = min(chunk, nch2 - 1) * KC * (int)sizeof(T);
#pragma unroll
        for (int i = 0; i < NV; ++i)
          raw[i] = *reinterpret_cast<const u32x4*>(xin2 + (unsigned)((src_pix[i] * p.cin2 + cvec * 8) * (int)sizeof(T) + cb));
      };
      auto store_all = [&](T* buf) {
#pragma unroll
        for (int i = 0; i < NV; ++i) store_vec(i, buf);
      };
      int a_ctr[MI];   // centre tap of the halo patch
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) a_ctr[mi] = a_off[mi] + PAD * ROW + PAD * PS;
      constexpr int D2 = 2;
      const __amdgpu_buffer_rsrc_t wrsrc2 = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.w2), 0, p.w2_bytes, 0x00020000);
      const int wcol2 = ((co0 >> 5) + wn * NI) * 1024;
      u32x4 bq2[D2][NI];
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) bq2[0][ni] = load_fragment(wrsrc2, lane16, wcol2 + ni * 1024);
      issue2(0);
      store_all(s_a);
      issue2(1);
      __syncthreads();
      auto none = [](auto) {};
      for (int c = 0; c < nch2; ++c) {
        const int bcur = wcol2 + c * KK * kk_stride;
        const int bnext = c + 1 < nch2 ? bcur + KK * kk_stride : bcur;
        mfma_chunk<T, MI, NI, 1, KC, ROW, PS, D2, false, -1>(s_a + (c & 1) * BUF, a_ctr, wrsrc2, bcur, bnext, 0, kk_stride, lane16, bq2, acc, none);
        if (c + 1 < nch2) store_all(s_a + ((c + 1) & 1) * BUF);
        issue2(c + 2);
        __syncthreads();
      }
    }
  }

  issue(0);
  // (built behind the first chunk's loads, so that its own global loads overlap them)
  // per-channel scale/shift table: a = gamma*rstd, b = beta - mean*a.  With SiLU the table holds -log2(e) * (a, b):
  // the staged value is u = -log2(e) * t, from which silu(t) = t / (1 + 2^u) = u / (-log2(e) - log2(e) * 2^u) takes
  // one exp2, one fma, one reciprocal and one multiply
  if constexpr (ACT > 0) {
    const int cpg = p.cin / p.groups;
    const float k = ACT == 2 ? -1.4426950408889634f : 1.0f;
    if (p.rows_in) {
      // mean / rstd of every group from the row triples its producer left: eight lanes per group take the rows
      // round-robin in order, then a fixed butterfly; (mean, rstd) parked behind the table
      float2* s_stat = s_ab + p.cin;
      // Launches that leave a wavefront alone on its SIMD (RING): gamma / beta of this thread's first two table
      // entries are requested together with the triples, one memory round trip less in front of the first chunk
      // (elsewhere other workgroups cover that latency and the registers are better left to the main loop).
      constexpr int PRE = RING > 6 ? 2 : 0;
      float gpre[2] = {0.f, 0.f}, bpre[2] = {0.f, 0.f};
#pragma unroll
      for (int j = 0; j < PRE; ++j) {
        const int c = min(tid + j * NT, p.cin - 1);
        gpre[j] = p.gamma[c]; bpre[j] = p.beta[c];
      }
      const int sub = tid & 7;
      for (int g = tid >> 3; g < p.groups; g += NT / 8) {
        const Moments* row = p.rows_in + (size_t)(n * p.groups + g) * p.rows_in_count;
        Moments m{0.f, 0.f, 0.f};
        for (int r0 = sub; r0 < p.rows_in_count; r0 += 64) {   // eight loads in flight per lane before the first merge
          Moments t[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            const int r = r0 + 8 * k;
            t[k] = row[min(r, p.rows_in_count - 1)];
            if (r >= p.rows_in_count) t[k].n = 0.f;
          }
#pragma unroll
          for (int k = 0; k < 8; ++k) m = merge(m, t[k]);
        }
        m = merge_to_first(m, lane, 8);
        if (sub == 0) s_stat[g] = make_float2(m.mean, 1.0f / sqrtf(m.m2 / m.n + p.eps));
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < PRE; ++j) {
        const int c = tid + j * NT;
        if (c < p.cin) {
          const float2 st = s_stat[c / cpg];
          const float a = gpre[j] * st.y;
          s_ab[c] = make_float2(k * a, k * (bpre[j] - st.x * a));
        }
      }
      for (int c = tid + PRE * NT; c < p.cin; c += NT) {
        const float2 st = s_stat[c / cpg];
        const float a = p.gamma[c] * st.y;
        s_ab[c] = make_float2(k * a, k * (p.beta[c] - st.x * a));
      }
    } else {
      for (int c = tid; c < p.cin; c += NT) {
        const int g = c / cpg;
        const float a = p.gamma[c] * p.rstd[n * p.groups + g];
        s_ab[c] = make_float2(k * a, k * (p.beta[c] - p.mean[n * p.groups + g] * a));
      }
    }
  }
  __syncthreads();            // scale/shift table complete
  activate_all(0, s_a);
  issue(1);
  __syncthreads();
  for (int c = 0; c < nchunks; ++c) {
    const bool more = c + 1 < nchunks;
    const int bcur = wcol + c * KK * kk_stride;
    const int bnext = more ? bcur + KK * kk_stride : bcur;
    const T* buf = s_a + (c & 1) * BUF;
    T* nbuf = s_a + ((c + 1) & 1) * BUF;
    const int c0n = (c + 1) * KC;
    if constexpr (SLICED) {
      // Slots FIRST .. SLOTS-1 share the NV*4 words of the next chunk evenly.  All vectors of a thread hold the same
      // channel octet, so the words are taken part by part (word `part` of every vector, then the next part) and
      // the four table entries of the octet are read from LDS once each, one part ahead of their first use: a read
      // issued right where it is needed would expose the LDS latency in every slot.
      auto slice = [&](auto slot_c) {
        constexpr int slot = decltype(slot_c)::value;
        constexpr int FIRST = SLOTS / 3, SPAN = SLOTS - FIRST, NW = NV * 4;
        if constexpr (slot == FIRST - 1) abv[0] = table_entry(0, c0n);
        if constexpr (slot >= FIRST) {
          constexpr int w0 = (slot - FIRST) * NW / SPAN, w1 = (slot - FIRST + 1) * NW / SPAN;
          static_for<w1 - w0>([&](auto k_c) {
            constexpr int wi = w0 + decltype(k_c)::value;
            constexpr int part = wi / NV, i = wi % NV;
            if constexpr (i == 0 && part < 3) abv[(part + 1) & 1] = table_entry(part + 1, c0n);
            raw[i][part] = activate_with(raw[i][part], abv[part & 1]);
            if constexpr (part == 3) store_vec(i, nbuf);
          });
        }
      };
      // the last chunk activates a harmless reload into the buffer nobody reads: one instruction stream, no
      // control flow inside the pinned schedule
      mfma_chunk<T, MI, NI, KT, KC, ROW, PS, D, true, SPREAD, decltype(slice)&, (RING > 6 ? 2 : 1)>(buf, a_off, wrsrc, bcur, bnext, tap_stride, kk_stride, lane16, bq, acc, slice);
    } else {
      auto none = [](auto) {};
      mfma_chunk<T, MI, NI, KT, KC, ROW, PS, D, false, -1, decltype(none)&, (RING > 6 ? 2 : 1)>(buf, a_off, wrsrc, bcur, bnext, tap_stride, kk_stride, lane16, bq, acc, none);
      if (more) activate_all(c0n, nbuf);
    }
    issue(c + 2);
    __syncthreads();          // other buffer staged; this one free for chunk c+2
  }

  // ---- epilogue: bias, residual, one rounding, store (through a wavefront-private LDS patch over the tile buffers)
  TO* yout = reinterpret_cast<TO*>(p.y) + (size_t)n * p.h * p.w_out * p.cout;
  const T* rin = p.res ? reinterpret_cast<const T*>(p.res) + (size_t)n * p.h * p.w_out * p.cout : nullptr;
  float* patch = reinterpret_cast<float*>(smem) + wave * patch_floats(NI);
  // statistics slot of this wavefront: [sample][group][spatial tile * WM + wave row]
  Moments* st = p.stats ? p.stats + (size_t)n * p.stats_groups * p.stats_slots + (tile * WM + wm) : nullptr;
  if (rin)
    epilogue_store<T, TO, MI, NI, MTW, MTH, MT_PER_ROW, true>(acc, patch, lane, PH ? 0 : wm * MI, ty0, tx0, co0 + wn * NI * 32, p.bias,
                                                              p.bias2, rin, yout, p.h, p.w_out, p.cout, false, st, p.stats_cpg, p.stats_slots,
                                                              PH ? 2 : 1, PH ? wave >> 1 : 0, PH ? wave & 1 : 0);
  else
    epilogue_store<T, TO, MI, NI, MTW, MTH, MT_PER_ROW, false>(acc, patch, lane, PH ? 0 : wm * MI, ty0, tx0, co0 + wn * NI * 32, p.bias,
                                                               p.bias2, rin, yout, p.h, p.w_out, p.cout, p.y_nchw != 0, st, p.stats_cpg, p.stats_slots,
                                                               PH ? 2 : 1, PH ? wave >> 1 : 0, PH ? wave & 1 : 0);

  // ---- row hand-over: the workgroup that finishes a (sample, tile row, channel tile) last merges the row's triples.
  // Same protocol as the single-launch statistics kernel: the triples were written with device-scope stores, every
  // wavefront waits for its stores, the workgroup takes a ticket (a wrapping counter that returns to zero by itself),
  // and only the last one reads, with device-scope loads, in a fixed order.
  if (p.rows_out) {
    __shared__ unsigned s_last;
    wait_stores();
    __syncthreads();
    const int tile_y = tile / p.tiles_x;
    if (tid == 0) s_last = atomicInc(p.tickets + ((size_t)n * p.tiles_y + tile_y) * p.ntiles + nt, p.tiles_x - 1) == (unsigned)(p.tiles_x - 1);
    __syncthreads();
    if (s_last) {
      const int per_row = p.tiles_x * WM;                  // triples of one group in this tile row
      const int g0 = co0 / p.stats_cpg, gcount = min(TN, p.cout - co0) / p.stats_cpg;
      const int sub = tid & 7;
      for (int gi = tid >> 3; gi < gcount; gi += NT / 8) {
        const Moments* src = p.stats + ((size_t)n * p.stats_groups + g0 + gi) * p.stats_slots + (size_t)tile_y * per_row;
        Moments m{0.f, 0.f, 0.f};
        for (int e0 = sub; e0 < per_row; e0 += 64) {     // eight loads in flight per lane
          Moments t[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            const int e = e0 + 8 * k;
            t[k] = load_device(src + min(e, per_row - 1));
            if (e >= per_row) t[k].n = 0.f;
          }
#pragma unroll
          for (int k = 0; k < 8; ++k) m = merge(m, t[k]);
        }
        m = merge_to_first(m, lane, 8);
        if (sub == 0) p.rows_out[((size_t)n * p.stats_groups + g0 + gi) * p.tiles_y + tile_y] = m;
      }
    }
  }
}

template <typename T, typename TO, int TH, int TW, int WM, int WN, int NI, int KS, int KC, bool PH = false, int RING = 0>
int launch_cfg(const ConvArgs& a, hipStream_t s) {
  constexpr int PAD = PH ? 1 : KS / 2;
  constexpr int TN = WN * NI * 32;
  WMDEC_REQUIRE(!PH || (a.wt_phase && a.h % 2 == 0 && a.w % 2 == 0), WMDEC_ERR_INVALID_ARG, "conv_mfma: upsampling convolution without phase weights");
  MfmaParams p;
  p.x = a.x; p.mean = a.mean; p.rstd = a.rstd; p.gamma = a.gamma; p.beta = a.beta;
  p.w = PH ? a.wt_phase : a.wt; p.bias = a.bias; p.res = a.res; p.y = a.y;
  p.silu = a.silu; p.groups = a.groups; p.norm = a.mean != nullptr;
  p.n = a.n; p.h = a.h; p.w_out = a.w; p.cin = a.cin; p.cout = a.cout; p.upsample = a.upsample;
  const int w_t = PH ? a.w / 2 : a.w, h_t = PH ? a.h / 2 : a.h;   // the grid the tiles live on
  p.tiles_x = (w_t + TW - 1) / TW; p.tiles_y = (h_t + TH - 1) / TH; p.ntiles = (a.cout + TN - 1) / TN;
  p.total = p.tiles_x * p.tiles_y * p.ntiles * a.n;
  p.cin_blocks = packed_cin_blocks(a.cin); p.cout_blocks = packed_cout_blocks(a.cout); p.y_nchw = a.y_nchw;
  p.w_bytes = (int)(packed_elems(PH ? 16 : KS * KS, a.cout, a.cin) * sizeof(T));
  p.stats = (Moments*)a.stats_ws; p.stats_groups = a.stats_groups; p.stats_cpg = a.stats_groups > 0 ? a.cout / a.stats_groups : 1;
  p.stats_slots = p.tiles_x * p.tiles_y * WM;
  p.rows_out = (Moments*)a.rows_out; p.tickets = (unsigned*)a.tickets;
  p.rows_in = (const Moments*)a.rows_in; p.rows_in_count = a.rows_in_count; p.eps = a.eps;
  WMDEC_REQUIRE(!p.rows_out || (p.stats && p.tickets), WMDEC_ERR_INVALID_ARG, "conv_mfma: row moments need the triple scratch and the ticket counters");
  WMDEC_REQUIRE(!p.rows_in || (p.rows_in_count >= 1 && p.rows_in_count <= 128), WMDEC_ERR_UNSUPPORTED, "conv_mfma: at most 128 triples per group can be merged in the prologue");
  p.norm = a.mean != nullptr || a.rows_in != nullptr;
  p.x2 = nullptr; p.w2 = nullptr; p.bias2 = nullptr; p.cin2 = 0; p.w2_bytes = 0;
  if (a.x2) {
    WMDEC_REQUIRE(KS == 3 && !PH && a.w2 && a.cin2 > 0 && a.cin2 % KC == 0 && (long)a.h * a.w * a.cin2 < (1L << 29), WMDEC_ERR_UNSUPPORTED,
                  "conv_mfma: a folded shortcut needs a 3x3 convolution without upsampling and cin2 %% %d == 0", KC);
    p.x2 = a.x2; p.w2 = a.w2; p.bias2 = a.bias2; p.cin2 = a.cin2;
    p.w2_bytes = (int)(packed_elems(1, a.cout, a.cin2) * sizeof(T));
  }
  constexpr int NT = 64 * WM * WN;
  size_t smem = (((size_t)2 * tile_buf_elems(TH, TW, PAD, KC) * 2 + 15) & ~(size_t)15) + (size_t)(a.cin + a.groups) * sizeof(float2);
  const size_t patch = (size_t)(WM * WN) * patch_floats(NI) * sizeof(float);   // epilogue patches of the wavefronts
  if (smem < patch) smem = patch;
  WMDEC_REQUIRE(smem <= 80 * 1024, WMDEC_ERR_UNSUPPORTED, "conv_mfma: %zu bytes of LDS needed", smem);
  void (*kern)(MfmaParams) = !p.norm ? conv_mfma_kernel<T, TO, TH, TW, WM, WN, NI, KS, KC, 0, PH, RING>
                             : (a.silu ? conv_mfma_kernel<T, TO, TH, TW, WM, WN, NI, KS, KC, 2, PH, RING>
                                       : conv_mfma_kernel<T, TO, TH, TW, WM, WN, NI, KS, KC, 1, PH, RING>);
  // once per instantiation and activation mode (80 KiB: two workgroups per compute unit)
  static std::once_flag attr_once[3];
  hipError_t attr_err = hipSuccess;
  std::call_once(attr_once[!p.norm ? 0 : (a.silu ? 2 : 1)],
                 [&] { attr_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024); });
  WMDEC_HIP(attr_err);
  hipLaunchKernelGGL(kern, dim3((unsigned)p.total), dim3(NT), smem, s, p);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

// Tile shapes: patch height x width, wavefront rows x columns, 32-channel tiles per wavefront.
struct TileShape { int th, tw, wm, wn, ni; };
enum TileId { T256x128 = 0, T128x128_ROW, T128x64_ROW, T128x64, T256x32, T_PHASE, T128x128_1x4, T128x256, kNumTiles };
constexpr TileShape kTiles[kNumTiles] = {
    {8, 32, 2, 2, 2},    // T256x128: 256 pixels x 128 channels (large 1x1 convolutions)
    {4, 32, 2, 2, 2},    // T128x128_ROW: 128 x 128 on a 4x32 patch (1x1 convolutions)
    {4, 32, 4, 1, 2},    // T128x64_ROW: 128 x 64 on a 4x32 patch (1x1 convolutions)
    {8, 16, 4, 1, 2},    // T128x64: 128 x 64 on an 8x16 patch
    {8, 32, 4, 1, 1},    // T256x32: 256 x 32 (few output channels: the frame)
    {8, 16, 4, 1, 2},    // T_PHASE: phase-decomposed upsampling convolution: 8x16 input pixels (16x32 outputs) x 64 channels
    {8, 16, 1, 4, 1},    // T128x128_1x4: 128 x 128, every wavefront all pixels x 32 channels: a weight fragment feeds four
                         //     MFMAs, which keeps the fragment loads off the limit of the vector L1 (64 B/clk per compute unit)
    {8, 16, 1, 4, 2},    // T128x256: 128 x 256, every wavefront all pixels x 64 channels: a staged (normalised, activated) patch
                         //     feeds twice the channels, i.e. half the staging work and input traffic per MFMA; two
                         //     workgroups per compute unit
};

// which tile shape a launch uses; a function of the per-sample shape only, so that the tiling, hence every summation
// order, does not depend on the batch
TileId pick_tile(const ConvArgs& a) {
  const long px = (long)a.h * a.w;
  const bool n128 = a.cout % 128 == 0;
  if (a.ksize == 3) {
    if (conv_mfma_uses_phase(a)) return T_PHASE;
    if (a.cout <= 32) return T256x32;
    // 128 pixels x 128 channels with every wavefront on all pixels x 32 channels (three workgroups per compute unit):
    // measured against the 256-pixel tile and the 2x2 wavefront layout on every layer shape of the decoder, it is
    // equal or faster everywhere (128 -> 128 at 480x720: 110 against 120 us; 512 -> 512 at 60x90: 33.5 against 35.1)
    // With 256 channels per workgroup the normalise + SiLU work and the input traffic per MFMA halve, at two workgroups
    // per compute unit instead of three: it pays (6 to 8 %) where that still leaves every compute unit two workgroups
    // (the 240x360 layers of the decoder), and loses on smaller layers.
    if (a.cout % 256 == 0 && ((px + 127) / 128) * (a.cout / 256) >= 2 * 256) return T128x256;
    // (a 96-pixel tile on 6x16 patches, which puts the 512 -> 512 layers at 60x90 on 240 instead of 192 compute units,
    // measured 3 % on those layers: a lone workgroup's time is set by its weight stream, 1.2 MB through the vector
    // L1 whatever its pixel count; not kept)
    return n128 ? T128x128_1x4 : T128x64;
  }
  if (n128 && a.cin % 64 == 0 && px * (a.cout / 128) >= 256L * 256 * 2) return T256x128;
  return n128 ? T128x128_ROW : T128x64_ROW;
}

// The 128x128 tile with a whole chunk of weight fragments in flight (see RING): launches of at most two workgroups per
// compute unit.  Unlike the tile shape this may depend on the batch: the ring changes no summation order.
bool whole_chunk_ring(const ConvArgs& a) {
  if (pick_tile(a) != T128x128_1x4) return false;
  const long wgs = (long)((a.h + 7) / 8) * ((a.w + 15) / 16) * (a.cout / 128) * a.n;
  return wgs <= 2 * 256;
}

template <typename T, typename TO>
int launch_3x3(const ConvArgs& a, hipStream_t s) {
  switch (pick_tile(a)) {
    case T128x64: return launch_cfg<T, TO, 8, 16, 4, 1, 2, 3, 32>(a, s);
    case T_PHASE: return launch_cfg<T, TO, 8, 16, 4, 1, 2, 3, 32, true>(a, s);
    case T128x128_1x4:
      return whole_chunk_ring(a) ? launch_cfg<T, TO, 8, 16, 1, 4, 1, 3, 32, false, 18>(a, s) : launch_cfg<T, TO, 8, 16, 1, 4, 1, 3, 32>(a, s);
    case T128x256: return launch_cfg<T, TO, 8, 16, 1, 4, 2, 3, 32>(a, s);
    default: return launch_cfg<T, TO, 8, 32, 4, 1, 1, 3, 32>(a, s);
  }
}

// chunk of input channels a 1x1 launch stages at a time: 64 halves the barriers
int chunk_1x1(const ConvArgs& a) { return a.cin % 64 == 0 ? 64 : 32; }

template <typename T, typename TO>
int launch_1x1(const ConvArgs& a, hipStream_t s) {
  const TileId t = pick_tile(a);
  if (chunk_1x1(a) == 64) {
    if (t == T256x128) return launch_cfg<T, TO, 8, 32, 2, 2, 2, 1, 64>(a, s);
    if (t == T128x128_ROW) return launch_cfg<T, TO, 4, 32, 2, 2, 2, 1, 64>(a, s);
    return launch_cfg<T, TO, 4, 32, 4, 1, 2, 1, 64>(a, s);
  }
  if (t == T128x128_ROW) return launch_cfg<T, TO, 4, 32, 2, 2, 2, 1, 32>(a, s);
  return launch_cfg<T, TO, 4, 32, 4, 1, 2, 1, 32>(a, s);
}

template <typename T>
int launch_type(const ConvArgs& a, hipStream_t s) {
  if (a.y_dtype == WMDEC_F32) return a.ksize == 3 ? launch_3x3<T, float>(a, s) : launch_1x1<T, float>(a, s);
  return a.ksize == 3 ? launch_3x3<T, T>(a, s) : launch_1x1<T, T>(a, s);
}

}  // namespace

bool conv_mfma_supported(const ConvArgs& a) {
  if (!is_16bit(a.op_dtype) || a.x_dtype != a.op_dtype) return false;
  if (a.res && a.res_dtype != a.op_dtype) return false;
  if (a.y_dtype != a.op_dtype && a.y_dtype != WMDEC_F32) return false;
  if (a.x_nchw) return false;
  if (a.y_nchw && !(a.cout <= 32 && a.y_dtype == WMDEC_F32 && !a.res && a.ksize == 3)) return false;
  if (a.cin % 32 != 0) return false;
  if (a.cout % 64 != 0 && !(a.y_nchw && a.cout <= 32)) return false;
  if (a.cin > 2048) return false;   // scale/shift table lives in LDS
  if (a.ksize != 1 && a.ksize != 3) return false;
  if ((long)a.h * a.w * a.cin >= (1L << 29) || (long)a.h * a.w * a.cout >= (1L << 29)) return false;   // 32-bit byte offsets per sample
  return true;
}

// Phase decomposition of an upsampling convolution (needs a.wt_phase at launch), f16 only: pre-added weights rounded
// to bf16 would cost that type a visible part of its error budget.
bool conv_mfma_uses_phase(const ConvArgs& a) {
  return conv_mfma_supported(a) && a.ksize == 3 && a.upsample && a.op_dtype == WMDEC_F16 && a.cout % 64 == 0;
}

int conv_mfma_stats_slots(const ConvArgs& a) {
  if (!conv_mfma_supported(a) || a.y_nchw || a.stats_groups <= 0 || a.cout % a.stats_groups != 0) return 0;
  const int cpg = a.cout / a.stats_groups;
  if ((cpg & (cpg - 1)) != 0 || cpg > 32) return 0;   // a group must sit inside one wavefront's 64-channel run
  const TileId t = pick_tile(a);
  const TileShape& ts = kTiles[t];
  const int w_t = t == T_PHASE ? a.w / 2 : a.w, h_t = t == T_PHASE ? a.h / 2 : a.h;
  return ((w_t + ts.tw - 1) / ts.tw) * ((h_t + ts.th - 1) / ts.th) * ts.wm;
}

// tile rows / channel tiles of a launch: the extents of the row moments it can leave and of its ticket counters
void conv_mfma_row_extents(const ConvArgs& a, int* tile_rows, int* channel_tiles, int* tiles_per_row) {
  const TileId t = pick_tile(a);
  const TileShape& ts = kTiles[t];
  const int h_t = t == T_PHASE ? a.h / 2 : a.h, w_t = t == T_PHASE ? a.w / 2 : a.w, tn = ts.wn * ts.ni * 32;
  *tile_rows = (h_t + ts.th - 1) / ts.th;
  *channel_tiles = (a.cout + tn - 1) / tn;
  *tiles_per_row = (w_t + ts.tw - 1) / ts.tw;
}

// the instantiation a launch would use, spelled like a profiler prints it
const char* conv_mfma_label(const ConvArgs& a) {
  static thread_local char buf[160];
  const TileId t = pick_tile(a);
  const int kc = a.ksize == 1 ? chunk_1x1(a) : 32;
  const TileShape& ts = kTiles[t];
  const char* ty = a.op_dtype == WMDEC_BF16 ? "wmdec::bf16_t" : "wmdec::f16_t";
  const int act = a.mean == nullptr && a.rows_in == nullptr && !a.groups_norm ? 0 : (a.silu ? 2 : 1);
  snprintf(buf, sizeof(buf), "conv_mfma_kernel<%s, %s, %d, %d, %d, %d, %d, %d, %d, %d, %s, %d>", ty,
           a.y_dtype == WMDEC_F32 ? "float" : ty, ts.th, ts.tw, ts.wm, ts.wn, ts.ni, a.ksize, kc, act, t == T_PHASE ? "true" : "false",
           a.ksize == 3 && whole_chunk_ring(a) ? 18 : 0);
  return buf;
}

int launch_conv_mfma(const ConvArgs& a, hipStream_t s) {
  return a.op_dtype == WMDEC_BF16 ? launch_type<bf16_t>(a, s) : launch_type<f16_t>(a, s);
}

}  // namespace wmdec
