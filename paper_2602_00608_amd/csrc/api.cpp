// C ABI of libwmdec.so: argument checking, per-op entry points and the decoder
// graph (plan built once at decoder_create, replayed by decoder_run).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <string>
#include <vector>

#include "common.hpp"
#include "pack_layout.hpp"

namespace wmdec {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int hip_fail(hipError_t e, const char* what) {
  set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
  return WMDEC_ERR_HIP;
}

int launch_conv(const ConvArgs& a, hipStream_t s) {
  if (conv_taps_supported(a)) return launch_conv_taps(a, s);
  if (conv_mfma_supported(a)) return launch_conv_mfma(a, s);
  WMDEC_REQUIRE(!a.x2, WMDEC_ERR_UNSUPPORTED, "conv: only the matrix-core kernel folds a shortcut into the contraction");
  if (conv_small_cin_supported(a)) return launch_conv_small_cin(a, s);
  return launch_conv_direct(a, s);
}

// Triples per (sample, group) that the kernel launch_conv picks for this shape emits with stats_ws set; 0: it emits none.
static int conv_stats_slots(const ConvArgs& a) {
  if (conv_taps_supported(a)) return 0;
  if (conv_mfma_supported(a)) return conv_mfma_stats_slots(a);
  return conv_small_cin_supported(a) ? conv_small_cin_stats_slots(a) : 0;
}

const char* conv_kernel_label(const ConvArgs& a) {
  if (conv_taps_supported(a)) return conv_taps_label(a);
  if (!conv_mfma_supported(a)) return conv_small_cin_supported(a) ? "conv_small_cin_kernel" : "conv_direct_kernel";
  return conv_mfma_label(a);
}

static inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// common checks of the convolution entry points
static int check_conv(const char* who, const void* x, int act_dtype, const float* mean, const float* rstd,
                      const float* gamma, const float* beta, int groups, const void* w_packed, const void* residual,
                      void* y, int y_dtype, int n, int h, int w, int cin, int cout) {
  WMDEC_REQUIRE(x && w_packed && y, WMDEC_ERR_INVALID_ARG, "%s: null tensor pointer", who);
  WMDEC_REQUIRE(valid_dtype(act_dtype) && valid_dtype(y_dtype), WMDEC_ERR_INVALID_ARG, "%s: bad dtype", who);
  WMDEC_REQUIRE(y_dtype == act_dtype || y_dtype == WMDEC_F32, WMDEC_ERR_UNSUPPORTED,
                "%s: y_dtype must equal act_dtype or be F32", who);
  WMDEC_REQUIRE(n > 0 && h > 0 && w > 0 && cin > 0 && cout > 0, WMDEC_ERR_INVALID_ARG, "%s: non-positive size", who);
  WMDEC_REQUIRE(aligned16(x) && aligned16(w_packed) && aligned16(y) && aligned16(residual), WMDEC_ERR_INVALID_ARG,
                "%s: pointers must be 16-byte aligned", who);
  WMDEC_REQUIRE(x != y, WMDEC_ERR_INVALID_ARG, "%s: x and y must not overlap", who);
  if (mean) {
    WMDEC_REQUIRE(rstd && gamma && beta, WMDEC_ERR_INVALID_ARG, "%s: mean given without rstd/gamma/beta", who);
    WMDEC_REQUIRE(groups > 0 && cin % groups == 0, WMDEC_ERR_SHAPE, "%s: cin %d not divisible by groups %d", who, cin, groups);
  }
  return WMDEC_OK;
}

// ---------------------------------------------------------------- decoder plan
enum BufId { BUF_LATENT = -2, BUF_OUT = -3, BUF_NONE = -1 };  // >= 0: activation ping-pong buffers

struct Param {  // one canonical parameter
  std::string name;
  int shape[4];
  int dtype;
  size_t offset, bytes;      // in the canonical blob
  size_t packed_offset;      // in the packed blob
  size_t packed_bytes;
  bool upconv = false;       // weights of an upsampling convolution: 9-tap pack followed by the 16-tap phase pack
};

struct Step {
  enum Kind { STATS, CONV, QKV_TRANSPOSE_V, FLASH, NONE } kind;
  int src = BUF_NONE, dst = BUF_NONE, res = BUF_NONE;
  int h = 0, w = 0, cin = 0, cout = 0;   // conv: OUTPUT h, w; stats: tensor h, w, c = cin
  int ksize = 3, upsample = 0, norm = 0, silu = 0;
  int x_nchw = 0, y_nchw = 0, to_attn = 0 /*1: dst is the qkv buffer, 2: src is the attention output*/;
  int emit_stats = 0;      // CONV: its epilogue also writes the GroupNorm moments of its output
  int from_producer = 0;   // STATS: only merge the moments the producing convolution left behind
  int emit_rows = -1;      // CONV (with emit_stats): also leaves row moments in row buffer 0 / 1; no merge launch follows
  int emit_direct = 0;     //   ... as the triples of its workgroups themselves (few spatial tiles), without a merge by row
  int rows_from = -1;      // CONV with norm: takes the statistics of its input from row buffer 0 / 1 ...
  int rows_count = 0;      //   ... which holds this many rows per (sample, group)
  size_t w_off = 0, b_off = 0, gamma_off = 0, beta_off = 0;
  int sc_src = BUF_NONE, sc_cin = 0;   // CONV 3x3: a 1x1 shortcut over this buffer is folded into the contraction
  size_t sc_w_off = 0, sc_b_off = 0;
  double flops = 0.0, bytes = 0.0;   // algorithmic work / HBM traffic of this step for one frame
  double flops_dense = 0.0;          // the same with an upsampling convolution priced as nine taps per output
};

}  // namespace wmdec

using namespace wmdec;

struct wmdec_decoder {
  wmdec_decoder_config cfg;
  std::vector<Param> params;
  std::vector<Step> steps;
  size_t weights_bytes = 0, packed_bytes = 0;
  size_t act_elems_per_frame = 0;   // largest activation tensor, elements per frame
  int attn_t = 0, attn_tpad = 0, attn_c = 0;
  size_t qkv_w_off = 0, qkv_b_off = 0;   // fused [3c][c] projection and its [3c] bias in the packed blob
  double flops = 0.0;         // executed multiply-adds x 2 of one frame
  double flops_dense = 0.0;   // 2*k*k*cin*cout per output pixel everywhere (what an unfused graph would execute)
  int launches = 0;
  void* ws = nullptr;
  size_t ws_bytes = 0;
  bool ws_fresh = true;    // the statistics ticket counter of a newly set workspace has not been zeroed yet
  bool profiling = false;
  int profiled_batch = 0;
  std::vector<hipEvent_t> events;   // steps.size() + 1 when profiling was ever enabled
  ~wmdec_decoder() {
    for (hipEvent_t e : events) (void)hipEventDestroy(e);
  }
};

namespace wmdec {

// the launch-shape part of a CONV step's arguments (pointers left null)
static ConvArgs step_shape_args(const wmdec_decoder& d, const Step& st, int batch) {
  ConvArgs a;
  a.op_dtype = d.cfg.act_dtype; a.res_dtype = a.op_dtype;
  a.x_dtype = st.src == BUF_LATENT ? d.cfg.latent_dtype : a.op_dtype; a.x_nchw = st.x_nchw;
  a.y_dtype = st.dst == BUF_OUT ? (int)WMDEC_F32 : a.op_dtype; a.y_nchw = st.y_nchw;
  a.n = batch; a.h = st.h; a.w = st.w; a.cin = st.cin; a.cout = st.cout; a.ksize = st.ksize; a.upsample = st.upsample;
  a.stats_groups = d.cfg.groups;
  return a;
}

struct Builder {
  wmdec_decoder& d;
  size_t off = 0, poff = 0;
  explicit Builder(wmdec_decoder& dec) : d(dec) {}

  int add(const std::string& name, int s0, int s1, int s2, int s3, int dtype, bool upconv = false) {
    Param p;
    p.name = name;
    p.upconv = upconv;
    p.shape[0] = s0; p.shape[1] = s1; p.shape[2] = s2; p.shape[3] = s3;
    p.dtype = dtype;
    p.bytes = (size_t)s0 * s1 * s2 * s3 * dtype_size(dtype);
    p.offset = off;
    off = align_up(off + p.bytes, 256);
    // packed: conv weights in the operand type, everything else copied as fp32
    p.packed_bytes = dtype == WMDEC_F32 ? p.bytes
                     : upconv ? upconv_packed_bytes(s0, s1, d.cfg.act_dtype)
                              : packed_elems(s2 * s3, s0, s1) * dtype_size(d.cfg.act_dtype);
    p.packed_offset = poff;
    poff = align_up(poff + p.packed_bytes, 256);
    d.params.push_back(p);
    return (int)d.params.size() - 1;
  }
  // conv parameters: weight then bias
  void conv_params(const std::string& name, int cout, int cin, int k, size_t* w_off, size_t* b_off, bool upconv = false) {
    const int wi = add(name + ".w", cout, cin, k, k, WMDEC_BF16, upconv);
    const int bi = add(name + ".b", cout, 1, 1, 1, WMDEC_F32);
    *w_off = d.params[wi].packed_offset;
    *b_off = d.params[bi].packed_offset;
  }
  void norm_params(const std::string& name, int c, size_t* g_off, size_t* b_off) {
    const int gi = add(name + ".gamma", c, 1, 1, 1, WMDEC_F32);
    const int bi = add(name + ".beta", c, 1, 1, 1, WMDEC_F32);
    *g_off = d.params[gi].packed_offset;
    *b_off = d.params[bi].packed_offset;
  }
  void stats(int src, int h, int w, int c) {
    Step s; s.kind = Step::STATS; s.src = src; s.h = h; s.w = w; s.cin = c;
    s.bytes = (double)h * w * c * dtype_size(d.cfg.act_dtype);
    d.steps.push_back(s);
    d.launches += gn_stats_num_launches(d.cfg.act_dtype, h, w, c, d.cfg.groups);
  }
  // call right after pushing a CONV step: accounts its work on the pushed copy
  void count_conv(const Step&) {
    Step& s = d.steps.back();
    const double es = (double)dtype_size(d.cfg.act_dtype);
    const double px_out = (double)s.h * s.w, px_in = s.upsample ? px_out / 4 : px_out;
    s.flops_dense = 2.0 * s.ksize * s.ksize * (double)s.cin * s.cout * px_out;
    // a phase-decomposed upsampling convolution executes a 2x2 convolution per output: 4/9 of the products.
    // Only executed work is counted, never the work avoided.
    s.flops = conv_mfma_uses_phase(step_shape_args(d, s, 1)) ? s.flops_dense * 4.0 / 9.0 : s.flops_dense;
    if (s.sc_src != BUF_NONE) {   // folded 1x1 shortcut: its products, its input and its weights
      const double f = 2.0 * (double)s.sc_cin * s.cout * px_out;
      s.flops += f; s.flops_dense += f;
    }
    s.bytes = px_in * s.cin * (s.src == BUF_LATENT ? (double)dtype_size(d.cfg.latent_dtype) : es)                  // input, once
              + px_out * s.cout * (s.dst == BUF_OUT ? 4.0 : es)                 // output, once
              + (s.res != BUF_NONE ? px_out * s.cout * es : 0.0)                // residual, once
              + (double)s.ksize * s.ksize * s.cin * s.cout * es                 // weights, once
              + (s.sc_src != BUF_NONE ? (px_out * s.sc_cin + (double)s.sc_cin * s.cout) * es : 0.0);   // shortcut input and weights
    d.flops += s.flops;
    d.flops_dense += s.flops_dense;
    d.launches += 1;
  }
  void track(int h, int w, int c) {
    const size_t e = (size_t)h * w * c;
    if (e > d.act_elems_per_frame) d.act_elems_per_frame = e;
  }
  // x (buffer a) -> out (buffer c), scratch b.  Returns nothing; caller rotates.
  void resblock(const std::string& name, int a, int b, int c, int h, int w, int cin, int cout) {
    Step c1; c1.kind = Step::CONV; c1.src = a; c1.dst = b; c1.h = h; c1.w = w; c1.cin = cin; c1.cout = cout;
    c1.norm = 1; c1.silu = 1;
    norm_params(name + ".norm1", cin, &c1.gamma_off, &c1.beta_off);
    conv_params(name + ".conv1", cout, cin, 3, &c1.w_off, &c1.b_off);
    Step c2; c2.kind = Step::CONV; c2.src = b; c2.dst = c; c2.h = h; c2.w = w; c2.cin = cout; c2.cout = cout;
    c2.norm = 1; c2.silu = 1;
    norm_params(name + ".norm2", cout, &c2.gamma_off, &c2.beta_off);
    conv_params(name + ".conv2", cout, cout, 3, &c2.w_off, &c2.b_off);
    Step sc; sc.kind = Step::CONV;
    bool fold = false;
    if (cin != cout) {
      sc.src = a; sc.dst = c; sc.h = h; sc.w = w; sc.cin = cin; sc.cout = cout; sc.ksize = 1;
      conv_params(name + ".shortcut", cout, cin, 1, &sc.w_off, &sc.b_off);
      // The 1x1 shortcut becomes extra contraction steps of conv2 (K = 9*cout + cin) where the matrix-core kernel
      // takes the layer; otherwise it stays a launch of its own that conv2 adds from its own output buffer.
      ConvArgs probe = step_shape_args(d, c2, 1);
      probe.res = nullptr;
      fold = !d.cfg.separate_shortcut && conv_mfma_supported(probe) && cin % 32 == 0;
      if (fold) { c2.sc_src = a; c2.sc_cin = cin; c2.sc_w_off = sc.w_off; c2.sc_b_off = sc.b_off; c2.res = BUF_NONE; }
      else c2.res = c;   // conv2 adds the shortcut it finds in its own output buffer
    } else {
      c2.res = a;
    }
    stats(a, h, w, cin);
    d.steps.push_back(c1); count_conv(c1);
    if (cin != cout && !fold) { d.steps.push_back(sc); count_conv(sc); }
    stats(b, h, w, cout);
    d.steps.push_back(c2); count_conv(c2);
    track(h, w, cin); track(h, w, cout);
  }
};


// Statistics passes whose input was written by a convolution that can emit moments in its epilogue become
// a merge of those moments: the tensor is not read again.  One partial buffer exists, so a producer is used
// only if no other emitting convolution runs between it and its statistics step.
static void fuse_stats_into_producers(wmdec_decoder& d) {
  int parity = 0;
  for (size_t i = 0; i < d.steps.size(); ++i) {
    Step& st = d.steps[i];
    if (st.kind != Step::STATS || st.src < 0) continue;
    int j = (int)i - 1;
    while (j >= 0 && !(d.steps[j].kind == Step::CONV && d.steps[j].dst == st.src && d.steps[j].to_attn != 1)) --j;
    if (j < 0) continue;
    bool clash = false;
    for (size_t k = j + 1; k < i; ++k) clash |= d.steps[k].kind == Step::CONV && d.steps[k].emit_stats;
    if (clash || conv_stats_slots(step_shape_args(d, d.steps[j], 1)) <= 0) continue;
    d.steps[j].emit_stats = 1;
    st.from_producer = 1;
    st.bytes = 0.0;          // no tensor traffic left in this step
    d.launches -= gn_stats_num_launches(d.cfg.act_dtype, st.h, st.w, st.cin, d.cfg.groups) - 1;   // one merge launch remains
    // The consumer of these statistics is the next step.  If it is a matrix-core convolution, the producer's last
    // workgroup per tile row merges that row and the consumer merges the rows while it builds its scale/shift table:
    // the merge launch disappears.  Two row buffers alternate, because a consumer is usually the next producer.
    if (d.cfg.separate_merge_launch || i + 1 >= d.steps.size()) continue;
    Step& cons = d.steps[i + 1];
    if (cons.kind != Step::CONV || !cons.norm || cons.src != st.src || !conv_mfma_supported(step_shape_args(d, cons, 1))) continue;
    if (conv_taps_supported(step_shape_args(d, cons, 1))) continue;   // that kernel takes mean / rstd only
    // A producer with few spatial tiles needs no merge of its own at all: the consumer reads its triples as they are.
    const int slots = conv_stats_slots(step_shape_args(d, d.steps[j], 1));
    if (slots <= 128) {
      d.steps[j].emit_rows = parity;
      d.steps[j].emit_direct = 1;
      cons.rows_from = parity;
      cons.rows_count = slots;
      parity ^= 1;
      st.kind = Step::NONE;
      d.launches -= 1;
      continue;
    }
    if (!conv_mfma_supported(step_shape_args(d, d.steps[j], 1))) continue;   // only that kernel merges by row
    int rows = 0, ctiles = 0, per_row = 0;
    conv_mfma_row_extents(step_shape_args(d, d.steps[j], 1), &rows, &ctiles, &per_row);
    if (rows > 64) continue;   // keeps the consumer's merge short
    // The hand-over keeps every workgroup of the producer resident for two more memory round trips (its stores, its
    // ticket).  Measured, that costs a launch of several rounds of workgroups as much as the merge launch it saves;
    // it wins where the producer is a single round (at most three workgroups per compute unit, per sample).
    if ((long)rows * per_row * ctiles > 3 * 256) continue;
    d.steps[j].emit_rows = parity;
    cons.rows_from = parity;
    cons.rows_count = rows;
    parity ^= 1;
    st.kind = Step::NONE;    // removed below
    d.launches -= 1;
  }
  std::vector<Step> kept;
  for (const Step& st : d.steps)
    if (st.kind != Step::NONE) kept.push_back(st);
  d.steps.swap(kept);
}

static int build_plan(wmdec_decoder& d) {
  const wmdec_decoder_config& c = d.cfg;
  Builder B(d);
  int h = c.latent_h, w = c.latent_w;
  const int c0 = c.level_channels[0];
  int cur = 0;  // buffer holding the current activation
  auto other = [&](int k) { return (cur + k) % 3; };

  {  // conv_in: NCHW latent -> NHWC
    Step s; s.kind = Step::CONV; s.src = BUF_LATENT; s.dst = cur; s.h = h; s.w = w; s.cin = c.latent_c; s.cout = c0;
    s.x_nchw = 1;
    B.conv_params("conv_in", c0, c.latent_c, 3, &s.w_off, &s.b_off);
    d.steps.push_back(s); B.count_conv(s); B.track(h, w, c0);
  }
  B.resblock("mid.res1", cur, other(1), other(2), h, w, c0, c0);
  cur = other(2);
  {  // attention: stats, fused qkv projection, V transpose, flash core, output projection + residual
    Step q; q.kind = Step::CONV; q.src = cur; q.to_attn = 1; q.h = h; q.w = w; q.cin = c0; q.cout = 3 * c0; q.ksize = 1;
    q.norm = 1; q.silu = 0;
    B.norm_params("mid.attn.norm", c0, &q.gamma_off, &q.beta_off);
    size_t woff[3], boff[3];
    B.conv_params("mid.attn.q", c0, c0, 1, &woff[0], &boff[0]);
    B.conv_params("mid.attn.k", c0, c0, 1, &woff[1], &boff[1]);
    B.conv_params("mid.attn.v", c0, c0, 1, &woff[2], &boff[2]);
    // the packed blob also holds q, k, v fused into one [3c][c] matrix and one [3c] bias
    d.qkv_w_off = B.poff; B.poff = align_up(B.poff + packed_elems(1, 3 * c0, c0) * dtype_size(c.act_dtype), 256);
    d.qkv_b_off = B.poff; B.poff = align_up(B.poff + (size_t)3 * c0 * sizeof(float), 256);
    q.w_off = d.qkv_w_off;
    q.b_off = d.qkv_b_off;
    B.stats(cur, h, w, c0);
    d.steps.push_back(q); B.count_conv(q);
    Step tv; tv.kind = Step::QKV_TRANSPOSE_V; tv.h = h; tv.w = w; tv.cin = c0;
    tv.bytes = 2.0 * h * w * c0 * dtype_size(c.act_dtype);
    d.steps.push_back(tv); d.launches += 1;
    Step f; f.kind = Step::FLASH; f.h = h; f.w = w; f.cin = c0;
    f.flops = 4.0 * (double)(h * w) * (double)(h * w) * c0;
    f.flops_dense = f.flops;
    f.bytes = 4.0 * h * w * c0 * dtype_size(c.act_dtype);
    d.steps.push_back(f); d.launches += 2;
    d.flops += f.flops;
    d.flops_dense += f.flops_dense;
    Step p; p.kind = Step::CONV; p.to_attn = 2; p.dst = other(1); p.res = cur; p.h = h; p.w = w; p.cin = c0; p.cout = c0; p.ksize = 1;
    B.conv_params("mid.attn.proj", c0, c0, 1, &p.w_off, &p.b_off);
    d.steps.push_back(p); B.count_conv(p);
    cur = other(1);
    d.attn_t = h * w; d.attn_tpad = (h * w + 31) / 32 * 32; d.attn_c = c0;
  }
  B.resblock("mid.res2", cur, other(1), other(2), h, w, c0, c0);
  cur = other(2);
  int prev = c0;
  for (int l = 0; l < c.num_levels; ++l) {
    const int ch = c.level_channels[l];
    for (int i = 0; i < c.resblocks_per_level; ++i) {
      char nm[64];
      snprintf(nm, sizeof(nm), "up.%d.res%d", l, i);
      B.resblock(nm, cur, other(1), other(2), h, w, i == 0 ? prev : ch, ch);
      cur = other(2);
    }
    prev = ch;
    if (l + 1 < c.num_levels) {
      char nm[64];
      snprintf(nm, sizeof(nm), "up.%d.upsample", l);
      Step s; s.kind = Step::CONV; s.src = cur; s.dst = other(1); s.h = 2 * h; s.w = 2 * w; s.cin = ch; s.cout = ch; s.upsample = 1;
      B.conv_params(nm, ch, ch, 3, &s.w_off, &s.b_off, true);
      d.steps.push_back(s); B.count_conv(s);
      h *= 2; w *= 2;
      B.track(h, w, ch);
      cur = other(1);
    }
  }
  {  // norm_out -> SiLU -> conv_out, NCHW fp32 frame
    Step s; s.kind = Step::CONV; s.src = cur; s.dst = BUF_OUT; s.h = h; s.w = w; s.cin = prev; s.cout = c.out_c;
    s.norm = 1; s.silu = 1; s.y_nchw = 1;
    B.norm_params("norm_out", prev, &s.gamma_off, &s.beta_off);
    B.conv_params("conv_out", c.out_c, prev, 3, &s.w_off, &s.b_off);
    B.stats(cur, h, w, prev);
    d.steps.push_back(s); B.count_conv(s);
  }
  d.weights_bytes = B.off;
  d.packed_bytes = B.poff;
  if (!c.separate_stats_pass) fuse_stats_into_producers(d);
  return WMDEC_OK;
}

static const Param* find_param(const wmdec_decoder* d, const char* name) {
  for (const Param& p : d->params)
    if (p.name == name) return &p;
  return nullptr;
}

// layout of the workspace for `batch` frames
struct WsLayout {
  size_t tickets, conv_tickets, conv_ticket_bytes, rows[2], act[3], qkv, vt, attn_o, attn_scratch, mean, rstd, stats_ws, stats_ws_bytes, total;
};

static WsLayout ws_layout(const wmdec_decoder* d, int batch) {
  WsLayout L;
  const size_t es = dtype_size(d->cfg.act_dtype);
  const size_t act = align_up(d->act_elems_per_frame * es * batch, 256);
  size_t o = 0;
  L.tickets = o; o += gn_stats_ticket_bytes(d->cfg.max_batch);   // same place and size for every batch: zeroed once
  // ticket counters and row moments of the convolutions that hand their statistics over without a merge launch (sized
  // for max_batch, like the counters above: they are zeroed once per workspace and return to zero by themselves)
  size_t max_tickets = 0, max_rows = 0;
  for (const Step& st : d->steps) {
    if (st.kind != Step::CONV || st.emit_rows < 0) continue;
    int rows = 0, ctiles = 0, per_row = 0;
    if (st.emit_direct) { rows = conv_stats_slots(step_shape_args(*d, st, 1)); ctiles = 0; }
    else conv_mfma_row_extents(step_shape_args(*d, st, 1), &rows, &ctiles, &per_row);
    if ((size_t)rows * ctiles > max_tickets) max_tickets = (size_t)rows * ctiles;
    if ((size_t)rows > max_rows) max_rows = rows;
  }
  L.conv_ticket_bytes = align_up(max_tickets * d->cfg.max_batch * sizeof(unsigned), 256);
  L.conv_tickets = o; o += L.conv_ticket_bytes;
  for (int i = 0; i < 2; ++i) { L.rows[i] = o; o += align_up(max_rows * d->cfg.max_batch * d->cfg.groups * 3 * sizeof(float), 256); }
  for (int i = 0; i < 3; ++i) { L.act[i] = o; o += act; }
  L.qkv = o; o += align_up((size_t)batch * d->attn_t * 3 * d->attn_c * es, 256);
  L.vt = o; o += align_up((size_t)batch * flash_attention_vt_elems(d->attn_t, d->attn_c) * es, 256);
  L.attn_o = o; o += align_up((size_t)batch * d->attn_t * d->attn_c * es, 256);
  L.attn_scratch = o; o += align_up(flash_attention_scratch_bytes(batch, d->attn_t, d->attn_c), 256);
  L.mean = o; o += align_up((size_t)batch * d->cfg.groups * sizeof(float), 256);
  L.rstd = o; o += align_up((size_t)batch * d->cfg.groups * sizeof(float), 256);
  L.stats_ws_bytes = gn_stats_moments_bytes(batch, d->cfg.groups);
  for (const Step& st : d->steps) {
    if (st.kind != Step::CONV || !st.emit_stats) continue;
    const size_t need = (size_t)batch * d->cfg.groups * conv_stats_slots(step_shape_args(*d, st, batch)) * 3 * sizeof(float);
    if (need > L.stats_ws_bytes) L.stats_ws_bytes = need;
  }
  L.stats_ws = o; o += align_up(L.stats_ws_bytes, 256);
  L.total = o;
  return L;
}

}  // namespace wmdec

// =====================================================================  C ABI
extern "C" {

const char* wmdec_last_error(void) { return g_err; }

const char* wmdec_status_string(int status) {
  switch (status) {
    case WMDEC_OK: return "ok";
    case WMDEC_ERR_INVALID_ARG: return "invalid argument";
    case WMDEC_ERR_UNSUPPORTED: return "unsupported";
    case WMDEC_ERR_SHAPE: return "inconsistent shape";
    case WMDEC_ERR_WORKSPACE: return "workspace missing or too small";
    case WMDEC_ERR_HIP: return "HIP failure";
    default: return "unknown status";
  }
}

size_t wmdec_gn_stats_workspace_bytes(int n, int h, int w, int c, int groups) {
  if (n <= 0 || h <= 0 || w <= 0 || c <= 0 || groups <= 0) return 0;
  (void)h; (void)w; (void)c;
  return gn_stats_ticket_bytes(n) + gn_stats_moments_bytes(n, groups);
}

int wmdec_gn_stats(const void* x, int x_dtype, int n, int h, int w, int c, int groups, float eps, float* mean,
                   float* rstd, void* workspace, size_t workspace_bytes, void* stream) {
  WMDEC_REQUIRE(x && mean && rstd, WMDEC_ERR_INVALID_ARG, "gn_stats: null pointer");
  WMDEC_REQUIRE(valid_dtype(x_dtype), WMDEC_ERR_INVALID_ARG, "gn_stats: bad dtype %d", x_dtype);
  WMDEC_REQUIRE(n > 0 && h > 0 && w > 0 && c > 0 && groups > 0, WMDEC_ERR_INVALID_ARG, "gn_stats: non-positive size");
  WMDEC_REQUIRE(c % groups == 0, WMDEC_ERR_SHAPE, "gn_stats: c %d not divisible by groups %d", c, groups);
  WMDEC_REQUIRE(eps >= 0.f, WMDEC_ERR_INVALID_ARG, "gn_stats: negative eps");
  WMDEC_REQUIRE(aligned16(x) && aligned16(workspace), WMDEC_ERR_INVALID_ARG, "gn_stats: pointers must be 16-byte aligned");
  const size_t head = gn_stats_ticket_bytes(n);
  WMDEC_REQUIRE(workspace && workspace_bytes > head, WMDEC_ERR_WORKSPACE, "gn_stats: workspace of %zu bytes is too small", workspace_bytes);
  return launch_gn_stats(x, x_dtype, n, h, w, c, groups, eps, mean, rstd, (unsigned*)workspace, (char*)workspace + head,
                         workspace_bytes - head, (hipStream_t)stream);
}

int wmdec_gn_stats_noalloc(const void* x, int x_dtype, int n, int h, int w, int c, int groups, float eps, float* mean,
                           float* rstd, void* stream) {
  WMDEC_REQUIRE(x && mean && rstd, WMDEC_ERR_INVALID_ARG, "gn_stats_noalloc: null pointer");
  WMDEC_REQUIRE(valid_dtype(x_dtype), WMDEC_ERR_INVALID_ARG, "gn_stats_noalloc: bad dtype %d", x_dtype);
  WMDEC_REQUIRE(n > 0 && h > 0 && w > 0 && c > 0 && groups > 0, WMDEC_ERR_INVALID_ARG, "gn_stats_noalloc: non-positive size");
  WMDEC_REQUIRE(c % groups == 0, WMDEC_ERR_SHAPE, "gn_stats_noalloc: c %d not divisible by groups %d", c, groups);
  WMDEC_REQUIRE(eps >= 0.f, WMDEC_ERR_INVALID_ARG, "gn_stats_noalloc: negative eps");
  WMDEC_REQUIRE(aligned16(x), WMDEC_ERR_INVALID_ARG, "gn_stats_noalloc: x must be 16-byte aligned");
  return launch_gn_stats_static(x, x_dtype, n, h, w, c, groups, eps, mean, rstd, (hipStream_t)stream);
}

size_t wmdec_conv_packed_bytes(int cout, int cin, int k, int op_dtype) {
  if (cout <= 0 || cin <= 0 || (k != 1 && k != 3) || !valid_dtype(op_dtype)) return 0;
  return packed_elems(k * k, cout, cin) * dtype_size(op_dtype);
}

int wmdec_pack_conv_weights(const void* src, int src_dtype, int cout, int cin, int k, void* packed, int op_dtype,
                            void* stream) {
  WMDEC_REQUIRE(src && packed, WMDEC_ERR_INVALID_ARG, "pack_conv_weights: null pointer");
  WMDEC_REQUIRE(src_dtype == WMDEC_F32 || src_dtype == WMDEC_BF16, WMDEC_ERR_UNSUPPORTED,
                "pack_conv_weights: source must be F32 or BF16");
  WMDEC_REQUIRE(valid_dtype(op_dtype), WMDEC_ERR_INVALID_ARG, "pack_conv_weights: bad op_dtype");
  WMDEC_REQUIRE(cout > 0 && cin > 0 && (k == 1 || k == 3), WMDEC_ERR_INVALID_ARG, "pack_conv_weights: bad shape");
  return launch_pack_conv(src, src_dtype, cout, cin, k, packed, op_dtype, 0, cout, (hipStream_t)stream);
}

size_t wmdec_upconv_packed_bytes(int cout, int cin, int op_dtype) {
  if (cout <= 0 || cin <= 0 || !valid_dtype(op_dtype)) return 0;
  return upconv_packed_bytes(cout, cin, op_dtype);
}

int wmdec_pack_upconv_weights(const void* src, int src_dtype, int cout, int cin, void* packed, int op_dtype, void* stream) {
  WMDEC_REQUIRE(src && packed, WMDEC_ERR_INVALID_ARG, "pack_upconv_weights: null pointer");
  WMDEC_REQUIRE(src_dtype == WMDEC_F32 || src_dtype == WMDEC_BF16, WMDEC_ERR_INVALID_ARG,
                "pack_upconv_weights: source must be F32 or BF16");
  WMDEC_REQUIRE(valid_dtype(op_dtype), WMDEC_ERR_INVALID_ARG, "pack_upconv_weights: bad op_dtype");
  WMDEC_REQUIRE(cout > 0 && cin > 0, WMDEC_ERR_INVALID_ARG, "pack_upconv_weights: bad shape");
  WMDEC_REQUIRE(aligned16(packed), WMDEC_ERR_INVALID_ARG, "pack_upconv_weights: packed must be 16-byte aligned");
  return launch_pack_upconv(src, src_dtype, cout, cin, packed, op_dtype, (hipStream_t)stream);
}

static int conv_entry(const char* who, int ksize, int upsample, const void* x, int act_dtype, const float* mean,
                      const float* rstd, const float* gamma, const float* beta, int groups, int apply_silu,
                      const void* w_packed, const float* bias, const void* residual, void* y, int y_dtype, int n,
                      int h_out, int w_out, int cin, int cout, void* stream) {
  const int rc = check_conv(who, x, act_dtype, mean, rstd, gamma, beta, groups, w_packed, residual, y, y_dtype, n,
                            h_out, w_out, cin, cout);
  if (rc != WMDEC_OK) return rc;
  ConvArgs a;
  a.x = x; a.x_dtype = act_dtype; a.mean = mean; a.rstd = mean ? rstd : nullptr; a.gamma = gamma; a.beta = beta;
  a.groups = mean ? groups : 1; a.silu = (mean && apply_silu) ? 1 : 0;
  a.wt = w_packed; a.op_dtype = act_dtype; a.bias = bias; a.res = residual; a.res_dtype = act_dtype;
  a.y = y; a.y_dtype = y_dtype; a.n = n; a.h = h_out; a.w = w_out; a.cin = cin; a.cout = cout;
  a.ksize = ksize; a.upsample = upsample;
  if (upsample) a.wt_phase = (const char*)w_packed + upconv_phase_offset_bytes(cout, cin, act_dtype);
  return launch_conv(a, (hipStream_t)stream);
}

int wmdec_gn_silu_conv3x3(const void* x, int act_dtype, const float* mean, const float* rstd, const float* gamma,
                          const float* beta, int groups, int apply_silu, const void* w_packed, const float* bias,
                          const void* residual, void* y, int y_dtype, int n, int h, int w, int cin, int cout,
                          void* stream) {
  return conv_entry("gn_silu_conv3x3", 3, 0, x, act_dtype, mean, rstd, gamma, beta, groups, apply_silu, w_packed, bias,
                    residual, y, y_dtype, n, h, w, cin, cout, stream);
}

int wmdec_gn_silu_conv3x3_shortcut(const void* x, int act_dtype, const float* mean, const float* rstd, const float* gamma,
                                   const float* beta, int groups, int apply_silu, const void* w_packed, const float* bias,
                                   const void* x2, int cin2, const void* w2_packed, const float* bias2, void* y, int y_dtype,
                                   int n, int h, int w, int cin, int cout, void* stream) {
  const char* who = "gn_silu_conv3x3_shortcut";
  const int rc = check_conv(who, x, act_dtype, mean, rstd, gamma, beta, groups, w_packed, nullptr, y, y_dtype, n, h, w, cin, cout);
  if (rc != WMDEC_OK) return rc;
  WMDEC_REQUIRE(x2 && w2_packed && cin2 > 0, WMDEC_ERR_INVALID_ARG, "%s: null shortcut input or weights, or cin2 <= 0", who);
  WMDEC_REQUIRE(aligned16(x2) && aligned16(w2_packed), WMDEC_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
  WMDEC_REQUIRE(x2 != y, WMDEC_ERR_INVALID_ARG, "%s: x2 and y must not overlap", who);
  ConvArgs a;
  a.x = x; a.x_dtype = act_dtype; a.mean = mean; a.rstd = mean ? rstd : nullptr; a.gamma = gamma; a.beta = beta;
  a.groups = mean ? groups : 1; a.silu = (mean && apply_silu) ? 1 : 0;
  a.wt = w_packed; a.op_dtype = act_dtype; a.bias = bias; a.res_dtype = act_dtype;
  a.y = y; a.y_dtype = y_dtype; a.n = n; a.h = h; a.w = w; a.cin = cin; a.cout = cout; a.ksize = 3;
  if (conv_mfma_supported(a) && cin2 % 32 == 0) {   // one launch: the shortcut is part of the contraction
    a.x2 = x2; a.cin2 = cin2; a.w2 = w2_packed; a.bias2 = bias2;
    return launch_conv(a, (hipStream_t)stream);
  }
  // other shapes and fp32: the shortcut is written to y first, and the convolution adds it from there (every
  // element is read and then written by the same thread)
  ConvArgs sc;
  sc.x = x2; sc.x_dtype = act_dtype; sc.wt = w2_packed; sc.op_dtype = act_dtype; sc.bias = bias2; sc.res_dtype = act_dtype;
  sc.y = y; sc.y_dtype = y_dtype; sc.n = n; sc.h = h; sc.w = w; sc.cin = cin2; sc.cout = cout; sc.ksize = 1;
  const int r1 = launch_conv_direct(sc, (hipStream_t)stream);
  if (r1 != WMDEC_OK) return r1;
  a.res = y; a.res_dtype = y_dtype;
  return launch_conv_direct(a, (hipStream_t)stream);
}

// shape-only arguments of a 3x3 launch that also emits the moments of its output
static ConvArgs stats_conv_shape(int act_dtype, int y_dtype, int n, int h, int w, int cin, int cout, int out_groups) {
  ConvArgs a;
  a.x_dtype = act_dtype; a.op_dtype = act_dtype; a.res_dtype = act_dtype; a.y_dtype = y_dtype;
  a.n = n; a.h = h; a.w = w; a.cin = cin; a.cout = cout; a.ksize = 3; a.stats_groups = out_groups;
  return a;
}

size_t wmdec_conv_stats_workspace_bytes(int act_dtype, int y_dtype, int n, int h, int w, int cin, int cout, int out_groups) {
  if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || cout <= 0 || out_groups <= 0 || !valid_dtype(act_dtype) || !valid_dtype(y_dtype)) return 0;
  const int slots = conv_stats_slots(stats_conv_shape(act_dtype, y_dtype, n, h, w, cin, cout, out_groups));
  return (size_t)n * out_groups * slots * 3 * sizeof(float);
}

int wmdec_gn_silu_conv3x3_stats(const void* x, int act_dtype, const float* mean, const float* rstd, const float* gamma,
                                const float* beta, int groups, int apply_silu, const void* w_packed, const float* bias,
                                const void* residual, void* y, int y_dtype, int n, int h, int w, int cin, int cout,
                                int out_groups, float out_eps, float* mean_out, float* rstd_out, void* workspace,
                                size_t workspace_bytes, void* stream) {
  const char* who = "gn_silu_conv3x3_stats";
  const int rc = check_conv(who, x, act_dtype, mean, rstd, gamma, beta, groups, w_packed, residual, y, y_dtype, n, h, w, cin, cout);
  if (rc != WMDEC_OK) return rc;
  WMDEC_REQUIRE(mean_out && rstd_out, WMDEC_ERR_INVALID_ARG, "%s: null output statistics", who);
  WMDEC_REQUIRE(out_groups > 0 && cout % out_groups == 0, WMDEC_ERR_SHAPE, "%s: cout %d not divisible by out_groups %d", who, cout, out_groups);
  WMDEC_REQUIRE(out_eps >= 0.f, WMDEC_ERR_INVALID_ARG, "%s: negative eps", who);
  ConvArgs a = stats_conv_shape(act_dtype, y_dtype, n, h, w, cin, cout, out_groups);
  a.x = x; a.mean = mean; a.rstd = mean ? rstd : nullptr; a.gamma = gamma; a.beta = beta;
  a.groups = mean ? groups : 1; a.silu = (mean && apply_silu) ? 1 : 0;
  a.wt = w_packed; a.bias = bias; a.res = residual; a.y = y;
  const int slots = conv_stats_slots(a);
  WMDEC_REQUIRE(slots > 0, WMDEC_ERR_UNSUPPORTED,
                "%s: this shape / type takes no kernel that emits moments (16-bit types and either cin %% 32 == 0, cout %% 64 == 0, "
                "channels per output group a power of two <= 32, or cin <= 8 without normalisation and residual, channels per "
                "output group a power of two <= 64); use wmdec_gn_stats on y", who);
  const size_t need = (size_t)n * out_groups * slots * 3 * sizeof(float);
  WMDEC_REQUIRE(workspace && aligned16(workspace) && workspace_bytes >= need, WMDEC_ERR_WORKSPACE,
                "%s: workspace needs %zu bytes, got %zu", who, need, workspace_bytes);
  a.stats_ws = workspace;
  const int rl = launch_conv(a, (hipStream_t)stream);
  if (rl != WMDEC_OK) return rl;
  return launch_gn_finalize(workspace, n * out_groups, slots, out_eps, mean_out, rstd_out, (hipStream_t)stream);
}

int wmdec_gn_conv1x1(const void* x, int act_dtype, const float* mean, const float* rstd, const float* gamma,
                     const float* beta, int groups, int apply_silu, const void* w_packed, const float* bias,
                     const void* residual, void* y, int y_dtype, int n, int h, int w, int cin, int cout, void* stream) {
  return conv_entry("gn_conv1x1", 1, 0, x, act_dtype, mean, rstd, gamma, beta, groups, apply_silu, w_packed, bias,
                    residual, y, y_dtype, n, h, w, cin, cout, stream);
}

int wmdec_upsample2x_conv3x3(const void* x, int act_dtype, const void* w_packed, const float* bias, void* y,
                             int y_dtype, int n, int h_in, int w_in, int cin, int cout, void* stream) {
  WMDEC_REQUIRE(h_in > 0 && w_in > 0 && h_in < (1 << 14) && w_in < (1 << 14), WMDEC_ERR_INVALID_ARG,
                "upsample2x_conv3x3: bad input size");
  return conv_entry("upsample2x_conv3x3", 3, 1, x, act_dtype, nullptr, nullptr, nullptr, nullptr, 1, 0, w_packed, bias,
                    nullptr, y, y_dtype, n, 2 * h_in, 2 * w_in, cin, cout, stream);
}

int wmdec_measure_copy(const void* src, void* dst, size_t bytes, void* stream) {
  WMDEC_REQUIRE(src && dst, WMDEC_ERR_INVALID_ARG, "measure_copy: null pointer");
  WMDEC_REQUIRE(aligned16(src) && aligned16(dst) && bytes % 16 == 0, WMDEC_ERR_INVALID_ARG,
                "measure_copy: pointers and byte count must be multiples of 16");
  const char* a = (const char*)src; const char* b = (const char*)dst;
  WMDEC_REQUIRE(a + bytes <= b || b + bytes <= a, WMDEC_ERR_INVALID_ARG, "measure_copy: src and dst must not overlap");
  return launch_copy_u128(src, dst, bytes, (hipStream_t)stream);
}

int wmdec_upsample2x_nearest(const void* x, void* y, int dtype, int n, int h_in, int w_in, int c, void* stream) {
  WMDEC_REQUIRE(x && y, WMDEC_ERR_INVALID_ARG, "upsample2x_nearest: null pointer");
  WMDEC_REQUIRE(valid_dtype(dtype), WMDEC_ERR_INVALID_ARG, "upsample2x_nearest: bad dtype");
  WMDEC_REQUIRE(n > 0 && h_in > 0 && w_in > 0 && c > 0, WMDEC_ERR_INVALID_ARG, "upsample2x_nearest: non-positive size");
  WMDEC_REQUIRE(aligned16(x) && aligned16(y), WMDEC_ERR_INVALID_ARG, "upsample2x_nearest: pointers must be 16-byte aligned");
  WMDEC_REQUIRE(x != y, WMDEC_ERR_INVALID_ARG, "upsample2x_nearest: x and y must not overlap");
  return launch_upsample2x(x, y, dtype, n, h_in, w_in, c, (hipStream_t)stream);
}

static int layout_entry(const char* who, bool to_nhwc, const void* src, int sd, void* dst, int dd, int n, int c, int h,
                        int w, void* stream) {
  WMDEC_REQUIRE(src && dst && src != dst, WMDEC_ERR_INVALID_ARG, "%s: null or aliased pointers", who);
  WMDEC_REQUIRE(valid_dtype(sd) && valid_dtype(dd), WMDEC_ERR_INVALID_ARG, "%s: bad dtype", who);
  WMDEC_REQUIRE(n > 0 && c > 0 && h > 0 && w > 0, WMDEC_ERR_INVALID_ARG, "%s: non-positive size", who);
  const size_t p = (size_t)h * w;
  // NCHW is [c][p] per sample, NHWC is [p][c]
  if (to_nhwc) return launch_transpose(src, sd, dst, dd, n, c, (int)p, p, p * c, (size_t)c, p * c, (hipStream_t)stream);
  return launch_transpose(src, sd, dst, dd, n, (int)p, c, (size_t)c, p * c, p, p * c, (hipStream_t)stream);
}

int wmdec_nchw_to_nhwc(const void* src, int sd, void* dst, int dd, int n, int c, int h, int w, void* stream) {
  return layout_entry("nchw_to_nhwc", true, src, sd, dst, dd, n, c, h, w, stream);
}
int wmdec_nhwc_to_nchw(const void* src, int sd, void* dst, int dd, int n, int c, int h, int w, void* stream) {
  return layout_entry("nhwc_to_nchw", false, src, sd, dst, dd, n, c, h, w, stream);
}

// ---- attention
static void attn_ws_layout(int n, int t, int c, size_t es, size_t* qkv, size_t* vt, size_t* o, size_t* scratch, size_t* total) {
  size_t off = 0;
  *qkv = off; off += align_up((size_t)n * t * 3 * c * es, 256);
  *vt = off; off += align_up((size_t)n * flash_attention_vt_elems(t, c) * es, 256);
  *o = off; off += align_up((size_t)n * t * c * es, 256);
  *scratch = off; off += align_up(flash_attention_scratch_bytes(n, t, c), 256);
  *total = off;
}

size_t wmdec_attention_workspace_bytes(int n, int h, int w, int c) {
  if (n <= 0 || h <= 0 || w <= 0 || c <= 0) return 0;
  size_t a, b, d, e, total;
  attn_ws_layout(n, h * w, c, 2, &a, &b, &d, &e, &total);
  return total;
}

static int attention_impl(const void* x, int act_dtype, const float* mean, const float* rstd, const float* gamma,
                          const float* beta, int groups, const void* wqkv, const float* bqkv, const void* wo,
                          const float* bo, void* y, int n, int h, int w, int c, void* qkv, void* vt, void* ob,
                          void* scratch, hipStream_t s) {
  const int t = h * w, tpad = (t + 31) / 32 * 32;
  const size_t es = 2;
  ConvArgs a;
  a.x = x; a.x_dtype = act_dtype; a.mean = mean; a.rstd = rstd; a.gamma = gamma; a.beta = beta; a.groups = groups; a.silu = 0;
  a.wt = wqkv; a.op_dtype = act_dtype; a.bias = bqkv; a.y = qkv; a.y_dtype = act_dtype;
  a.n = n; a.h = h; a.w = w; a.cin = c; a.cout = 3 * c; a.ksize = 1;
  int rc = launch_conv(a, s);
  if (rc != WMDEC_OK) return rc;
  // V^T[n][d][key]: transpose the v columns of the qkv buffer
  rc = launch_transpose((const char*)qkv + (size_t)2 * c * es, act_dtype, vt, act_dtype, n, t, c, (size_t)3 * c,
                        (size_t)t * 3 * c, 0 /* blocks of 32 keys */, flash_attention_vt_elems(t, c), s);
  if (rc != WMDEC_OK) return rc;
  rc = launch_flash_attention(qkv, (const char*)qkv + (size_t)c * es, (size_t)3 * c, (size_t)t * 3 * c, vt, tpad, ob,
                              scratch, act_dtype, n, t, c, 1.0f / sqrtf((float)c), s);
  if (rc != WMDEC_OK) return rc;
  ConvArgs p;
  p.x = ob; p.x_dtype = act_dtype; p.wt = wo; p.op_dtype = act_dtype; p.bias = bo; p.res = x; p.res_dtype = act_dtype;
  p.y = y; p.y_dtype = act_dtype; p.n = n; p.h = h; p.w = w; p.cin = c; p.cout = c; p.ksize = 1;
  return launch_conv(p, s);
}

int wmdec_attention(const void* x, int act_dtype, const float* mean, const float* rstd, const float* gamma,
                    const float* beta, int groups, const void* wqkv_packed, const float* bqkv, const void* wo_packed,
                    const float* bo, void* y, int n, int h, int w, int c, void* workspace, size_t workspace_bytes,
                    void* stream) {
  WMDEC_REQUIRE(x && mean && rstd && gamma && beta && wqkv_packed && bqkv && wo_packed && bo && y,
                WMDEC_ERR_INVALID_ARG, "attention: null pointer");
  WMDEC_REQUIRE(is_16bit(act_dtype), WMDEC_ERR_UNSUPPORTED, "attention: act_dtype must be BF16 or F16");
  WMDEC_REQUIRE(n > 0 && h > 0 && w > 0, WMDEC_ERR_INVALID_ARG, "attention: non-positive size");
  WMDEC_REQUIRE(c == 512, WMDEC_ERR_UNSUPPORTED, "attention: c must be 512 (got %d)", c);
  WMDEC_REQUIRE(groups > 0 && c % groups == 0, WMDEC_ERR_SHAPE, "attention: c %d not divisible by groups %d", c, groups);
  WMDEC_REQUIRE(x != y, WMDEC_ERR_INVALID_ARG, "attention: x and y must not overlap");
  WMDEC_REQUIRE(aligned16(x) && aligned16(y) && aligned16(workspace) && aligned16(wqkv_packed) && aligned16(wo_packed),
                WMDEC_ERR_INVALID_ARG, "attention: pointers must be 16-byte aligned");
  size_t qo, vo, oo, so, total;
  attn_ws_layout(n, h * w, c, 2, &qo, &vo, &oo, &so, &total);
  WMDEC_REQUIRE(workspace && workspace_bytes >= total, WMDEC_ERR_WORKSPACE, "attention: workspace needs %zu bytes, got %zu",
                total, workspace_bytes);
  char* ws = (char*)workspace;
  return attention_impl(x, act_dtype, mean, rstd, gamma, beta, groups, wqkv_packed, bqkv, wo_packed, bo, y, n, h, w, c,
                        ws + qo, ws + vo, ws + oo, ws + so, (hipStream_t)stream);
}

// ---- horizontally fused AdaLN projections
int wmdec_adaln_max_batch(int d_cond) { return adaln_max_batch(d_cond); }

int wmdec_adaln_fused_projection(const void* c, int c_dtype, const void* w_fused, int w_dtype, const float* bias, float* out,
                                 int batch, int d_cond, int rows, int apply_silu, void* stream) {
  WMDEC_REQUIRE(c && w_fused && out, WMDEC_ERR_INVALID_ARG, "adaln_fused_projection: null pointer");
  WMDEC_REQUIRE(valid_dtype(c_dtype) && valid_dtype(w_dtype), WMDEC_ERR_INVALID_ARG, "adaln_fused_projection: bad dtype");
  WMDEC_REQUIRE(batch > 0 && d_cond > 0 && rows > 0, WMDEC_ERR_INVALID_ARG, "adaln_fused_projection: non-positive size");
  WMDEC_REQUIRE(aligned16(c) && aligned16(w_fused) && aligned16(out), WMDEC_ERR_INVALID_ARG, "adaln_fused_projection: pointers must be 16-byte aligned");
  WMDEC_REQUIRE(d_cond % (int)(16 / dtype_size(w_dtype)) == 0 && d_cond % (int)(16 / dtype_size(c_dtype)) == 0, WMDEC_ERR_SHAPE,
                "adaln_fused_projection: d_cond %d must be a multiple of 8 for 16-bit operands and of 4 for F32 (16-byte vectors)", d_cond);
  WMDEC_REQUIRE(d_cond <= adaln_max_d_cond(w_dtype), WMDEC_ERR_UNSUPPORTED, "adaln_fused_projection: d_cond %d above the limit of %d for this weight type",
                d_cond, adaln_max_d_cond(w_dtype));
  WMDEC_REQUIRE(batch <= adaln_max_batch(d_cond), WMDEC_ERR_UNSUPPORTED,
                "adaln_fused_projection: at most %d conditioning vectors of length %d per call (they are held in LDS); "
                "larger batches are a GEMM: use wmdec_gn_conv1x1 on a [1,1,batch,d_cond] tensor", adaln_max_batch(d_cond), d_cond);
  return launch_adaln_projection(c, c_dtype, w_fused, w_dtype, bias, out, batch, d_cond, rows, apply_silu ? 1 : 0, (hipStream_t)stream);
}

// ---- decoder
void decoder_default_config(wmdec_decoder_config* cfg) {
  if (!cfg) return;
  memset(cfg, 0, sizeof(*cfg));
  cfg->latent_c = 4; cfg->latent_h = 60; cfg->latent_w = 90;
  cfg->num_levels = 4;
  cfg->level_channels[0] = 512; cfg->level_channels[1] = 512; cfg->level_channels[2] = 256; cfg->level_channels[3] = 128;
  cfg->resblocks_per_level = 3;
  cfg->groups = 32; cfg->eps = 1e-6f; cfg->out_c = 3;
  cfg->act_dtype = WMDEC_F16; cfg->max_batch = 4;
  cfg->latent_dtype = WMDEC_BF16; cfg->separate_stats_pass = 0; cfg->separate_shortcut = 0; cfg->separate_merge_launch = 0;
}

int decoder_create(const wmdec_decoder_config* cfg, wmdec_decoder** out) {
  WMDEC_REQUIRE(cfg && out, WMDEC_ERR_INVALID_ARG, "decoder_create: null pointer");
  *out = nullptr;
  WMDEC_REQUIRE(cfg->latent_c > 0 && cfg->latent_h > 0 && cfg->latent_w > 0 && cfg->out_c > 0, WMDEC_ERR_INVALID_ARG,
                "decoder_create: non-positive size");
  WMDEC_REQUIRE(cfg->num_levels >= 1 && cfg->num_levels <= 4, WMDEC_ERR_INVALID_ARG, "decoder_create: num_levels must be 1..4");
  WMDEC_REQUIRE(cfg->resblocks_per_level >= 1 && cfg->resblocks_per_level <= 16, WMDEC_ERR_INVALID_ARG,
                "decoder_create: resblocks_per_level must be 1..16");
  WMDEC_REQUIRE(cfg->groups > 0, WMDEC_ERR_INVALID_ARG, "decoder_create: groups must be positive");
  for (int l = 0; l < cfg->num_levels; ++l)
    WMDEC_REQUIRE(cfg->level_channels[l] > 0 && cfg->level_channels[l] % cfg->groups == 0, WMDEC_ERR_SHAPE,
                  "decoder_create: level %d has %d channels, not a multiple of %d groups", l, cfg->level_channels[l], cfg->groups);
  WMDEC_REQUIRE(cfg->level_channels[0] == 512, WMDEC_ERR_UNSUPPORTED,
                "decoder_create: the mid-block attention needs 512 channels at level 0");
  WMDEC_REQUIRE(is_16bit(cfg->act_dtype), WMDEC_ERR_UNSUPPORTED, "decoder_create: act_dtype must be BF16 or F16");
  WMDEC_REQUIRE(cfg->max_batch >= 1 && cfg->max_batch <= 64, WMDEC_ERR_INVALID_ARG, "decoder_create: max_batch must be 1..64");
  WMDEC_REQUIRE(cfg->eps >= 0.f, WMDEC_ERR_INVALID_ARG, "decoder_create: negative eps");
  WMDEC_REQUIRE(valid_dtype(cfg->latent_dtype), WMDEC_ERR_INVALID_ARG, "decoder_create: bad latent_dtype %d", cfg->latent_dtype);
  wmdec_decoder* d = new (std::nothrow) wmdec_decoder();
  WMDEC_REQUIRE(d, WMDEC_ERR_INVALID_ARG, "decoder_create: out of host memory");
  d->cfg = *cfg;
  const int rc = build_plan(*d);
  if (rc != WMDEC_OK) { delete d; return rc; }
  *out = d;
  return WMDEC_OK;
}

int decoder_destroy(wmdec_decoder* dec) {
  delete dec;
  return WMDEC_OK;
}

size_t decoder_weights_bytes(const wmdec_decoder* dec) { return dec ? dec->weights_bytes : 0; }
size_t decoder_packed_bytes(const wmdec_decoder* dec) { return dec ? dec->packed_bytes : 0; }
int decoder_num_weights(const wmdec_decoder* dec) { return dec ? (int)dec->params.size() : 0; }
int decoder_num_launches(const wmdec_decoder* dec) { return dec ? dec->launches : 0; }
double decoder_flops_per_frame(const wmdec_decoder* dec) { return dec ? dec->flops : 0.0; }
double decoder_dense_flops_per_frame(const wmdec_decoder* dec) { return dec ? dec->flops_dense : 0.0; }

int decoder_weight_info(const wmdec_decoder* dec, int index, const char** name, size_t* offset, size_t* bytes,
                        int* dtype, int shape[4]) {
  WMDEC_REQUIRE(dec, WMDEC_ERR_INVALID_ARG, "decoder_weight_info: null decoder");
  WMDEC_REQUIRE(index >= 0 && index < (int)dec->params.size(), WMDEC_ERR_INVALID_ARG, "decoder_weight_info: index %d out of range", index);
  const Param& p = dec->params[index];
  if (name) *name = p.name.c_str();
  if (offset) *offset = p.offset;
  if (bytes) *bytes = p.bytes;
  if (dtype) *dtype = p.dtype;
  if (shape) memcpy(shape, p.shape, sizeof(p.shape));
  return WMDEC_OK;
}

int decoder_weight_offset(const wmdec_decoder* dec, const char* name, size_t* offset, size_t* bytes) {
  WMDEC_REQUIRE(dec && name, WMDEC_ERR_INVALID_ARG, "decoder_weight_offset: null pointer");
  const Param* p = find_param(dec, name);
  WMDEC_REQUIRE(p, WMDEC_ERR_INVALID_ARG, "decoder_weight_offset: no parameter named '%s'", name);
  if (offset) *offset = p->offset;
  if (bytes) *bytes = p->bytes;
  return WMDEC_OK;
}

int decoder_pack_weights(const wmdec_decoder* dec, const void* weights, void* packed, void* stream) {
  WMDEC_REQUIRE(dec && weights && packed, WMDEC_ERR_INVALID_ARG, "decoder_pack_weights: null pointer");
  WMDEC_REQUIRE(aligned16(weights) && aligned16(packed), WMDEC_ERR_INVALID_ARG, "decoder_pack_weights: pointers must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const char* src = (const char*)weights;
  char* dst = (char*)packed;
  const int c0 = dec->cfg.level_channels[0];
  for (const Param& p : dec->params) {
    int rc;
    const int part = p.name.compare(0, 11, "mid.attn.q.") == 0 ? 0
                     : p.name.compare(0, 11, "mid.attn.k.") == 0 ? 1
                     : p.name.compare(0, 11, "mid.attn.v.") == 0 ? 2 : -1;
    if (part >= 0 && p.dtype == WMDEC_F32) {
      rc = launch_copy_f32((const float*)(src + p.offset), (float*)(dst + dec->qkv_b_off) + part * c0, (size_t)c0, s);
    } else if (part >= 0) {
      // q, k, v become rows [0,c), [c,2c), [2c,3c) of the fused [3c][c] matrix
      rc = launch_pack_conv(src + p.offset, p.dtype, c0, c0, 1, dst + dec->qkv_w_off, dec->cfg.act_dtype, part * c0, 3 * c0, s);
    } else if (p.dtype == WMDEC_F32) {
      rc = launch_copy_f32((const float*)(src + p.offset), (float*)(dst + p.packed_offset), p.bytes / 4, s);
    } else if (p.upconv) {
      rc = launch_pack_upconv(src + p.offset, p.dtype, p.shape[0], p.shape[1], dst + p.packed_offset, dec->cfg.act_dtype, s);
    } else {
      rc = launch_pack_conv(src + p.offset, p.dtype, p.shape[0], p.shape[1], p.shape[2], dst + p.packed_offset,
                            dec->cfg.act_dtype, 0, p.shape[0], s);
    }
    if (rc != WMDEC_OK) return rc;
  }
  return WMDEC_OK;
}

size_t decoder_workspace_bytes(const wmdec_decoder* dec, int batch) {
  if (!dec || batch < 1 || batch > dec->cfg.max_batch) return 0;
  return ws_layout(dec, batch).total;
}

int decoder_set_workspace(wmdec_decoder* dec, void* workspace, size_t bytes) {
  WMDEC_REQUIRE(dec && workspace, WMDEC_ERR_INVALID_ARG, "decoder_set_workspace: null pointer");
  WMDEC_REQUIRE(aligned16(workspace), WMDEC_ERR_INVALID_ARG, "decoder_set_workspace: workspace must be 16-byte aligned");
  dec->ws = workspace;
  dec->ws_bytes = bytes;
  dec->ws_fresh = true;
  return WMDEC_OK;
}

// enqueues one step of the plan; *emitted_slots carries the slot count of the last emitting convolution
// the latent of a run: either `z` holds one latent per frame, or (step != null) frame i is z[0] + (i + 1) * scale * step
struct LatentSource { const void* z; const void* step; float scale; };

static int launch_step(wmdec_decoder* dec, const WsLayout& L, const Step& st, const LatentSource& latent, const void* packed,
                       void* out, int batch, int* emitted_slots, hipStream_t s) {
  char* ws = (char*)dec->ws;
  const char* pk = (const char*)packed;
  const wmdec_decoder_config& c = dec->cfg;
  float* mean = (float*)(ws + L.mean);
  float* rstd = (float*)(ws + L.rstd);
  auto buf = [&](int id) -> void* { return id >= 0 ? (void*)(ws + L.act[id]) : nullptr; };
  {
    int rc = WMDEC_OK;
    switch (st.kind) {
      case Step::STATS:
        if (st.from_producer && (*emitted_slots) > 0)
          rc = launch_gn_finalize(ws + L.stats_ws, batch * c.groups, (*emitted_slots), c.eps, mean, rstd, s);
        else
          rc = launch_gn_stats(buf(st.src), c.act_dtype, batch, st.h, st.w, st.cin, c.groups, c.eps, mean, rstd,
                               (unsigned*)(ws + L.tickets), ws + L.stats_ws, L.stats_ws_bytes, s);
        break;
      case Step::CONV: {
        ConvArgs a;
        a.op_dtype = c.act_dtype; a.res_dtype = c.act_dtype;
        if (st.src == BUF_LATENT) { a.x = latent.z; a.x_dtype = c.latent_dtype; a.x_nchw = 1; a.x_step = latent.step; a.step_scale = latent.scale; }
        else if (st.to_attn == 2) { a.x = ws + L.attn_o; a.x_dtype = c.act_dtype; }
        else { a.x = buf(st.src); a.x_dtype = c.act_dtype; }
        if (st.norm) {
          a.gamma = (const float*)(pk + st.gamma_off); a.beta = (const float*)(pk + st.beta_off); a.groups = c.groups; a.silu = st.silu;
          if (st.rows_from >= 0) { a.rows_in = ws + L.rows[st.rows_from]; a.rows_in_count = st.rows_count; a.eps = c.eps; }
          else { a.mean = mean; a.rstd = rstd; }
        }
        a.wt = pk + st.w_off; a.bias = (const float*)(pk + st.b_off);
        if (st.upsample) a.wt_phase = pk + st.w_off + upconv_phase_offset_bytes(st.cout, st.cin, c.act_dtype);
        a.res = buf(st.res);
        if (st.sc_src != BUF_NONE) { a.x2 = buf(st.sc_src); a.cin2 = st.sc_cin; a.w2 = pk + st.sc_w_off; a.bias2 = (const float*)(pk + st.sc_b_off); }
        if (st.dst == BUF_OUT) { a.y = out; a.y_dtype = WMDEC_F32; a.y_nchw = 1; }
        else if (st.to_attn == 1) { a.y = ws + L.qkv; a.y_dtype = c.act_dtype; }
        else { a.y = buf(st.dst); a.y_dtype = c.act_dtype; }
        a.n = batch; a.h = st.h; a.w = st.w; a.cin = st.cin; a.cout = st.cout; a.ksize = st.ksize; a.upsample = st.upsample;
        if (st.emit_stats) {
          a.stats_groups = c.groups;
          (*emitted_slots) = conv_stats_slots(a);
          if ((*emitted_slots) > 0) a.stats_ws = st.emit_direct ? ws + L.rows[st.emit_rows] : ws + L.stats_ws;
          if (st.emit_rows >= 0 && !st.emit_direct) { a.rows_out = ws + L.rows[st.emit_rows]; a.tickets = ws + L.conv_tickets; }
        }
        rc = launch_conv(a, s);
        break;
      }
      case Step::QKV_TRANSPOSE_V: {
        const size_t es = dtype_size(c.act_dtype);
        const int t = st.h * st.w;
        rc = launch_transpose(ws + L.qkv + (size_t)2 * st.cin * es, c.act_dtype, ws + L.vt, c.act_dtype, batch, t, st.cin,
                              (size_t)3 * st.cin, (size_t)t * 3 * st.cin, 0 /* blocks of 32 keys */, flash_attention_vt_elems(t, st.cin), s);
        break;
      }
      case Step::NONE: break;
      case Step::FLASH: {
        const size_t es = dtype_size(c.act_dtype);
        const int t = st.h * st.w;
        rc = launch_flash_attention(ws + L.qkv, ws + L.qkv + (size_t)st.cin * es, (size_t)3 * st.cin, (size_t)t * 3 * st.cin,
                                    ws + L.vt, dec->attn_tpad, ws + L.attn_o, ws + L.attn_scratch, c.act_dtype, batch, t, st.cin,
                                    1.0f / sqrtf((float)st.cin), s);
        break;
      }
    }
    return rc;
  }
}

static int run_graph(const char* who, wmdec_decoder* dec, const LatentSource& latent, const void* packed, void* out, int batch,
                     void* stream) {
  WMDEC_REQUIRE(dec && latent.z && packed && out, WMDEC_ERR_INVALID_ARG, "%s: null pointer", who);
  WMDEC_REQUIRE(batch >= 1 && batch <= dec->cfg.max_batch, WMDEC_ERR_INVALID_ARG, "%s: batch %d outside 1..%d", who, batch, dec->cfg.max_batch);
  WMDEC_REQUIRE(aligned16(latent.z) && aligned16(latent.step) && aligned16(packed) && aligned16(out), WMDEC_ERR_INVALID_ARG,
                "%s: pointers must be 16-byte aligned", who);
  const WsLayout L = ws_layout(dec, batch);
  WMDEC_REQUIRE(dec->ws && dec->ws_bytes >= L.total, WMDEC_ERR_WORKSPACE, "%s: workspace needs %zu bytes, has %zu", who, L.total, dec->ws_bytes);
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)dec->ws;
  if (dec->ws_fresh) {   // once per workspace: the ticket counter of the statistics kernel starts at zero
    const int rc0 = launch_zero_u32(ws + L.tickets, (int)((gn_stats_ticket_bytes(dec->cfg.max_batch) + L.conv_ticket_bytes) / 4), s);
    if (rc0 != WMDEC_OK) return rc0;
    dec->ws_fresh = false;
  }
  const bool prof = dec->profiling;
  if (prof) { dec->profiled_batch = batch; WMDEC_HIP(hipEventRecord(dec->events[0], s)); }
  size_t step_index = 0;
  int emitted_slots = 0;   // moment slots per (sample, group) left by the last emitting convolution
  for (const Step& st : dec->steps) {
    const int rc = launch_step(dec, L, st, latent, packed, out, batch, &emitted_slots, s);
    if (rc != WMDEC_OK) return rc;
    ++step_index;
    if (prof) WMDEC_HIP(hipEventRecord(dec->events[step_index], s));
  }
  return WMDEC_OK;
}

int decoder_run(wmdec_decoder* dec, const void* latent, const void* packed, void* out, int batch, void* stream) {
  return run_graph("decoder_run", dec, LatentSource{latent, nullptr, 0.f}, packed, out, batch, stream);
}

int decoder_run_extrapolated(wmdec_decoder* dec, const void* z_prev, const void* v_prev, float lambda, const void* packed,
                             void* out, int batch, void* stream) {
  WMDEC_REQUIRE(v_prev, WMDEC_ERR_INVALID_ARG, "decoder_run_extrapolated: null motion vector");
  WMDEC_REQUIRE(isfinite(lambda), WMDEC_ERR_INVALID_ARG, "decoder_run_extrapolated: lambda is not finite");
  return run_graph("decoder_run_extrapolated", dec, LatentSource{z_prev, v_prev, lambda}, packed, out, batch, stream);
}

int wmdec_latent_extrapolate(const void* z_prev, const void* v_prev, int dtype, float lambda, int steps, void* z_out,
                             int out_dtype, size_t count, void* stream) {
  WMDEC_REQUIRE(z_prev && v_prev && z_out, WMDEC_ERR_INVALID_ARG, "latent_extrapolate: null pointer");
  WMDEC_REQUIRE(valid_dtype(dtype) && valid_dtype(out_dtype), WMDEC_ERR_INVALID_ARG, "latent_extrapolate: bad dtype");
  WMDEC_REQUIRE(steps >= 0 && isfinite(lambda), WMDEC_ERR_INVALID_ARG, "latent_extrapolate: bad steps or lambda");
  if (count == 0) return WMDEC_OK;
  return launch_axpy(z_prev, v_prev, dtype, (float)steps * lambda, z_out, out_dtype, count, (hipStream_t)stream);
}

int decoder_time_step(wmdec_decoder* dec, const void* latent, const void* packed, void* out, int batch, int step,
                      int reps, float* ms_per_launch, void* stream) {
  WMDEC_REQUIRE(dec && latent && packed && out && ms_per_launch, WMDEC_ERR_INVALID_ARG, "decoder_time_step: null pointer");
  WMDEC_REQUIRE(batch >= 1 && batch <= dec->cfg.max_batch, WMDEC_ERR_INVALID_ARG, "decoder_time_step: batch %d outside 1..%d", batch, dec->cfg.max_batch);
  WMDEC_REQUIRE(step >= 0 && step < (int)dec->steps.size() && reps >= 1, WMDEC_ERR_INVALID_ARG, "decoder_time_step: bad step or reps");
  WMDEC_REQUIRE(!dec->ws_fresh, WMDEC_ERR_INVALID_ARG, "decoder_time_step: run decoder_run on this workspace first");
  const WsLayout L = ws_layout(dec, batch);
  WMDEC_REQUIRE(dec->ws && dec->ws_bytes >= L.total, WMDEC_ERR_WORKSPACE, "decoder_time_step: workspace needs %zu bytes, has %zu", L.total, dec->ws_bytes);
  hipStream_t s = (hipStream_t)stream;
  int emitted_slots = 0;   // what the emitting convolutions before this step left behind
  for (int i = 0; i < step; ++i) {
    const Step& st = dec->steps[i];
    if (st.kind == Step::CONV && st.emit_stats) emitted_slots = conv_stats_slots(step_shape_args(*dec, st, batch));
  }
  hipEvent_t e0, e1;
  WMDEC_HIP(hipEventCreate(&e0));
  WMDEC_HIP(hipEventCreate(&e1));
  int rc = WMDEC_OK;
  hipError_t he = hipEventRecord(e0, s);
  for (int r = 0; r < reps && rc == WMDEC_OK && he == hipSuccess; ++r) {
    int slots = emitted_slots;
    rc = launch_step(dec, L, dec->steps[step], LatentSource{latent, nullptr, 0.f}, packed, out, batch, &slots, s);
  }
  if (he == hipSuccess) he = hipEventRecord(e1, s);
  if (he == hipSuccess) he = hipEventSynchronize(e1);
  float ms = 0.f;
  if (he == hipSuccess) he = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != WMDEC_OK) return rc;
  if (he != hipSuccess) return hip_fail(he, "decoder_time_step events");
  *ms_per_launch = ms / (float)reps;
  return WMDEC_OK;
}

int decoder_set_profiling(wmdec_decoder* dec, int enable) {
  WMDEC_REQUIRE(dec, WMDEC_ERR_INVALID_ARG, "decoder_set_profiling: null decoder");
  if (enable && dec->events.empty()) {
    for (size_t i = 0; i <= dec->steps.size(); ++i) {
      hipEvent_t e;
      WMDEC_HIP(hipEventCreate(&e));
      dec->events.push_back(e);
    }
  }
  dec->profiling = enable != 0;
  return WMDEC_OK;
}

int decoder_num_steps(const wmdec_decoder* dec) { return dec ? (int)dec->steps.size() : 0; }

int decoder_step_info(const wmdec_decoder* dec, int index, const char** kernel, double* flops, double* bytes) {
  WMDEC_REQUIRE(dec, WMDEC_ERR_INVALID_ARG, "decoder_step_info: null decoder");
  WMDEC_REQUIRE(index >= 0 && index < (int)dec->steps.size(), WMDEC_ERR_INVALID_ARG, "decoder_step_info: index %d out of range", index);
  const Step& st = dec->steps[index];
  if (flops) *flops = st.flops;
  if (bytes) *bytes = st.bytes;
  if (kernel) {
    switch (st.kind) {
      case Step::STATS: *kernel = st.from_producer ? "gn_finalize" : "gn_stats_vec"; break;
      case Step::QKV_TRANSPOSE_V: *kernel = "transpose_kernel"; break;
      case Step::FLASH: *kernel = "flash_attn_kernel"; break;
      case Step::NONE: *kernel = ""; break;
      case Step::CONV: {
        ConvArgs a = step_shape_args(*dec, st, 1);   // only the fields the kernel choice looks at
        a.groups_norm = st.norm; a.silu = st.silu;
        *kernel = conv_kernel_label(a);
        break;
      }
    }
  }
  return WMDEC_OK;
}

int decoder_step_times(const wmdec_decoder* dec, float* ms, int count) {
  WMDEC_REQUIRE(dec && ms, WMDEC_ERR_INVALID_ARG, "decoder_step_times: null pointer");
  WMDEC_REQUIRE(dec->profiling && dec->profiled_batch > 0, WMDEC_ERR_INVALID_ARG,
                "decoder_step_times: no profiled decoder_run has been enqueued");
  WMDEC_REQUIRE(count == (int)dec->steps.size(), WMDEC_ERR_INVALID_ARG, "decoder_step_times: count must be %zu", dec->steps.size());
  WMDEC_HIP(hipEventSynchronize(dec->events.back()));
  for (int i = 0; i < count; ++i) WMDEC_HIP(hipEventElapsedTime(&ms[i], dec->events[i], dec->events[i + 1]));
  return WMDEC_OK;
}

}  // extern "C"
