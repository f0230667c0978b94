/*
 * wmdec -- fused latent -> frame convolutional decoder for AMD MI355X (gfx950).
 *
 * C ABI of libwmdec.so.  The library implements the memory-bound decoder stage
 * that the paper's vertical operator fusion targets (Sec. IV-A, Eq. 8: the
 * unfused graph materialises every Conv2d / GroupNorm / SiLU result in HBM;
 * Sec. IV-B-1, Eq. 9: the fused graph reads its input once and writes its
 * output once).  On gfx950 the fusion is: one GroupNorm statistics pass, then
 * normalise + SiLU applied while an input tile is staged into LDS for an
 * implicit-GEMM convolution on the matrix cores, nearest-2x upsampling folded
 * into that gather, bias and residual added in the epilogue.
 *
 * Conventions (all entry points)
 *  - Every tensor pointer is a DEVICE pointer owned by the caller; the library
 *    never allocates, frees or copies device memory and never synchronises.
 *    All work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *    the default stream).  Host-side handles (wmdec_decoder) are library-owned.
 *  - Activations are dense NHWC ("channels last"): element (n, y, x, c) of a
 *    logical [N,C,H,W] tensor lives at ((n*H + y)*W + x)*C + c.  Only
 *    decoder_run's latent input and frame output are NCHW.
 *  - Tensor pointers must be 16-byte aligned.
 *  - Return value: 0 (WMDEC_OK) or a negative wmdec_status.  Argument errors
 *    are detected before anything is launched; wmdec_last_error() returns a
 *    thread-local description of the last failure.  No exception crosses the ABI.
 *  - Same inputs give bitwise identical outputs (no order-dependent atomics).
 */
#ifndef WMDEC_H
#define WMDEC_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  WMDEC_OK = 0,
  WMDEC_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, bad enum */
  WMDEC_ERR_UNSUPPORTED = -2, /* valid in principle, not implemented for this dtype / shape */
  WMDEC_ERR_SHAPE = -3,       /* sizes inconsistent (c % groups != 0, ...) */
  WMDEC_ERR_WORKSPACE = -4,   /* workspace missing or too small */
  WMDEC_ERR_HIP = -5          /* a HIP call or kernel launch failed */
} wmdec_status;

/* Storage / arithmetic types.  F32: fp32 storage, fp32 FMA arithmetic.
 * BF16 / F16: 16-bit storage, matrix-core (MFMA) products of that type with
 * fp32 accumulation; statistics, normalisation, SiLU, softmax, bias and
 * residual adds are always fp32. */
typedef enum { WMDEC_F32 = 0, WMDEC_BF16 = 1, WMDEC_F16 = 2 } wmdec_dtype;

const char* wmdec_last_error(void);
const char* wmdec_status_string(int status);

/* ------------------------------------------------------------------------
 * GroupNorm statistics pass (operator list of Sec. IV-B-1; the paper does not
 * say how per-group statistics survive spatial tiling -- here they are a
 * separate streaming pass).
 *   group g of sample n = channels [g*c/groups, (g+1)*c/groups) over all h*w
 *   pixels;  mean[n*groups+g] = average,  rstd[...] = 1/sqrt(biased variance + eps).
 * x: [n,h,w,c] NHWC of x_dtype.  mean, rstd: fp32 [n*groups] outputs.
 * workspace: at least wmdec_gn_stats_workspace_bytes(...) bytes of device
 * memory, ZERO-FILLED once before the first call that uses it: its head holds
 * one ticket counter per sample, which every call leaves at zero again, so
 * the buffer can be reused (also with other shapes of the same n) without
 * clearing.  The rest is scratch (contents undefined afterwards).
 * Calls sharing a workspace must be ordered on one stream.
 * Errors: c % groups != 0 -> WMDEC_ERR_SHAPE. */
size_t wmdec_gn_stats_workspace_bytes(int n, int h, int w, int c, int groups);
int wmdec_gn_stats(const void* x, int x_dtype, int n, int h, int w, int c, int groups, float eps,
                   float* mean, float* rstd, void* workspace, size_t workspace_bytes, void* stream);

/* The same statistics for callers that cannot allocate device memory or hand
 * over a workspace (code under HIP-graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the partial moments and the ticket
 * counters live in a file-scope device array of the library, 1 MiB + 256
 * bytes per GPU, held until the process ends.  The call allocates nothing and
 * enqueues kernels only (a small fill kernel puts the counters back to zero,
 * then the statistics kernels of wmdec_gn_stats run on that array), so mean
 * and rstd equal wmdec_gn_stats's bit for bit.
 * Limits: n <= 64 and n * groups * slabs * 12 bytes <= 1 MiB, where slabs <=
 * 256 for shapes of the single-launch layout (16-bit: c % 8 == 0, c/8 divides
 * 1024, channels per group a power of two <= 64) and <= 2048 otherwise; e.g.
 * every activation of the 720x480 decoder up to batch 10.  Beyond the limit:
 * WMDEC_ERR_WORKSPACE and nothing is launched.
 * All calls on one GPU share the array: calls that overlap in time on one GPU
 * (different streams or threads) race; order them on one stream. */
int wmdec_gn_stats_noalloc(const void* x, int x_dtype, int n, int h, int w, int c, int groups, float eps,
                           float* mean, float* rstd, void* stream);

/* ------------------------------------------------------------------------
 * Weight packing.  Convolution kernels read weights in a packed order: per
 * tap, fragments of 32 output x 16 input channels, each stored as 1 KiB (for
 * 16-bit types) in the lane order of the matrix-core B operand, C_in padded to
 * a multiple of 16 and C_out to a multiple of 32 with zeros, in the operand
 * type `op_dtype` (F32 for the fp32 path, else BF16 or F16).  The layout is
 * private to the library: always produce it with this call.  src is the
 * logical [cout][cin][k][k] tensor (k = 1 or 3) of src_dtype (F32 or BF16).
 * BF16 -> F16 conversion is exact for normal-range values.  `packed` must hold
 * wmdec_conv_packed_bytes(...) bytes. */
size_t wmdec_conv_packed_bytes(int cout, int cin, int k, int op_dtype);
int wmdec_pack_conv_weights(const void* src, int src_dtype, int cout, int cin, int k,
                            void* packed, int op_dtype, void* stream);

/* ------------------------------------------------------------------------
 * Fused GroupNorm-apply -> SiLU -> 3x3 convolution (+bias, +residual):
 * Conv2d, GroupNorm, SiLU of Sec. IV-B-1 in one kernel (Eq. 9).
 *   u[n,y,x,ci] = act(gamma[ci]*(x - mean[n,g])*rstd[n,g] + beta[ci]),  act = SiLU if apply_silu
 *   y[n,oy,ox,co] = bias[co] + sum_{ky,kx,ci} W[co,ci,ky,kx] * u[n,oy+ky-1,ox+kx-1,ci] (+ residual)
 * with u = 0 outside the image (padding acts on the activated tensor).
 * mean == NULL (then rstd, gamma, beta are ignored) skips normalisation and
 * activation: a plain convolution.  act_dtype: type of x, residual and of the
 * MFMA operands (w_packed must be packed for it).  y_dtype: act_dtype or F32.
 * bias (fp32 [cout]) and residual ([n,h,w,cout], act_dtype) may be NULL.
 * x and y must not overlap.  gamma, beta: fp32 [cin]. */
int wmdec_gn_silu_conv3x3(const void* x, int act_dtype, const float* mean, const float* rstd,
                          const float* gamma, const float* beta, int groups, int apply_silu,
                          const void* w_packed, const float* bias, const void* residual,
                          void* y, int y_dtype, int n, int h, int w, int cin, int cout, void* stream);

/* The same convolution, which in addition returns the GroupNorm statistics of
 * its own output y, so that the next normalisation needs no statistics pass
 * and y is not read again (the "one read, one write" accounting of Eq. 9
 * applied to the Conv2d -> GroupNorm pair of Sec. IV-B-1):
 *   mean_out[n*out_groups+g], rstd_out[...] = mean and 1/sqrt(biased variance
 *   + out_eps) of y[n,:,:,g*cout/out_groups .. (g+1)*cout/out_groups), taken
 * over the values as stored in y (after the rounding to y_dtype), i.e. what
 * wmdec_gn_stats would return for y up to fp32 summation order.  Every
 * workgroup writes per-group partial moments of its tile to `workspace`
 * (wmdec_conv_stats_workspace_bytes(...) bytes, no initialisation needed); a
 * second small launch merges them in a fixed order.
 * Two kernels can emit moments, both for 16-bit act_dtype: the matrix-core
 * kernel (cin % 32 == 0, cout % 64 == 0, cout/out_groups a power of two <= 32)
 * and the kernel for cin <= 8 (the decoder's conv_in: no normalisation of x,
 * no residual, cout/out_groups a power of two <= 64); any other shape gives
 * WMDEC_ERR_UNSUPPORTED (the workspace query then returns 0). */
size_t wmdec_conv_stats_workspace_bytes(int act_dtype, int y_dtype, int n, int h, int w, int cin,
                                        int cout, int out_groups);
int wmdec_gn_silu_conv3x3_stats(const void* x, int act_dtype, const float* mean, const float* rstd,
                                const float* gamma, const float* beta, int groups, int apply_silu,
                                const void* w_packed, const float* bias, const void* residual,
                                void* y, int y_dtype, int n, int h, int w, int cin, int cout,
                                int out_groups, float out_eps, float* mean_out, float* rstd_out,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Second convolution of a channel-changing ResBlock with the block's 1x1
 * shortcut folded into its contraction (the Eq. 9 accounting applied to
 * S(x) + conv3x3(...): the shortcut tensor is neither written nor read back):
 *   y = bias + conv3x3(u) + bias2 + W2 * x2,   u as above,
 * i.e. a contraction over K = 9*cin + cin2.  x2: [n,h,w,cin2] of act_dtype, taken
 * as stored (no normalisation); w2_packed: [cout][cin2] packed with k = 1; bias2
 * fp32 [cout] or NULL.  x2 and y must not overlap.  Shapes the matrix-core
 * kernel takes (16-bit types, cin % 32 == 0, cin2 % 32 == 0, cout % 64 == 0) run
 * as one launch; anything else (and F32) as two launches of the general kernel,
 * the second adding the shortcut it finds in y. */
int wmdec_gn_silu_conv3x3_shortcut(const void* x, int act_dtype, const float* mean, const float* rstd,
                                   const float* gamma, const float* beta, int groups, int apply_silu,
                                   const void* w_packed, const float* bias,
                                   const void* x2, int cin2, const void* w2_packed, const float* bias2,
                                   void* y, int y_dtype, int n, int h, int w, int cin, int cout,
                                   void* stream);

/* 1x1 convolution (a GEMM over pixels; the workload's attention projections
 * q, k, v, proj and the 1x1 shortcut of a channel-changing ResBlock -- the
 * "plus a residual" of the ResBlock when C_in != C_out) with the same optional
 * normalise-on-load, bias and residual:
 *   y[n,p,co] = bias[co] + sum_ci W[co,ci] * u[n,p,ci] (+ residual),
 * u as for the 3x3 form.  A Conv2d of Sec. IV-B-1 with k = 1.
 * w_packed: packed with k = 1. */
int wmdec_gn_conv1x1(const void* x, int act_dtype, const float* mean, const float* rstd,
                     const float* gamma, const float* beta, int groups, int apply_silu,
                     const void* w_packed, const float* bias, const void* residual,
                     void* y, int y_dtype, int n, int h, int w, int cin, int cout, void* stream);

/* ------------------------------------------------------------------------
 * Upsample -> Conv2d fused (first two operators of the chain in Sec. IV-B-1):
 *   y[n,oy,ox,co] = bias[co] + sum W[co,ci,ky,kx] * x[n,(oy+ky-1)>>1,(ox+kx-1)>>1,ci]
 * for 0 <= oy+ky-1 < 2*h_in and 0 <= ox+kx-1 < 2*w_in, zero otherwise.
 * x: [n,h_in,w_in,cin]; y: [n,2*h_in,2*w_in,cout].  The upsampled tensor is
 * never materialised.  On the matrix-core path the sum is evaluated per output
 * phase (oy&1, ox&1): the 3x3 taps that read the same input pixel are added
 * once, when the weights are packed, so each output costs a 2x2 convolution
 * (4/9 of the multiplications; same sum, the pre-added weights are rounded to
 * the operand type once).
 * w_packed: from wmdec_pack_upconv_weights (NOT wmdec_pack_conv_weights): the
 * 9-tap pack followed by the 16-tap phase pack, wmdec_upconv_packed_bytes()
 * bytes in total, 16-byte aligned. */
size_t wmdec_upconv_packed_bytes(int cout, int cin, int op_dtype);
int wmdec_pack_upconv_weights(const void* src, int src_dtype, int cout, int cin, void* packed,
                              int op_dtype, void* stream);
int wmdec_upsample2x_conv3x3(const void* x, int act_dtype, const void* w_packed, const float* bias,
                             void* y, int y_dtype, int n, int h_in, int w_in, int cin, int cout,
                             void* stream);

/* Stand-alone nearest-neighbour 2x upsample (the Upsample operator of
 * Sec. IV-B-1 on its own, as the unfused graph of Eq. 8 would run it; the
 * workload's upsample stage, x[1,256,120,180] -> [1,256,240,360]):
 *   y[n,oy,ox,c] = x[n,oy>>1,ox>>1,c];  bit-exact copy of elements of `dtype`.
 * Reads x once, writes 4x its size; bounded by HBM bandwidth. */
int wmdec_upsample2x_nearest(const void* x, void* y, int dtype, int n, int h_in, int w_in, int c,
                             void* stream);

/* ------------------------------------------------------------------------
 * Layout / type conversion between the logical NCHW order (B x C x H x W, the
 * order Sec. IV-A writes feature maps in) and the library's NHWC order:
 * dst = convert(src) element by element (round to nearest even when
 * narrowing).  Not on the decoder path (decoder_run reads and writes NCHW at
 * its two ends itself); for callers of the per-operator entry points. */
int wmdec_nchw_to_nhwc(const void* src, int src_dtype, void* dst, int dst_dtype,
                       int n, int c, int h, int w, void* stream);
int wmdec_nhwc_to_nchw(const void* src, int src_dtype, void* dst, int dst_dtype,
                       int n, int c, int h, int w, void* stream);

/* ------------------------------------------------------------------------
 * Mid-block single-head self-attention with residual over the h*w tokens of
 * the 60x90 feature map (the workload's "single-head self-attention over 5400
 * tokens, d = 512, GroupNorm before QKV"; the paper names no attention in its
 * decoder and only cites flash-style kernels as prior art, Sec. II).  The
 * score matrix is never materialised, in the spirit of Eq. 9: q, k, v are
 * read once per key block, the output written once:
 *   hn = gamma*(x-mean)*rstd+beta (no SiLU);  [q|k|v] = Wqkv hn + bqkv;
 *   o = softmax_rows(q k^T / sqrt(c)) v;  y = x + Wo o + bo.
 * Tokens are the h*w pixels of one sample.  x, y: [n,h,w,c] of act_dtype
 * (BF16 or F16).  wqkv_packed: the [3c][c] matrix (rows q, then k, then v)
 * packed as a 1x1 convolution with cout = 3c; wo_packed: [c][c] likewise.
 * bqkv: fp32 [3c]; bo: fp32 [c].  c must be 512.  workspace: at least
 * wmdec_attention_workspace_bytes(n,h,w,c) bytes. */
size_t wmdec_attention_workspace_bytes(int n, int h, int w, int c);
int wmdec_attention(const void* x, int act_dtype, const float* mean, const float* rstd,
                    const float* gamma, const float* beta, int groups,
                    const void* wqkv_packed, const float* bqkv, const void* wo_packed, const float* bo,
                    void* y, int n, int h, int w, int c,
                    void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Horizontal fusion for the DiT's AdaLN block (Sec. IV-B-2).  A block's
 * modulation vectors are three small products of the same conditioning vector,
 *   shift = W_shift a + b_shift,  scale = W_scale a + b_scale,  gate = W_gate a + b_gate,
 * a = SiLU(c) if apply_silu else c.  With the matrices stored as one
 * row-concatenated block W_fused = [W_shift; W_scale; W_gate] (and likewise the
 * biases) they are one product and one launch:
 *   out[b, j] = bias[j] + sum_k W_fused[j, k] * a[b, k],   j < rows, k < d_cond,
 * so rows = 3 * d_model (any number of row blocks works: the call does not
 * care where one matrix ends).  c: [batch, d_cond] of c_dtype; w_fused:
 * row-major [rows, d_cond] of w_dtype (no packing); bias: fp32 [rows] or NULL;
 * out: fp32 [batch, rows], so shift, scale, gate of sample b are the three
 * thirds of row b.  Products and sums in fp32.
 * With a few conditioning vectors per call (one per frame) this is bound by
 * the one read of the weights from HBM, not by arithmetic; the conditioning
 * vectors are held in LDS, which limits a call to wmdec_adaln_max_batch(d_cond)
 * of them (the largest power of two <= 16 with batch * d_cond <= 16384, e.g. 8
 * for d_cond = 1920); beyond: WMDEC_ERR_UNSUPPORTED.  d_cond must be a multiple
 * of 8 and at most 4096 (16-bit weights), or a multiple of 4 and at most 2048
 * (F32). */
int wmdec_adaln_max_batch(int d_cond);
int wmdec_adaln_fused_projection(const void* c, int c_dtype, const void* w_fused, int w_dtype,
                                 const float* bias, float* out, int batch, int d_cond, int rows,
                                 int apply_silu, void* stream);

/* ------------------------------------------------------------------------
 * Whole decoder:  latent z[N,latent_c,h,w] -> frame [N,out_c,8h,8w]
 * (the I_t <- VAE_Decode(z_t) step of Alg. 1 / Alg. 2).
 * Graph: conv_in 3x3; mid = ResBlock, attention, ResBlock; per level
 * `resblocks_per_level` ResBlocks (the first maps the previous level's channel
 * count, with a 1x1-conv shortcut when it changes) followed -- except after the
 * last level -- by upsample-conv; then GroupNorm -> SiLU -> conv_out.
 * ResBlock(x) = S(x) + conv3x3(SiLU(GN(conv3x3(SiLU(GN(x)))))). */
typedef struct wmdec_decoder wmdec_decoder; /* opaque, host memory, library-owned */

typedef struct {
  int latent_c, latent_h, latent_w; /* 4, 60, 90 */
  int num_levels;                   /* 1..4 */
  int level_channels[4];            /* 512, 512, 256, 128 */
  int resblocks_per_level;          /* 3 */
  int groups;                       /* 32 */
  float eps;                        /* 1e-6 */
  int out_c;                        /* 3 */
  int act_dtype;                    /* WMDEC_BF16 or WMDEC_F16: storage of activations and MFMA operand type */
  int max_batch;                    /* largest batch decoder_run will be given */
  int latent_dtype;                 /* storage type of the latent handed to decoder_run: WMDEC_BF16 (the workloads),
                                       WMDEC_F16 or WMDEC_F32 */
  int separate_stats_pass;          /* 0: a GroupNorm takes its statistics from the epilogue of the convolution that
                                       produced its input (no extra read of the tensor); 1: every GroupNorm runs the
                                       streaming statistics pass (wmdec_gn_stats) -- the graph before that fusion */
  int separate_merge_launch;        /* 0: where producer and consumer of a GroupNorm's statistics are both matrix-core
                                       convolutions, the producer's last workgroup per tile row merges that row's partial
                                       moments and the consumer merges the rows in its prologue: no launch in between;
                                       1: a small merge launch (the graph before that fusion) */
  int separate_shortcut;            /* 0: the 1x1 shortcut of a channel-changing ResBlock is folded into the contraction
                                       of the block's second convolution; 1: it is a launch of its own whose output the
                                       second convolution adds -- the graph before that fusion */
} wmdec_decoder_config;

/* Fills *cfg with the 720x480 decoder above (act_dtype = WMDEC_F16, max_batch = 4,
 * latent_dtype = WMDEC_BF16, separate_stats_pass = 0, separate_merge_launch = 0,
 * separate_shortcut = 0). */
void decoder_default_config(wmdec_decoder_config* cfg);

/* Validates cfg and builds the host-side plan.  Allocates no device memory. */
int decoder_create(const wmdec_decoder_config* cfg, wmdec_decoder** out);
int decoder_destroy(wmdec_decoder* dec);

/* Canonical weight blob (what the caller provides to decoder_pack_weights):
 * parameters in execution order, each at a 256-byte aligned offset; conv /
 * linear weights are BF16 [cout][cin][k][k], biases, gamma, beta are F32.
 * decoder_num_weights / decoder_weight_info enumerate them; names are
 * "conv_in.w", "mid.res1.norm1.gamma", "mid.attn.q.w", "up.2.res0.shortcut.w",
 * "up.0.upsample.b", "norm_out.beta", "conv_out.w", ...  */
size_t decoder_weights_bytes(const wmdec_decoder* dec);
int decoder_num_weights(const wmdec_decoder* dec);
int decoder_weight_info(const wmdec_decoder* dec, int index, const char** name, size_t* offset,
                        size_t* bytes, int* dtype, int shape[4]);
int decoder_weight_offset(const wmdec_decoder* dec, const char* name, size_t* offset, size_t* bytes);

/* Packed blob (what decoder_run reads): conv weights re-ordered / converted for
 * the kernels, q/k/v fused into one matrix, small parameters copied.  `packed`
 * must hold decoder_packed_bytes(dec) bytes.  Done once per set of weights. */
size_t decoder_packed_bytes(const wmdec_decoder* dec);
int decoder_pack_weights(const wmdec_decoder* dec, const void* weights, void* packed, void* stream);

/* Scratch for activations and statistics of one decoder_run of `batch` frames. */
size_t decoder_workspace_bytes(const wmdec_decoder* dec, int batch);
int decoder_set_workspace(wmdec_decoder* dec, void* workspace, size_t bytes);

/* latent: [batch,latent_c,h,w] NCHW of cfg.latent_dtype.  packed: from decoder_pack_weights.
 * out: [batch,out_c,8h,8w] NCHW, F32.  1 <= batch <= max_batch.  Enqueues the
 * whole graph on `stream`; no host synchronisation, no allocation, kernels
 * only (after the first call on a workspace, which also sets kernel attributes
 * and zeroes the statistics counters, the call may be captured in a HIP graph).
 * Calls that share one decoder (hence one workspace) must be ordered on the
 * same stream. */
int decoder_run(wmdec_decoder* dec, const void* latent, const void* packed, void* out, int batch,
                void* stream);

/* ------------------------------------------------------------------------
 * Latent extrapolation in front of the decoder (Sec. IV-C, Alg. 2, hit
 * branch: when the action is stable the world model is skipped and
 *   z_t = z_{t-1} + lambda * v_{t-1},   I_t = VAE_Decode(z_t),
 * with v the motion vector z_{t-1} - z_{t-2}; on consecutive hits v is not
 * updated, so the j-th skipped frame decodes z_{t-1} + (j+1)*lambda*v).
 *
 * decoder_run_extrapolated decodes `batch` such frames in one graph: frame j
 * (j = 0..batch-1) is VAE_Decode(z_prev + (j+1)*lambda*v_prev).  The sum is
 * formed where conv_in stages its input (one fp32 fused multiply-add of the
 * stored values, one rounding to the operand type), so the extrapolated
 * latents never exist in memory.  z_prev, v_prev: ONE latent each,
 * [latent_c,h,w] NCHW of cfg.latent_dtype.  Everything else as decoder_run.
 *
 * wmdec_latent_extrapolate materialises one extrapolated latent (the state a
 * caller carries to the next step of Alg. 2):
 *   z_out[i] = fma((float)steps * lambda, v_prev[i], z_prev[i])  (fp32), rounded
 * once to out_dtype.  With out_dtype = WMDEC_F32 and a decoder whose
 * latent_dtype is WMDEC_F32, decoder_run(z_out) reproduces frame steps-1 of
 * decoder_run_extrapolated bit for bit.  z_prev, v_prev: `count` elements of
 * `dtype`; z_out: `count` elements of out_dtype; may alias z_prev if the
 * types have the same size. */
int decoder_run_extrapolated(wmdec_decoder* dec, const void* z_prev, const void* v_prev, float lambda,
                             const void* packed, void* out, int batch, void* stream);
int wmdec_latent_extrapolate(const void* z_prev, const void* v_prev, int dtype, float lambda, int steps,
                             void* z_out, int out_dtype, size_t count, void* stream);

/* Number of kernel launches one decoder_run enqueues, and the FLOP count of
 * one frame: 2*k*k*cin*cout per output pixel of every convolution plus
 * 4*T*T*c for the attention -- except that an upsampling convolution
 * evaluated per output phase (see wmdec_upsample2x_conv3x3) counts the 2x2
 * taps it executes, 4/9 of the nine-tap figure.  decoder_dense_flops_per_frame
 * is the nine-tap figure throughout: what the unfused graph would execute. */
int decoder_num_launches(const wmdec_decoder* dec);
double decoder_flops_per_frame(const wmdec_decoder* dec);
double decoder_dense_flops_per_frame(const wmdec_decoder* dec);

#ifdef __cplusplus
}
#endif
#endif /* WMDEC_H */
