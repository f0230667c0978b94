"""Python face of the fp64 oracle -- TEST INFRASTRUCTURE ONLY (see wmdec_oracle.c).

Every function takes and returns float64 numpy arrays in logical NCHW order.
The per-operator arithmetic lives in wmdec_oracle.c (direct loops); this file
only composes operators into the blocks and the decoder graph.  The operator
list is the one the paper's vertical fusion names (Sec. IV-B-1: Upsample,
Conv2d, GroupNorm, SiLU); by the paper's cost model (Eq. 8 against Eq. 9) the
fused path must produce the values of the unfused graph, which is what is
written here.  The decoder topology is not given by the paper; the reading used
is documented at `decoder`.
"""
import ctypes
import math
import os

import numpy as np

from . import build as _build

_lib = None
_D = ctypes.POINTER(ctypes.c_double)


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
        for name in ("orc_gn_stats", "orc_silu", "orc_gn_apply", "orc_conv2d",
                     "orc_upsample2x", "orc_attention_core"):
            getattr(_lib, name).restype = None
    return _lib


def _p(a):
    return a.ctypes.data_as(_D)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def gn_stats(x, groups, eps):
    """Per (sample, group) mean and 1/sqrt(biased var + eps): two passes."""
    x = _f64(x)
    n, c, h, w = x.shape
    assert c % groups == 0
    mean = np.empty((n, groups))
    rstd = np.empty((n, groups))
    _load().orc_gn_stats(_p(x), n, c, h, w, groups, ctypes.c_double(eps), _p(mean), _p(rstd))
    return mean, rstd


def silu(x):
    x = _f64(x)
    y = np.empty_like(x)
    _load().orc_silu(_p(x), ctypes.c_size_t(x.size), _p(y))
    return y


def group_norm(x, groups, eps, gamma, beta, apply_silu=False):
    """gamma*(x-mean)*rstd+beta per channel, optionally followed by SiLU."""
    x = _f64(x)
    n, c, h, w = x.shape
    mean, rstd = gn_stats(x, groups, eps)
    gamma = _f64(gamma)
    beta = _f64(beta)
    assert gamma.shape == (c,) and beta.shape == (c,)
    y = np.empty_like(x)
    _load().orc_gn_apply(_p(x), n, c, h, w, groups, _p(mean), _p(rstd), _p(gamma), _p(beta),
                         1 if apply_silu else 0, _p(y))
    return y


def conv2d(x, w, b=None):
    """k x k cross-correlation, stride 1, zero padding k//2 (k in {1,3})."""
    x = _f64(x)
    w = _f64(w)
    n, cin, h, wd = x.shape
    cout, cin2, k, k2 = w.shape
    assert cin == cin2 and k == k2 and k in (1, 3)
    bp = None
    if b is not None:
        b = _f64(b)
        assert b.shape == (cout,)
        bp = _p(b)
    y = np.empty((n, cout, h, wd))
    _load().orc_conv2d(_p(x), _p(w), bp, n, cin, cout, h, wd, k, _p(y))
    return y


def upsample2x(x):
    """Nearest 2x: out[.., y, x] = in[.., y//2, x//2]."""
    x = _f64(x)
    n, c, h, w = x.shape
    y = np.empty((n, c, 2 * h, 2 * w))
    _load().orc_upsample2x(_p(x), n, c, h, w, _p(y))
    return y


def upconv(x, w, b=None):
    """3x3 conv of the materialised 2x-upsampled tensor (padding on the upsampled grid)."""
    return conv2d(upsample2x(x), w, b)


def resblock(x, p, groups=32, eps=1e-6):
    """x -> S(x) + conv2(SiLU(GN2(conv1(SiLU(GN1(x)))))); S = 1x1 conv iff 'shortcut.w' present.

    p maps 'norm1.gamma', 'norm1.beta', 'conv1.w', 'conv1.b', 'norm2.*', 'conv2.*'
    (and optionally 'shortcut.w', 'shortcut.b') to arrays.
    """
    h = group_norm(x, groups, eps, p["norm1.gamma"], p["norm1.beta"], apply_silu=True)
    h = conv2d(h, p["conv1.w"], p["conv1.b"])
    h = group_norm(h, groups, eps, p["norm2.gamma"], p["norm2.beta"], apply_silu=True)
    h = conv2d(h, p["conv2.w"], p["conv2.b"])
    s = conv2d(x, p["shortcut.w"], p["shortcut.b"]) if "shortcut.w" in p else _f64(x)
    return s + h


def attention_core(q, k, v, scale):
    """softmax_rows(q k^T * scale) v for token-major [T, d] matrices."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    t, d = q.shape
    assert k.shape == (t, d) and v.shape == (t, d)
    o = np.empty((t, d))
    _load().orc_attention_core(_p(q), _p(k), _p(v), t, d, ctypes.c_double(scale), _p(o))
    return o


def attention_block(x, p, groups=32, eps=1e-6):
    """Single-head spatial self-attention with residual.

    h = GN(x) (no SiLU); q,k,v = 1x1 convs of h with bias; tokens are the pixels
    in row-major (y*W + x) order; scores scaled by 1/sqrt(C); out = x + proj(o).
    p maps 'norm.gamma', 'norm.beta', 'q.w','q.b','k.w','k.b','v.w','v.b','proj.w','proj.b'.
    """
    x = _f64(x)
    n, c, hh, ww = x.shape
    h = group_norm(x, groups, eps, p["norm.gamma"], p["norm.beta"], apply_silu=False)
    q = conv2d(h, p["q.w"], p["q.b"])
    k = conv2d(h, p["k.w"], p["k.b"])
    v = conv2d(h, p["v.w"], p["v.b"])
    o = np.empty_like(x)
    for i in range(n):
        tok = lambda a: np.ascontiguousarray(a[i].reshape(c, hh * ww).T)  # [T, C]
        oi = attention_core(tok(q), tok(k), tok(v), 1.0 / math.sqrt(c))
        o[i] = oi.T.reshape(c, hh, ww)
    return x + conv2d(o, p["proj.w"], p["proj.b"])


def _sub(weights, prefix):
    pl = len(prefix) + 1
    return {k[pl:]: v for k, v in weights.items() if k.startswith(prefix + ".")}


def decoder(z, weights, level_channels=(512, 512, 256, 128), resblocks_per_level=3,
            groups=32, eps=1e-6):
    """Latent z[N,Cz,h,w] -> frame [N,Cout,8h,8w].

    Topology (the paper gives none; this is the reading of the workload
    description): conv_in 3x3 Cz->C0; mid = ResBlock(C0), attention, ResBlock(C0);
    for each level l: `resblocks_per_level` ResBlocks, the first one mapping the
    previous level's channels to this level's (1x1 conv shortcut when they
    differ), then -- except after the last level -- nearest-2x upsample followed
    by a 3x3 conv that keeps the channel count; finally GN -> SiLU -> conv_out.
    """
    x = conv2d(z, weights["conv_in.w"], weights["conv_in.b"])
    x = resblock(x, _sub(weights, "mid.res1"), groups, eps)
    x = attention_block(x, _sub(weights, "mid.attn"), groups, eps)
    x = resblock(x, _sub(weights, "mid.res2"), groups, eps)
    nlev = len(level_channels)
    for l in range(nlev):
        for i in range(resblocks_per_level):
            x = resblock(x, _sub(weights, f"up.{l}.res{i}"), groups, eps)
        if l + 1 < nlev:
            x = upconv(x, weights[f"up.{l}.upsample.w"], weights[f"up.{l}.upsample.b"])
    x = group_norm(x, groups, eps, weights["norm_out.gamma"], weights["norm_out.beta"], apply_silu=True)
    return conv2d(x, weights["conv_out.w"], weights["conv_out.b"])


def latent_extrapolate(z_prev, v_prev, lam):
    """Hit branch of the latent-extrapolation algorithm (Sec. IV-C, Alg. 2): the world model is skipped and the
    next latent is the first-order Taylor step of that section, z_t = z_{t-1} + lambda * v_{t-1}, with the motion
    vector v_{t-1} = z_{t-1} - z_{t-2} standing in for dz/dt."""
    return _f64(z_prev) + float(lam) * _f64(v_prev)


def extrapolated_latents(z_prev, v_prev, lam, hits):
    """`hits` consecutive hit steps of Alg. 2.  The motion vector is only updated on a miss, so every step adds the
    same lambda * v to the latent the previous step produced.  Returns [hits, ...]: the latent of every step."""
    z = _f64(z_prev)
    out = []
    for _ in range(int(hits)):
        z = latent_extrapolate(z, v_prev, lam)
        out.append(z)
    return np.stack(out) if out else np.empty((0,) + z.shape)


def adaln_modulation(c, p, apply_silu=True):
    """The AdaLN block's three small projections of the conditioning vector as the unfused graph runs them
    (Sec. IV-B-2: one small product per parameter): with a = SiLU(c) (the usual activation in front of the
    modulation; a = c if apply_silu is false),
        shift = W_shift a + b_shift,   scale = W_scale a + b_scale,   gate = W_gate a + b_gate.
    c: [batch, d_cond]; p maps 'shift.w', 'scale.w', 'gate.w' ([d_model, d_cond]) and '.b' ([d_model]).
    Returns (shift, scale, gate), each [batch, d_model].  Horizontal fusion stores the three matrices as one block
    and runs one product; it must return exactly these values, concatenated."""
    a = silu(c) if apply_silu else _f64(c)
    out = []
    for name in ("shift", "scale", "gate"):
        w, b = _f64(p[name + ".w"]), _f64(p[name + ".b"])
        y = np.empty((a.shape[0], w.shape[0]))
        for i in range(a.shape[0]):          # one matrix-vector product per conditioning vector and parameter
            y[i] = w @ a[i] + b
        out.append(y)
    return tuple(out)


def rel_err(got, want):
    """max|got-want| / rms(want): the comparison metric of every parity test."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    rms = math.sqrt(float(np.mean(want * want)))
    return float(np.max(np.abs(got - want))) / (rms if rms > 0 else 1.0)
