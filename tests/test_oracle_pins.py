"""Pins for the fp64 oracle: every operator is checked against something that is
not the oracle itself -- brute force in pure Python, closed forms, invariants,
or an independent library routine (scipy / numpy)."""
import itertools
import os
import math

import numpy as np
import pytest
import scipy.signal
import scipy.special

from oracle import ref

RNG = np.random.default_rng(20260200608)


# ----------------------------------------------------------------- conv
def brute_conv(x, w, b):
    n, cin, h, wd = x.shape
    cout, _, k, _ = w.shape
    pad = k // 2
    y = np.zeros((n, cout, h, wd))
    for i, co, oy, ox in itertools.product(range(n), range(cout), range(h), range(wd)):
        acc = float(b[co]) if b is not None else 0.0
        for ci, ky, kx in itertools.product(range(cin), range(k), range(k)):
            iy, ix = oy + ky - pad, ox + kx - pad
            if 0 <= iy < h and 0 <= ix < wd:
                acc += float(w[co, ci, ky, kx]) * float(x[i, ci, iy, ix])
        y[i, co, oy, ox] = acc
    return y


@pytest.mark.parametrize("shape,cout,k", [((1, 3, 5, 4), 2, 3), ((2, 2, 1, 1), 3, 3),
                                          ((1, 1, 2, 7), 1, 3), ((2, 3, 4, 3), 4, 1)])
def test_conv_brute_force(shape, cout, k):
    x = RNG.standard_normal(shape)
    w = RNG.standard_normal((cout, shape[1], k, k))
    b = RNG.standard_normal(cout)
    np.testing.assert_allclose(ref.conv2d(x, w, b), brute_conv(x, w, b), rtol=0, atol=1e-13)
    np.testing.assert_allclose(ref.conv2d(x, w, None), brute_conv(x, w, None), rtol=0, atol=1e-13)


def test_conv_delta_kernel_is_identity_and_shift():
    x = RNG.standard_normal((2, 5, 7, 6))
    w = np.zeros((5, 5, 3, 3))
    for c in range(5):
        w[c, c, 1, 1] = 1.0
    assert np.array_equal(ref.conv2d(x, w, np.zeros(5)), x)
    # tap (ky,kx) = (0,2) reads x[y-1, x+1]: image moves down one row and left one column
    w = np.zeros((5, 5, 3, 3))
    for c in range(5):
        w[c, c, 0, 2] = 1.0
    want = np.zeros_like(x)
    want[:, :, 1:, :-1] = x[:, :, :-1, 1:]
    assert np.array_equal(ref.conv2d(x, w, None), want)
    # a delta that permutes channels: cross-correlation indexing w[co, ci]
    w = np.zeros((5, 5, 3, 3))
    for c in range(5):
        w[c, (c + 1) % 5, 1, 1] = 1.0
    assert np.array_equal(ref.conv2d(x, w, None), np.roll(x, -1, axis=1))


def test_conv_all_ones_counts_taps():
    y = ref.conv2d(np.ones((1, 1, 5, 6)), np.ones((1, 1, 3, 3)), None)[0, 0]
    assert y[2, 3] == 9 and y[0, 2] == 6 and y[3, 0] == 6 and y[0, 0] == 4 and y[4, 5] == 4
    assert y.sum() == 9 * 30 - 2 * 3 * (5 + 6) + 4  # 9 per pixel minus the taps that fall outside


def test_conv_no_kernel_flip_vs_scipy():
    x = RNG.standard_normal((1, 3, 9, 8))
    w = RNG.standard_normal((4, 3, 3, 3))
    b = RNG.standard_normal(4)
    want = np.zeros((1, 4, 9, 8))
    for co in range(4):
        for ci in range(3):
            want[0, co] += scipy.signal.correlate2d(x[0, ci], w[co, ci], mode="same", boundary="fill")
        want[0, co] += b[co]
    np.testing.assert_allclose(ref.conv2d(x, w, b), want, rtol=0, atol=1e-12)


def test_conv_as_nine_shifted_matmuls_and_linearity():
    x = RNG.standard_normal((2, 6, 10, 11))
    w = RNG.standard_normal((5, 6, 3, 3))
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
    want = np.zeros((2, 5, 10, 11))
    for ky in range(3):
        for kx in range(3):
            want += np.einsum("oc,nchw->nohw", w[:, :, ky, kx], xp[:, :, ky:ky + 10, kx:kx + 11])
    np.testing.assert_allclose(ref.conv2d(x, w, None), want, rtol=0, atol=1e-12)
    x2 = RNG.standard_normal(x.shape)
    w2 = RNG.standard_normal(w.shape)
    np.testing.assert_allclose(ref.conv2d(2 * x - 3 * x2, w, None),
                               2 * ref.conv2d(x, w, None) - 3 * ref.conv2d(x2, w, None), atol=1e-11)
    np.testing.assert_allclose(ref.conv2d(x, w + 0.5 * w2, None),
                               ref.conv2d(x, w, None) + 0.5 * ref.conv2d(x, w2, None), atol=1e-11)


def test_conv1x1_is_matmul():
    x = RNG.standard_normal((2, 7, 4, 5))
    w = RNG.standard_normal((3, 7, 1, 1))
    b = RNG.standard_normal(3)
    want = np.einsum("oc,nchw->nohw", w[:, :, 0, 0], x) + b[None, :, None, None]
    np.testing.assert_allclose(ref.conv2d(x, w, b), want, rtol=0, atol=1e-13)


# ----------------------------------------------------------------- GroupNorm / SiLU
def test_gn_stats_vs_numpy_and_brute():
    x = RNG.standard_normal((3, 12, 5, 7)) * 3.0 + 1.5
    eps = 1e-6
    mean, rstd = ref.gn_stats(x, 4, eps)
    xg = x.reshape(3, 4, -1)
    np.testing.assert_allclose(mean, xg.mean(axis=2), rtol=0, atol=1e-13)
    np.testing.assert_allclose(rstd, 1.0 / np.sqrt(xg.var(axis=2) + eps), rtol=1e-13)
    # brute force for one group: channels 3..5 of sample 1 form group 1 (contiguous channels)
    vals = [float(x[1, c, i, j]) for c in (3, 4, 5) for i in range(5) for j in range(7)]
    mu = sum(vals) / len(vals)
    var = sum((v - mu) ** 2 for v in vals) / len(vals)          # biased: divide by M
    assert abs(mean[1, 1] - mu) < 1e-13
    assert abs(rstd[1, 1] - 1.0 / math.sqrt(var + eps)) < 1e-12  # eps inside the root


def test_gn_zero_mean_unit_variance():
    x = RNG.standard_normal((2, 64, 9, 11)) * 2.5 - 4.0
    eps = 1e-6
    y = ref.group_norm(x, 32, eps, np.ones(64), np.zeros(64))
    yg = y.reshape(2, 32, -1)
    var_in = x.reshape(2, 32, -1).var(axis=2)
    assert np.max(np.abs(yg.mean(axis=2))) < 1e-12
    np.testing.assert_allclose(yg.var(axis=2), var_in / (var_in + eps), rtol=1e-12)
    assert np.max(np.abs(yg.var(axis=2) - 1.0)) < 1e-5


def test_gn_constant_input_and_affine_invariance():
    gamma = RNG.standard_normal(8)
    beta = RNG.standard_normal(8)
    y = ref.group_norm(np.full((1, 8, 3, 3), 7.25), 4, 1e-6, gamma, beta)
    assert np.array_equal(y, np.broadcast_to(beta[None, :, None, None], y.shape))
    x = RNG.standard_normal((2, 8, 6, 5))
    a = ref.group_norm(x, 2, 1e-12, gamma, beta)
    b = ref.group_norm(3.5 * x + 11.0, 2, 1e-12, gamma, beta)
    np.testing.assert_allclose(a, b, atol=1e-9)
    # per-channel affine is applied after normalisation
    c = ref.group_norm(x, 2, 1e-12, np.ones(8), np.zeros(8))
    np.testing.assert_allclose(a, c * gamma[None, :, None, None] + beta[None, :, None, None], atol=1e-12)


def test_silu_closed_forms():
    t = np.linspace(-30, 30, 2001)
    s = ref.silu(t)
    assert ref.silu(np.zeros(1))[0] == 0.0
    np.testing.assert_allclose(s - ref.silu(-t), t, atol=1e-13)          # SiLU(t) - SiLU(-t) = t
    np.testing.assert_allclose(s, t * scipy.special.expit(t), rtol=1e-14, atol=1e-300)
    assert abs(ref.silu(np.array([40.0]))[0] - 40.0) < 1e-12
    assert -1e-12 < ref.silu(np.array([-40.0]))[0] < 0
    # minimum at t* = -(1 + W(1/e)), value t*/(1+exp(-t*)) = -W(1/e)
    w0 = float(np.real(scipy.special.lambertw(1.0 / math.e)))
    tstar = -(1.0 + w0)
    assert abs(ref.silu(np.array([tstar]))[0] + w0) < 1e-14
    fine = ref.silu(np.linspace(-3, 0, 300001))
    assert abs(fine.min() + w0) < 1e-9 and abs(w0 - 0.2784645427610738) < 1e-12
    # fused GN->SiLU equals SiLU of GN
    x = RNG.standard_normal((1, 4, 3, 5))
    g, b = RNG.standard_normal(4), RNG.standard_normal(4)
    assert np.array_equal(ref.group_norm(x, 2, 1e-6, g, b, apply_silu=True),
                          ref.silu(ref.group_norm(x, 2, 1e-6, g, b)))


# ----------------------------------------------------------------- upsample / upconv
def test_upsample_index_invariants():
    x = RNG.standard_normal((2, 3, 5, 7))
    y = ref.upsample2x(x)
    assert y.shape == (2, 3, 10, 14)
    for a in (0, 1):
        for b in (0, 1):
            assert np.array_equal(y[:, :, a::2, b::2], x)
    pooled = y.reshape(2, 3, 5, 2, 7, 2).mean(axis=(3, 5))
    assert np.array_equal(pooled, x)
    assert np.array_equal(y, np.repeat(np.repeat(x, 2, axis=2), 2, axis=3))


def test_upconv_gather_table_exhaustive():
    """The fused gather src = ((oy+ky-1)>>1, (ox+kx-1)>>1), zero outside the upsampled
    grid, enumerates the same taps as materialised upsample + padded 3x3 window."""
    h, w = 3, 4
    ids = np.arange(1, h * w + 1, dtype=np.float64).reshape(1, 1, h, w)  # pixel id, 0 = padding
    up = np.pad(ref.upsample2x(ids)[0, 0], 1)
    for oy, ox, ky, kx in itertools.product(range(2 * h), range(2 * w), range(3), range(3)):
        uy, ux = oy + ky - 1, ox + kx - 1
        fused = ids[0, 0, uy >> 1, ux >> 1] if (0 <= uy < 2 * h and 0 <= ux < 2 * w) else 0.0
        assert fused == up[oy + ky, ox + kx]
        # and the oracle's upconv picks exactly that pixel for a one-hot kernel
    for ky, kx in itertools.product(range(3), range(3)):
        wk = np.zeros((1, 1, 3, 3))
        wk[0, 0, ky, kx] = 1.0
        assert np.array_equal(ref.upconv(ids, wk)[0, 0], up[ky:ky + 2 * h, kx:kx + 2 * w])


def test_upconv_phase_decomposition():
    """Output parity class (py,px) equals a 2x2 conv of the source grid with pre-summed taps."""
    x = RNG.standard_normal((2, 3, 5, 6))
    w = RNG.standard_normal((4, 3, 3, 3))
    b = RNG.standard_normal(4)
    got = ref.upconv(x, w, b)
    n, cin, h, wd = x.shape
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
    # rows: even output row 2i reads source rows {i-1: w0, i: w1+w2}; odd row 2i+1 reads {i: w0+w1, i+1: w2}
    rowsets = {0: [(-1, [0]), (0, [1, 2])], 1: [(0, [0, 1]), (1, [2])]}
    want = np.zeros_like(got)
    for py in (0, 1):
        for px in (0, 1):
            acc = np.zeros((n, 4, h, wd))
            for dy, kys in rowsets[py]:
                for dx, kxs in rowsets[px]:
                    wsum = sum(w[:, :, ky, kx] for ky in kys for kx in kxs)
                    acc += np.einsum("oc,nchw->nohw", wsum, xp[:, :, 1 + dy:1 + dy + h, 1 + dx:1 + dx + wd])
            want[:, :, py::2, px::2] = acc + b[None, :, None, None]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


# ----------------------------------------------------------------- blocks
def _rb_params(cin, cout, random_affine=True):
    p = {
        "norm1.gamma": 1 + 0.2 * RNG.standard_normal(cin), "norm1.beta": 0.2 * RNG.standard_normal(cin),
        "conv1.w": RNG.standard_normal((cout, cin, 3, 3)) / math.sqrt(9 * cin), "conv1.b": 0.01 * RNG.standard_normal(cout),
        "norm2.gamma": 1 + 0.2 * RNG.standard_normal(cout), "norm2.beta": 0.2 * RNG.standard_normal(cout),
        "conv2.w": RNG.standard_normal((cout, cout, 3, 3)) / math.sqrt(9 * cout), "conv2.b": 0.01 * RNG.standard_normal(cout),
    }
    if cin != cout:
        p["shortcut.w"] = RNG.standard_normal((cout, cin, 1, 1)) / math.sqrt(cin)
        p["shortcut.b"] = 0.01 * RNG.standard_normal(cout)
    return p


def np_group_norm(x, groups, eps, gamma, beta):
    n, c, h, w = x.shape
    xg = x.reshape(n, groups, -1)
    y = ((xg - xg.mean(axis=2, keepdims=True)) / np.sqrt(xg.var(axis=2, keepdims=True) + eps)).reshape(x.shape)
    return y * gamma[None, :, None, None] + beta[None, :, None, None]


def np_conv(x, w, b):
    n, cin, h, wd = x.shape
    k = w.shape[2]
    y = np.zeros((n, w.shape[0], h, wd))
    for i in range(n):
        for co in range(w.shape[0]):
            for ci in range(cin):
                y[i, co] += scipy.signal.correlate2d(x[i, ci], w[co, ci], mode="same", boundary="fill")
            y[i, co] += b[co]
    return y


def np_silu(t):
    return t * scipy.special.expit(t)


def np_resblock(x, p, groups, eps):
    h = np_conv(np_silu(np_group_norm(x, groups, eps, p["norm1.gamma"], p["norm1.beta"])), p["conv1.w"], p["conv1.b"])
    h = np_conv(np_silu(np_group_norm(h, groups, eps, p["norm2.gamma"], p["norm2.beta"])), p["conv2.w"], p["conv2.b"])
    s = np_conv(x, p["shortcut.w"], p["shortcut.b"]) if "shortcut.w" in p else x
    return s + h


def test_resblock_zero_branch_and_independent_route():
    x = RNG.standard_normal((2, 8, 6, 7))
    p = _rb_params(8, 8)
    np.testing.assert_allclose(ref.resblock(x, p, 4, 1e-6), np_resblock(x, p, 4, 1e-6), atol=1e-12)
    p["conv2.w"] = np.zeros_like(p["conv2.w"])
    p["conv2.b"] = np.zeros_like(p["conv2.b"])
    assert np.array_equal(ref.resblock(x, p, 4, 1e-6), x)
    q = _rb_params(8, 4)
    np.testing.assert_allclose(ref.resblock(x, q, 4, 1e-6), np_resblock(x, q, 4, 1e-6), atol=1e-12)
    q["conv2.w"] = np.zeros_like(q["conv2.w"])
    q["conv2.b"] = np.zeros_like(q["conv2.b"])
    np.testing.assert_allclose(ref.resblock(x, q, 4, 1e-6),
                               np_conv(x, q["shortcut.w"], q["shortcut.b"]), atol=1e-13)


# ----------------------------------------------------------------- attention
def brute_attention(q, k, v, scale):
    t, d = q.shape
    o = np.zeros((t, d))
    for i in range(t):
        s = [scale * sum(float(q[i, e]) * float(k[j, e]) for e in range(d)) for j in range(t)]
        m = max(s)
        ex = [math.exp(a - m) for a in s]
        z = sum(ex)
        for e in range(d):
            o[i, e] = sum(ex[j] / z * float(v[j, e]) for j in range(t))
    return o


def test_attention_core_pins():
    t, d = 7, 4
    q, k, v = (RNG.standard_normal((t, d)) for _ in range(3))
    sc = 1.0 / math.sqrt(d)
    o = ref.attention_core(q, k, v, sc)
    np.testing.assert_allclose(o, brute_attention(q, k, v, sc), atol=1e-13)
    # library route
    np.testing.assert_allclose(o, scipy.special.softmax(q @ k.T * sc, axis=1) @ v, atol=1e-13)
    # q = 0 -> uniform weights -> mean of v rows
    np.testing.assert_allclose(ref.attention_core(np.zeros((t, d)), k, v, sc),
                               np.broadcast_to(v.mean(axis=0), (t, d)), atol=1e-14)
    # softmax shift invariance: adding a constant vector c to every key shifts row i by q_i.c only
    c = RNG.standard_normal(d)
    np.testing.assert_allclose(ref.attention_core(q, k + c, v, sc), o, atol=1e-12)
    # large scores do not overflow (max subtraction)
    big = ref.attention_core(q * 1e3, k * 1e3, v, 1.0)
    assert np.all(np.isfinite(big))
    # rows of P sum to one: with v = ones, o = ones
    np.testing.assert_allclose(ref.attention_core(q, k, np.ones((t, d)), sc), np.ones((t, d)), atol=1e-14)
    # token permutation equivariance
    perm = RNG.permutation(t)
    np.testing.assert_allclose(ref.attention_core(q[perm], k[perm], v[perm], sc), o[perm], atol=1e-13)
    # one token: o = v
    np.testing.assert_allclose(ref.attention_core(q[:1], k[:1], v[:1], sc), v[:1], atol=1e-15)


def _attn_params(c):
    p = {"norm.gamma": 1 + 0.2 * RNG.standard_normal(c), "norm.beta": 0.2 * RNG.standard_normal(c)}
    for nm in ("q", "k", "v", "proj"):
        p[nm + ".w"] = RNG.standard_normal((c, c, 1, 1)) / math.sqrt(c)
        p[nm + ".b"] = 0.01 * RNG.standard_normal(c)
    return p


def np_attention_block(x, p, groups, eps):
    n, c, hh, ww = x.shape
    h = np_group_norm(x, groups, eps, p["norm.gamma"], p["norm.beta"])
    out = np.empty_like(x)
    for i in range(n):
        tok = h[i].reshape(c, -1).T                                  # [T, C], token = y*W + x
        q = tok @ p["q.w"][:, :, 0, 0].T + p["q.b"]
        k = tok @ p["k.w"][:, :, 0, 0].T + p["k.b"]
        v = tok @ p["v.w"][:, :, 0, 0].T + p["v.b"]
        o = scipy.special.softmax(q @ k.T / math.sqrt(c), axis=1) @ v
        out[i] = x[i] + (o @ p["proj.w"][:, :, 0, 0].T + p["proj.b"]).T.reshape(c, hh, ww)
    return out


def test_attention_block_independent_route():
    x = RNG.standard_normal((2, 8, 3, 5))
    p = _attn_params(8)
    np.testing.assert_allclose(ref.attention_block(x, p, 4, 1e-6), np_attention_block(x, p, 4, 1e-6), atol=1e-12)
    # zero projection -> identity (residual from the un-normalised input)
    p["proj.w"] = np.zeros_like(p["proj.w"])
    p["proj.b"] = np.zeros_like(p["proj.b"])
    assert np.array_equal(ref.attention_block(x, p, 4, 1e-6), x)


# ----------------------------------------------------------------- whole decoder (reduced size)
def test_decoder_reduced_size_independent_route():
    from paper_2602_00608_amd import synth
    chans = (16, 16, 8, 4)
    spec = synth.decoder_weight_spec(level_channels=chans, resblocks_per_level=2, latent_c=4, out_c=3)
    wts = {k: v.astype(np.float64) for k, v in synth.draw_params(spec, 7, random_affine=True).items()}
    z = RNG.standard_normal((2, 4, 3, 5))
    got = ref.decoder(z, wts, level_channels=chans, resblocks_per_level=2, groups=4, eps=1e-6)
    assert got.shape == (2, 3, 24, 40)

    def sub(prefix):
        return {k[len(prefix) + 1:]: v for k, v in wts.items() if k.startswith(prefix + ".")}
    x = np_conv(z, wts["conv_in.w"], wts["conv_in.b"])
    x = np_resblock(x, sub("mid.res1"), 4, 1e-6)
    x = np_attention_block(x, sub("mid.attn"), 4, 1e-6)
    x = np_resblock(x, sub("mid.res2"), 4, 1e-6)
    for l in range(4):
        for i in range(2):
            x = np_resblock(x, sub(f"up.{l}.res{i}"), 4, 1e-6)
        if l < 3:
            x = np.repeat(np.repeat(x, 2, axis=2), 2, axis=3)
            x = np_conv(x, wts[f"up.{l}.upsample.w"], wts[f"up.{l}.upsample.b"])
    x = np_silu(np_group_norm(x, 4, 1e-6, wts["norm_out.gamma"], wts["norm_out.beta"]))
    want = np_conv(x, wts["conv_out.w"], wts["conv_out.b"])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-10)
    # frames are decoded independently
    one = ref.decoder(z[1:2], wts, level_channels=chans, resblocks_per_level=2, groups=4, eps=1e-6)
    np.testing.assert_allclose(one, got[1:2], rtol=0, atol=1e-12)


def test_latent_extrapolation_pins():
    """Alg. 2, hit branch (Sec. IV-C).  A trajectory that really is linear in time, z(t) = a + t*d, is reproduced
    exactly by the scheme with lambda = 1 and v = z(t-1) - z(t-2) (catches a flipped sign, a wrong operand, a
    motion vector that is updated on hits); lambda = 0 is the identity; the step is linear in lambda and in v; k
    hits equal the closed form z + k*lambda*v; a hand loop over a tiny latent."""
    r = np.random.default_rng(77)
    a, d = r.standard_normal((4, 5, 6)), r.standard_normal((4, 5, 6))
    traj = lambda t: a + t * d
    z2, z1 = traj(5.0), traj(6.0)
    got = ref.extrapolated_latents(z1, z1 - z2, 1.0, 3)
    for j in range(3):
        assert np.allclose(got[j], traj(7.0 + j), rtol=0, atol=1e-12)
    z, v = r.standard_normal((2, 3, 3)), r.standard_normal((2, 3, 3))
    assert np.array_equal(ref.latent_extrapolate(z, v, 0.0), z)
    assert np.allclose(ref.latent_extrapolate(z, v, 0.7) - z, 0.7 * v, atol=1e-15)
    assert np.allclose(ref.latent_extrapolate(z, 2.0 * v, 0.35), ref.latent_extrapolate(z, v, 0.7), atol=1e-15)
    k = ref.extrapolated_latents(z, v, 0.3, 4)
    assert k.shape == (4, 2, 3, 3) and np.allclose(k[3], z + 4 * 0.3 * v, atol=1e-14)
    assert ref.extrapolated_latents(z, v, 0.3, 0).shape == (0, 2, 3, 3)
    want = np.empty_like(z)
    for c in range(2):
        for y in range(3):
            for x in range(3):
                want[c, y, x] = z[c, y, x] + 0.3 * v[c, y, x]
    assert np.array_equal(ref.latent_extrapolate(z, v, 0.3), want)
    # extrapolating halfway (lambda = 1/2) twice lands where one full step does
    half = ref.extrapolated_latents(z, v, 0.5, 2)
    assert np.allclose(half[1], ref.latent_extrapolate(z, v, 1.0), atol=1e-15)


def test_adaln_modulation_pins():
    """Sec. IV-B-2: three small projections of one conditioning vector.  Brute-force loops on a tiny case; identity
    matrices return the activated vector itself; SiLU(0) = 0 leaves only the biases; each output is linear in its own
    matrix and blind to the other two; and the row-concatenated matrix in ONE product (what horizontal fusion runs)
    gives the three results side by side."""
    r = np.random.default_rng(88)
    b, dc, dm = 3, 5, 4
    c = r.standard_normal((b, dc))
    p = {n + s: r.standard_normal((dm, dc) if s == ".w" else (dm,)) for n in ("shift", "scale", "gate") for s in (".w", ".b")}
    got = ref.adaln_modulation(c, p, apply_silu=True)
    for k, name in enumerate(("shift", "scale", "gate")):
        want = np.empty((b, dm))
        for i in range(b):
            for j in range(dm):
                acc = p[name + ".b"][j]
                for t in range(dc):
                    x = c[i, t]
                    acc += p[name + ".w"][j, t] * (x / (1.0 + math.exp(-x)))
                want[i, j] = acc
        assert np.allclose(got[k], want, rtol=0, atol=1e-13)
    eye = {n + ".w": np.eye(dc) for n in ("shift", "scale", "gate")}
    eye.update({n + ".b": np.zeros(dc) for n in ("shift", "scale", "gate")})
    for y in ref.adaln_modulation(c, eye, apply_silu=False):
        assert np.array_equal(y, c)
    for k, name in enumerate(("shift", "scale", "gate")):
        assert np.allclose(ref.adaln_modulation(np.zeros((2, dc)), p)[k], np.tile(p[name + ".b"], (2, 1)), atol=1e-15)
    q = dict(p)
    q["scale.w"] = 2.0 * p["scale.w"]
    got2 = ref.adaln_modulation(c, q)
    assert np.array_equal(got2[0], got[0]) and np.array_equal(got2[2], got[2])
    assert np.allclose(got2[1] - p["scale.b"], 2.0 * (got[1] - p["scale.b"]), atol=1e-13)
    w_fused = np.vstack([p["shift.w"], p["scale.w"], p["gate.w"]])
    b_fused = np.concatenate([p["shift.b"], p["scale.b"], p["gate.b"]])
    one = ref.silu(c) @ w_fused.T + b_fused
    assert np.allclose(one, np.hstack(got), rtol=0, atol=1e-13)


def test_rel_err_metric():
    want = np.array([3.0, -4.0])
    assert abs(ref.rel_err(want + np.array([0.0, 0.5]), want) - 0.5 / math.sqrt(12.5)) < 1e-15


def test_reduced_decoder_matches_stored_oracle_values():
    """Drift guard: the oracle's reduced decoder against values it wrote earlier (tests/golden/make_golden.py).
    Not a pin by itself -- the pins are the tests above -- but any change to the oracle's arithmetic shows here."""
    import importlib.util
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    shape, idx, vals, rms = mg.reduced_decoder_samples()
    rows = [l.split() for l in open(os.path.join(here, "golden", "reduced_decoder_f64.txt")) if not l.startswith("#")]
    want_idx = np.array([int(r[0]) for r in rows]); want = np.array([float(r[1]) for r in rows])
    assert shape == (1, 3, 56, 72) and np.array_equal(idx, want_idx)
    assert np.max(np.abs(vals - want)) <= 1e-9 * rms
