"""GPU parity: every per-op entry point of the C ABI against the fp64 oracle on
the same seeded inputs, element by element.  Sizes span several tiles and a
ragged tail; degenerate shapes included."""
import math

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2602_00608_amd import synth, wmdec
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def rng(seed):
    return np.random.default_rng(synth.SEED_BASE + seed)


# ------------------------------------------------------------------ a1: GroupNorm statistics
@pytest.mark.parametrize("dtype,n,c,h,w,groups", [
    ("f32", 1, 64, 32, 32, 32),      # workload 1 shape
    ("f32", 2, 12, 5, 7, 4),         # general path, tiny
    ("bf16", 1, 128, 37, 53, 32),    # 4 channels per group: one 16-byte vector spans two groups
    ("bf16", 2, 256, 24, 36, 32),
    ("f16", 1, 512, 15, 23, 32),     # 16 channels per group: a group spans two vectors
    ("f16", 3, 24, 9, 11, 3),        # general path, 16 bit
    ("f32", 1, 32, 1, 1, 32),        # one element per group: variance 0
    ("bf16", 1, 128, 480, 720, 32),  # workload 3 size
    ("f16", 70, 64, 3, 5, 32),       # more samples than one 256-byte block of ticket counters holds
    ("f16", 2, 1024, 4, 6, 32),      # widest tensor of the single-launch path (one pixel per sweep)
    ("bf16", 1, 2048, 3, 3, 32),     # wider than that: general path
])
def test_gn_stats(dtype, n, c, h, w, groups):
    x = G.stored(rng(1).standard_normal((n, c, h, w)) * 1.7 + 0.6, dtype)
    eps = 1e-6
    mean, rstd = G.gn_stats(G.dev_nhwc(x, dtype), groups, eps)
    wm, wr = ref.gn_stats(x, groups, eps)
    gm, gr = mean.cpu().numpy().reshape(n, groups), rstd.cpu().numpy().reshape(n, groups)
    sd = 1.0 / wr
    assert np.max(np.abs(gm - wm) / sd) < 2e-5, np.max(np.abs(gm - wm) / sd)
    assert np.max(np.abs(gr / wr - 1.0)) < 2e-5, np.max(np.abs(gr / wr - 1.0))


def test_gn_stats_large_offset_no_cancellation():
    # mean >> std: a naive E[x^2]-E[x]^2 in fp32 would lose the variance
    x = (rng(2).standard_normal((1, 64, 40, 40)) * 0.01 + 100.0).astype(np.float32)
    mean, rstd = G.gn_stats(G.dev_nhwc(x, "f32"), 32, 1e-6)
    wm, wr = ref.gn_stats(x, 32, 1e-6)
    assert np.max(np.abs(rstd.cpu().numpy() / wr.ravel() - 1.0)) < 1e-3
    assert np.max(np.abs(mean.cpu().numpy() - wm.ravel())) < 1e-4


def test_gn_stats_deterministic():
    x = G.dev_nhwc(G.stored(rng(3).standard_normal((2, 128, 61, 47)), "bf16"), "bf16")
    a = G.gn_stats(x, 32, 1e-6)
    b = G.gn_stats(x, 32, 1e-6)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_gn_stats_workspace_reuse_across_tensors():
    """One workspace (ticket counters zeroed once) serves many calls on different tensors and shapes of the same
    batch size, back to back on one stream: every call must see only its own partial moments and leave the
    counters at zero for the next."""
    n, groups, eps = 2, 32, 1e-6
    shapes = [(128, 61, 47), (256, 30, 44), (512, 9, 13), (128, 120, 90), (64, 5, 7)]
    ws = torch.zeros(max(wmdec.gn_stats_workspace_bytes(n, h, w, c, groups) for c, h, w in shapes), dtype=torch.uint8, device="cuda")
    xs, outs = [], []
    for rep in range(4):
        for i, (c, h, w) in enumerate(shapes):
            x = G.stored(rng(100 + 10 * rep + i).standard_normal((n, c, h, w)) * (1.0 + i) - rep, "f16")
            xd = G.dev_nhwc(x, "f16")
            mean = torch.empty(n * groups, dtype=torch.float32, device="cuda")
            rstd = torch.empty(n * groups, dtype=torch.float32, device="cuda")
            wmdec.gn_stats(xd, groups, eps, mean, rstd, ws)
            xs.append(x); outs.append((mean, rstd, xd))
    torch.cuda.synchronize()
    for x, (mean, rstd, _) in zip(xs, outs):
        wm, wr = ref.gn_stats(x, groups, eps)
        assert np.max(np.abs(mean.cpu().numpy() - wm.ravel()) * wr.ravel()) < 2e-5
        assert np.max(np.abs(rstd.cpu().numpy() / wr.ravel() - 1.0)) < 2e-5
    assert int(ws[:256].view(torch.int32).abs().sum()) == 0   # tickets back at zero


def test_gn_stats_hand_over_is_never_stale():
    """The single-launch kernel hands partial moments from every workgroup to the last one without a fence (device-
    scope stores, a wait, a ticket).  A stale read would show as a result that differs between repetitions: many
    shapes and batches are run round-robin on one workspace, 40 rounds, and every result must equal the first
    round's bit for bit (and the oracle's to fp32 accuracy)."""
    groups, eps = 32, 1e-6
    shapes = [(1, 128, 480, 720), (2, 256, 120, 180), (4, 512, 60, 90), (3, 128, 61, 47), (1, 1024, 9, 13), (4, 64, 33, 5)]
    xs = [G.dev_nhwc(G.stored(rng(300 + i).standard_normal((n, c, h, w)) * (0.5 + i) + 0.1 * i, "f16"), "f16")
          for i, (n, c, h, w) in enumerate(shapes)]
    ws = torch.zeros(max(wmdec.gn_stats_workspace_bytes(n, h, w, c, groups) for n, c, h, w in shapes), dtype=torch.uint8, device="cuda")
    first = None
    for rnd in range(40):
        outs = []
        for x in xs:
            n = x.shape[0]
            mean = torch.empty(n * groups, dtype=torch.float32, device="cuda")
            rstd = torch.empty(n * groups, dtype=torch.float32, device="cuda")
            wmdec.gn_stats(x, groups, eps, mean, rstd, ws)
            outs.append((mean, rstd))
        torch.cuda.synchronize()
        if first is None:
            first = outs
            for x, (mean, rstd) in zip(xs[1:], outs[1:]):     # the first shape is checked against the oracle elsewhere
                wm, wr = ref.gn_stats(G.host_nchw(x), groups, eps)
                assert np.max(np.abs(mean.cpu().numpy() - wm.ravel()) * wr.ravel()) < 2e-5
                assert np.max(np.abs(rstd.cpu().numpy() / wr.ravel() - 1.0)) < 2e-5
        else:
            for i, ((m0, r0), (m1, r1)) in enumerate(zip(first, outs)):
                assert torch.equal(m0, m1) and torch.equal(r0, r1), (rnd, shapes[i])


# ------------------------------------------------------------------ a3': nearest-2x upsample (bit exact)
@pytest.mark.parametrize("dtype,n,c,h,w", [("bf16", 1, 256, 120, 180), ("f32", 2, 3, 5, 7), ("f16", 1, 8, 1, 1),
                                           ("bf16", 2, 20, 6, 3), ("bf16", 1, 5, 4, 9)])
def test_upsample2x_nearest_bit_exact(dtype, n, c, h, w):
    x = G.stored(rng(4).standard_normal((n, c, h, w)), dtype)
    xd = G.dev_nhwc(x, dtype)
    y, check = G.canaried((n, 2 * h, 2 * w, c), G.TORCH[dtype])
    wmdec.upsample2x_nearest(xd, y)
    check()
    want = ref.upsample2x(x)      # exact in fp64
    got = G.host_nchw(y)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ layout conversion
@pytest.mark.parametrize("sd,dd", [("f32", "f32"), ("f32", "bf16"), ("bf16", "f32"), ("f16", "f16")])
def test_layout_roundtrip(sd, dd):
    x = G.stored(G.stored(rng(5).standard_normal((2, 7, 33, 45)), sd), dd)   # representable in both
    src = torch.from_numpy(x).to(G.TORCH[sd]).cuda()
    nhwc = torch.empty((2, 33, 45, 7), dtype=G.TORCH[dd], device="cuda")
    wmdec.nchw_to_nhwc(src, nhwc)
    assert np.array_equal(G.host_nchw(nhwc), x.astype(np.float64))
    back = torch.empty((2, 7, 33, 45), dtype=G.TORCH[sd], device="cuda")
    wmdec.nhwc_to_nchw(nhwc, back)
    assert torch.equal(back, src)


# ------------------------------------------------------------------ a2/a4: fused norm -> SiLU -> conv3x3 (+bias, +residual)
def run_conv(x, dtype, w, b, res, norm, silu, groups, ydtype, k=3, eps=1e-6, gamma=None, beta=None):
    """x, res: float32 NCHW arrays of storable values; returns (gpu NCHW float64, oracle NCHW float64)."""
    n, cin, h, wd = x.shape
    cout = w.shape[0]
    xd = G.dev_nhwc(x, dtype)
    wp = G.pack(w, dtype)
    wq = G.stored(w, dtype) if dtype != "f32" else w
    y, check = G.canaried((n, h, wd, cout), G.TORCH[ydtype])
    mean = rstd = gd = bd = None
    if norm:
        mean, rstd = G.gn_stats(xd, groups, eps)
        gd, bd = G.dev_f32(gamma), G.dev_f32(beta)
    fn = wmdec.gn_silu_conv3x3 if k == 3 else wmdec.gn_conv1x1
    fn(xd, mean, rstd, gd, bd, groups, silu, wp, None if b is None else G.dev_f32(b),
       None if res is None else G.dev_nhwc(res, dtype), y)
    torch.cuda.synchronize()
    check()
    u = x.astype(np.float64)
    if norm:
        u = ref.group_norm(u, groups, eps, gamma, beta, apply_silu=silu)
    want = ref.conv2d(u, wq, b)
    if res is not None:
        want = want + res
    return G.host_nchw(y), want


CONV_CASES = [
    # dtype, ydtype, n, cin, cout, h, w, norm, silu, bias, residual
    ("f32", "f32", 1, 64, 64, 32, 32, True, True, True, True),       # workload 1 conv
    ("f32", "f32", 2, 4, 3, 5, 7, False, False, True, False),        # tiny, odd channels
    ("f32", "f32", 1, 12, 20, 9, 10, True, True, False, True),
    ("f32", "f32", 1, 8, 8, 1, 1, True, False, True, False),         # one pixel
    ("bf16", "f32", 1, 128, 128, 40, 56, True, True, True, True),
    ("bf16", "bf16", 2, 64, 96, 19, 21, True, True, True, True),
    ("f16", "f16", 1, 256, 128, 17, 33, True, True, True, False),
    ("f16", "f32", 1, 128, 3, 24, 31, True, True, True, False),      # conv_out shape class
    ("bf16", "f32", 1, 4, 64, 12, 18, False, False, True, False),    # conv_in shape class
    ("f16", "f16", 2, 4, 512, 9, 70, False, False, True, False),     # conv_in: two channel blocks, three row segments
    ("f16", "f16", 1, 7, 100, 5, 33, False, False, False, False),    # few input channels, ragged channel block
    ("bf16", "f32", 1, 512, 512, 15, 23, True, True, True, True),
    ("f16", "f32", 1, 32, 32, 64, 3, True, True, True, True),        # narrow image
]


@pytest.mark.parametrize("dtype,ydtype,n,cin,cout,h,w,norm,silu,bias,residual", CONV_CASES)
def test_gn_silu_conv3x3(dtype, ydtype, n, cin, cout, h, w, norm, silu, bias, residual):
    r = rng(10)
    x = G.stored(r.standard_normal((n, cin, h, w)) * 1.3 + 0.2, dtype)
    wt, b = synth.conv_params(r, cout, cin, 3, dtype != "f32")
    res = G.stored(r.standard_normal((n, cout, h, w)), dtype) if residual else None
    groups = 32 if cin % 32 == 0 else 4
    gamma = (1 + 0.2 * r.standard_normal(cin)).astype(np.float32)
    beta = (0.2 * r.standard_normal(cin)).astype(np.float32)
    got, want = run_conv(x, dtype, wt, b if bias else None, res, norm, silu, groups, ydtype, gamma=gamma, beta=beta)
    err = ref.rel_err(got, want)
    tol = G.TOL[dtype]
    assert err <= tol, err
    if dtype != "f32" and ydtype == "f32":
        assert err <= tol / 2, err   # fp32 output of 16-bit operands: well inside the bar


# moments of a convolution's own output from its epilogue: one case per tile shape of the matrix-core kernel
@pytest.mark.parametrize("dtype,ydtype,n,cin,cout,h,w,residual", [
    ("f16", "f16", 1, 128, 128, 40, 56, True),      # 128 x 128 tile, wavefronts 2x2
    ("bf16", "bf16", 2, 256, 128, 24, 36, True),    # two samples
    ("f16", "f16", 1, 64, 64, 17, 33, False),       # 128 x 64 tile, ragged
    ("f16", "f32", 1, 128, 256, 19, 21, False),     # fp32 output: nothing is rounded
    ("bf16", "bf16", 1, 64, 512, 9, 13, True),      # 16 channels per group: a group spans two channel octets
    ("f16", "f16", 1, 256, 256, 240, 360, True),    # 128 x 128 tile with one weight fragment per four MFMAs
    ("f16", "f16", 1, 128, 128, 480, 720, True),    # 256 x 128 tile (full-resolution layer)
    ("bf16", "bf16", 1, 128, 128, 480, 720, False),
    ("f16", "f16", 1, 4, 512, 60, 90, False),       # conv_in: the kernel for few input channels, no normalisation of x
    ("bf16", "bf16", 2, 4, 64, 13, 37, False),      # two channels per group, ragged segment, two samples
    ("f16", "f16", 1, 8, 2048, 5, 50, False),       # 64 channels per group: a group is a whole wavefront
])
def test_conv_epilogue_statistics(dtype, ydtype, n, cin, cout, h, w, residual):
    """wmdec_gn_silu_conv3x3_stats: mean / rstd of the tensor the kernel stored, per (sample, output group), must
    equal the oracle's statistics of exactly that stored tensor, and the streaming pass over it, to fp32 accuracy."""
    r = rng(14)
    groups, eps = 32, 1e-6
    x = G.stored(r.standard_normal((n, cin, h, w)) * 1.3 + 0.2, dtype)
    wt, b = synth.conv_params(r, cout, cin, 3, True)
    b = (b + 0.5).astype(np.float32)                 # a mean well away from zero
    xd = G.dev_nhwc(x, dtype)
    res = G.dev_nhwc(G.stored(r.standard_normal((n, cout, h, w)), dtype), dtype) if residual else None
    norm = cin % groups == 0
    mean, rstd = G.gn_stats(xd, groups, eps) if norm else (None, None)
    gamma = G.dev_f32((1 + 0.2 * r.standard_normal(cin)).astype(np.float32)) if norm else None
    beta = G.dev_f32((0.2 * r.standard_normal(cin)).astype(np.float32)) if norm else None
    y = torch.empty((n, h, w, cout), dtype=G.TORCH[ydtype], device="cuda")
    nbytes = wmdec.conv_stats_workspace_bytes(G.ENUM[dtype], G.ENUM[ydtype], n, h, w, cin, cout, groups)
    assert nbytes > 0
    ws = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")     # needs no initialisation
    mo = torch.empty(n * groups, dtype=torch.float32, device="cuda")
    ro = torch.empty(n * groups, dtype=torch.float32, device="cuda")
    wmdec.gn_silu_conv3x3_stats(xd, mean, rstd, gamma, beta, groups, norm, G.pack(wt, dtype), G.dev_f32(b), res, y,
                                groups, eps, mo, ro, ws)
    torch.cuda.synchronize()
    wm, wr = ref.gn_stats(G.host_nchw(y), groups, eps)
    em = float(np.max(np.abs(mo.cpu().numpy() - wm.ravel()) * wr.ravel()))
    er = float(np.max(np.abs(ro.cpu().numpy() / wr.ravel() - 1.0)))
    assert em < 2e-5 and er < 2e-5, (em, er)
    m2, r2 = G.gn_stats(y, groups, eps)
    assert float(torch.max(torch.abs(mo - m2) * r2)) < 2e-5 and float(torch.max(torch.abs(ro / r2 - 1.0))) < 2e-5
    # the tensor itself is the one the plain entry point writes
    y2 = torch.empty_like(y)
    wmdec.gn_silu_conv3x3(xd, mean, rstd, gamma, beta, groups, norm, G.pack(wt, dtype), G.dev_f32(b), res, y2)
    assert torch.equal(y, y2)


def test_conv_epilogue_statistics_unsupported_shapes_are_refused():
    x = torch.zeros((1, 8, 8, 32), dtype=torch.float32, device="cuda")
    assert wmdec.conv_stats_workspace_bytes(wmdec.F32, wmdec.F32, 1, 8, 8, 32, 64, 32) == 0
    assert wmdec.conv_stats_workspace_bytes(wmdec.F16, wmdec.F16, 1, 8, 8, 32, 96, 32) == 0     # 3 channels per group
    y = torch.zeros((1, 8, 8, 64), dtype=torch.float32, device="cuda")
    ws = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    mo = torch.zeros(32, dtype=torch.float32, device="cuda")
    with pytest.raises(wmdec.WmdecError) as e:
        wmdec.gn_silu_conv3x3_stats(x, None, None, None, None, 32, False, ws, None, None, y, 32, 1e-6, mo, mo.clone(), ws)
    assert e.value.status == wmdec.ERR_UNSUPPORTED


# second convolution of a channel-changing ResBlock with the 1x1 shortcut folded into its contraction
@pytest.mark.parametrize("dtype,ydtype,n,cin,cin2,cout,h,w", [
    ("f16", "f32", 1, 256, 512, 256, 24, 36),       # 128 x 128 tile, wavefronts 2x2
    ("bf16", "bf16", 2, 128, 256, 128, 40, 56),
    ("f16", "f16", 1, 64, 96, 64, 17, 33),          # 128 x 64 tile, ragged, cin2 not a multiple of 64
    ("f16", "f16", 1, 32, 64, 32, 20, 28),          # cout % 64 != 0: two launches of the general kernel
    ("f32", "f32", 1, 24, 12, 40, 7, 9),            # fp32 path
    ("f16", "f16", 1, 256, 512, 256, 240, 360),     # full size: tile with one weight fragment per four MFMAs
    ("f16", "f32", 1, 128, 256, 128, 480, 720),     # full size: 256 x 128 tile
    ("bf16", "f32", 1, 128, 256, 128, 480, 720),
])
def test_gn_silu_conv3x3_shortcut(dtype, ydtype, n, cin, cin2, cout, h, w):
    r = rng(15)
    sixteen = dtype != "f32"
    x = G.stored(r.standard_normal((n, cin, h, w)) * 1.3 + 0.2, dtype)
    x2 = G.stored(r.standard_normal((n, cin2, h, w)), dtype)
    wt, b = synth.conv_params(r, cout, cin, 3, sixteen)
    w2, b2 = synth.conv_params(r, cout, cin2, 1, sixteen)
    groups = 32 if cin % 32 == 0 else 4
    gamma = (1 + 0.2 * r.standard_normal(cin)).astype(np.float32)
    beta = (0.2 * r.standard_normal(cin)).astype(np.float32)
    xd, x2d = G.dev_nhwc(x, dtype), G.dev_nhwc(x2, dtype)
    mean, rstd = G.gn_stats(xd, groups, 1e-6)
    y, check = G.canaried((n, h, w, cout), G.TORCH[ydtype])
    wmdec.gn_silu_conv3x3_shortcut(xd, mean, rstd, G.dev_f32(gamma), G.dev_f32(beta), groups, True, G.pack(wt, dtype),
                                   G.dev_f32(b), x2d, G.pack(w2, dtype), G.dev_f32(b2), y)
    torch.cuda.synchronize()
    check()
    want = ref.conv2d(ref.group_norm(x, groups, 1e-6, gamma, beta, apply_silu=True), wt, b) + ref.conv2d(x2, w2, b2)
    err = ref.rel_err(G.host_nchw(y), want)
    assert err <= G.TOL[dtype] / (2 if sixteen and ydtype == "f32" else 1), err


def test_conv_padding_is_applied_after_activation():
    # constant input, beta chosen so that SiLU(GN(x)) != 0: border outputs must see zeros, not SiLU(beta)
    x = np.full((1, 32, 6, 6), 3.0, np.float32)
    w = np.zeros((32, 32, 3, 3), np.float32)
    w[:, :, :, :] = 1.0 / 32
    gamma, beta = np.ones(32, np.float32), np.full(32, 2.0, np.float32)
    got, want = run_conv(x, "f32", w, None, None, True, True, 32, "f32", gamma=gamma, beta=beta)
    s = 2.0 / (1 + math.exp(-2.0))
    assert abs(want[0, 0, 0, 0] - 4 * s) < 1e-12 and abs(want[0, 0, 2, 2] - 9 * s) < 1e-12
    assert ref.rel_err(got, want) < 1e-5


@pytest.mark.parametrize("dtype,ydtype,n,cin,cout,h,w,norm,residual", [
    ("f32", "f32", 1, 24, 40, 7, 9, True, True),
    ("bf16", "f32", 1, 512, 256, 24, 36, False, False),      # ResBlock shortcut shape class
    ("f16", "f16", 2, 512, 1536, 5, 7, True, False),         # fused q,k,v projection shape class
    ("bf16", "bf16", 1, 256, 128, 31, 17, False, True),
])
def test_gn_conv1x1(dtype, ydtype, n, cin, cout, h, w, norm, residual):
    r = rng(11)
    x = G.stored(r.standard_normal((n, cin, h, w)), dtype)
    wt, b = synth.conv_params(r, cout, cin, 1, dtype != "f32")
    res = G.stored(r.standard_normal((n, cout, h, w)), dtype) if residual else None
    groups = 32 if cin % 32 == 0 else 4
    gamma = (1 + 0.2 * r.standard_normal(cin)).astype(np.float32)
    beta = (0.2 * r.standard_normal(cin)).astype(np.float32)
    got, want = run_conv(x, dtype, wt, b, res, norm, False, groups, ydtype, k=1, gamma=gamma, beta=beta)
    assert ref.rel_err(got, want) <= G.TOL[dtype]


# ------------------------------------------------------------------ a3: upsample-conv
@pytest.mark.parametrize("dtype,ydtype,n,cin,cout,h,w", [
    ("f32", "f32", 1, 6, 10, 5, 7),
    ("bf16", "f32", 1, 256, 256, 20, 28),
    ("f16", "f16", 2, 128, 64, 9, 13),
    ("bf16", "bf16", 1, 64, 64, 1, 1),
])
def test_upsample2x_conv3x3(dtype, ydtype, n, cin, cout, h, w):
    r = rng(12)
    x = G.stored(r.standard_normal((n, cin, h, w)), dtype)
    wt, b = synth.conv_params(r, cout, cin, 3, dtype != "f32")
    y, check = G.canaried((n, 2 * h, 2 * w, cout), G.TORCH[ydtype])
    wmdec.upsample2x_conv3x3(G.dev_nhwc(x, dtype), G.pack_upconv(wt, dtype), G.dev_f32(b), y)
    torch.cuda.synchronize()
    check()
    want = ref.upconv(x, G.stored(wt, dtype) if dtype != "f32" else wt, b)
    assert ref.rel_err(G.host_nchw(y), want) <= G.TOL[dtype] / (2 if ydtype == "f32" else 1)


# 32 channels: general kernel; 64: matrix-core kernel, 3x3 form (bf16) and phase-decomposed form (f16)
@pytest.mark.parametrize("ch,dtype", [(32, "bf16"), (64, "bf16"), (64, "f16")])
def test_upconv_gather_index_map_bit_exact(ch, dtype):
    """One-hot kernels turn the fused upsample-conv into a pure gather: the output must equal the
    shifted, zero-padded upsampled input bit for bit, for all nine taps."""
    r = rng(13)
    x = G.stored(r.standard_normal((1, ch, 7, 10)), dtype)
    up = np.pad(ref.upsample2x(x), ((0, 0), (0, 0), (1, 1), (1, 1)))
    xd = G.dev_nhwc(x, dtype)
    for ky in range(3):
        for kx in range(3):
            w = np.zeros((ch, ch, 3, 3), np.float32)
            for c in range(ch):
                w[c, c, ky, kx] = 1.0
            y = torch.empty((1, 14, 20, ch), dtype=G.TORCH[dtype], device="cuda")
            wmdec.upsample2x_conv3x3(xd, G.pack_upconv(w, dtype), None, y)
            assert np.array_equal(G.host_nchw(y), up[:, :, ky:ky + 14, kx:kx + 20]), (ky, kx)


# ------------------------------------------------------------------ a5: attention block
def run_attention(dtype, n, h, w, seed, sharpen=None):
    c, groups, eps = 512, 32, 1e-6
    r = rng(seed)
    x = G.stored(r.standard_normal((n, c, h, w)), dtype)
    p = {"norm.gamma": (1 + 0.2 * r.standard_normal(c)).astype(np.float32),
         "norm.beta": (0.2 * r.standard_normal(c)).astype(np.float32)}
    for nm in ("q", "k", "v", "proj"):
        p[nm + ".w"], p[nm + ".b"] = synth.conv_params(r, c, c, 1, True)
    # f16: sharpen the softmax (logit std 4 instead of 1) so that it is far from uniform.  bf16 keeps
    # logit std 1: q and k stored with 8 significant bits put an error of ~0.2% x logit std on every
    # logit, which a peaked softmax amplifies beyond the 2e-2 bar (a property of the format, not the kernel).
    if sharpen is None:
        sharpen = 2.0 if dtype == "f16" else 1.0
    p["q.w"] = synth.bf16_round(p["q.w"] * sharpen)
    p["k.w"] = synth.bf16_round(p["k.w"] * sharpen)
    xd = G.dev_nhwc(x, dtype)
    mean, rstd = G.gn_stats(xd, groups, eps)
    wqkv = np.concatenate([p["q.w"], p["k.w"], p["v.w"]], axis=0)
    bqkv = np.concatenate([p["q.b"], p["k.b"], p["v.b"]])
    ws = torch.empty(wmdec.attention_workspace_bytes(n, h, w, c), dtype=torch.uint8, device="cuda")
    y, check = G.canaried((n, h, w, c), G.TORCH[dtype])
    wmdec.attention(xd, mean, rstd, G.dev_f32(p["norm.gamma"]), G.dev_f32(p["norm.beta"]), groups,
                    G.pack(wqkv, dtype), G.dev_f32(bqkv), G.pack(p["proj.w"], dtype), G.dev_f32(p["proj.b"]), y, ws)
    torch.cuda.synchronize()
    check()
    want = ref.attention_block(x, p, groups, eps)
    run_attention.last_params = p
    return G.host_nchw(y), want, x


def branch_tolerance(dtype, want, x):
    """Bound for the attention branch y - x.  The kernel's own error is held to 3x the bar; on top of it the output
    y is stored in `dtype`, whose rounding error (half an ulp: 2^-9 |y| in bf16, 2^-12 |y| in f16) lands entirely
    in the branch, which is small against y when many tokens are averaged."""
    ulp_half = 2.0 ** -9 if dtype == "bf16" else 2.0 ** -12
    rms_branch = math.sqrt(float(np.mean((want - x) ** 2)))
    return 3 * G.TOL[dtype] + ulp_half * float(np.max(np.abs(want))) / rms_branch


# 5x7, 1x1: one ragged query block; 9x8, 16x20: several query blocks with a ragged last one and two key splits;
# 13x37 = 481 tokens: 8 query blocks (the last holds one query), 16 key blocks over 8 splits
@pytest.mark.parametrize("dtype,n,h,w", [("f16", 1, 5, 7), ("bf16", 2, 9, 8), ("f16", 1, 1, 1), ("bf16", 1, 16, 20),
                                         ("f16", 2, 13, 37)])
def test_attention_small(dtype, n, h, w):
    got, want, x = run_attention(dtype, n, h, w, 20)
    assert ref.rel_err(got, want) <= G.TOL[dtype]
    # the attention branch itself (output minus residual input) must agree too, not just x + small
    assert ref.rel_err(got - x, want - x) <= branch_tolerance(dtype, want, x)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_attention_full_size_5400_tokens(dtype):
    got, want, x = run_attention(dtype, 1, 60, 90, 21)
    assert ref.rel_err(got, want) <= G.TOL[dtype]
    assert ref.rel_err(got - x, want - x) <= branch_tolerance(dtype, want, x)


def test_attention_bf16_sharp_softmax_with_the_same_storage_points():
    """bf16 with a 4x sharper softmax (logit std 4).  q and k stored with 8 significant bits shift every logit by
    ~0.16 % of its size, and a peaked softmax turns that into percents of the output: a property of the format,
    which the plain oracle (exact q, k) does not share.  So here the oracle is given the same storage points: its
    q, k, v are rounded to bf16 where the kernel stores them, everything else stays fp64.  Against that reference
    the kernel itself must meet the bar, branch included."""
    dtype, n, h, w = "bf16", 1, 16, 20
    got, _, x = run_attention(dtype, n, h, w, 22, sharpen=2.0)
    p = run_attention.last_params
    c, groups, eps = 512, 32, 1e-6
    hn = ref.group_norm(x, groups, eps, p["norm.gamma"], p["norm.beta"], apply_silu=False)
    hn = G.stored(hn, dtype)                       # MFMA operand of the projection
    q, k, v = (G.stored(ref.conv2d(hn, p[m + ".w"], p[m + ".b"]), dtype).astype(np.float64) for m in ("q", "k", "v"))
    tok = lambda a: np.ascontiguousarray(a[0].reshape(c, h * w).T)
    o = ref.attention_core(tok(q), tok(k), tok(v), 1.0 / math.sqrt(c)).T.reshape(1, c, h, w)
    want = x + ref.conv2d(o, p["proj.w"], p["proj.b"])
    assert ref.rel_err(got, want) <= G.TOL[dtype]
    assert ref.rel_err(got - x, want - x) <= branch_tolerance(dtype, want, x)


# ------------------------------------------------------------------ horizontally fused AdaLN projections (DiT)
# d_model = d_cond = 1920 stands for the paper's 30-head transformer (64 per head; the paper gives no widths)
@pytest.mark.parametrize("cdtype,wdtype,batch,d_cond,d_model,silu", [
    ("f32", "bf16", 1, 1920, 1920, True),      # one frame's conditioning vector
    ("f32", "bf16", 4, 1920, 1920, True),      # a batch of four frames
    ("bf16", "bf16", 8, 1920, 1920, True),
    ("f16", "f16", 3, 520, 77, False),         # ragged: d_cond not a multiple of a wavefront's 512, rows of 8 and 32
    ("f32", "f32", 2, 12, 5, True),
    ("f32", "bf16", 16, 1024, 40, True),       # the largest batch one launch takes
])
def test_adaln_fused_projection(cdtype, wdtype, batch, d_cond, d_model, silu):
    """One launch on the row-concatenated [W_shift; W_scale; W_gate] against the oracle's three separate products."""
    sixteen = wdtype != "f32"
    p = synth.adaln_params(synth.weight_seed(20), d_model, d_cond, sixteen_bit=sixteen)
    if wdtype == "f16":
        p = {k: (G.stored(v, "f16") if k.endswith(".w") else v) for k, v in p.items()}
    c = G.stored(rng(30).standard_normal((batch, d_cond)) * 1.5, cdtype)
    w_fused = np.vstack([p["shift.w"], p["scale.w"], p["gate.w"]])
    b_fused = np.concatenate([p["shift.b"], p["scale.b"], p["gate.b"]])
    cd = torch.from_numpy(c).to(G.TORCH[cdtype]).cuda()
    wd = torch.from_numpy(w_fused).to(G.TORCH[wdtype]).cuda()
    out, check = G.canaried((batch, 3 * d_model), torch.float32)
    wmdec.adaln_fused_projection(cd, wd, G.dev_f32(b_fused), out, apply_silu=silu)
    torch.cuda.synchronize()
    check()
    shift, scale, gate = ref.adaln_modulation(c, p, apply_silu=silu)
    got = out.cpu().numpy().astype(np.float64)
    for k, want in enumerate((shift, scale, gate)):
        err = ref.rel_err(got[:, k * d_model:(k + 1) * d_model], want)
        assert err <= 1e-4, (k, err)          # fp32 products and sums of exactly stored operands


def test_adaln_fused_projection_limits():
    assert wmdec.adaln_max_batch(1920) == 8 and wmdec.adaln_max_batch(512) == 16
    c = torch.zeros((9, 1920), dtype=torch.float32, device="cuda")
    w = torch.zeros((24, 1920), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((9, 24), dtype=torch.float32, device="cuda")
    with pytest.raises(wmdec.WmdecError) as e:
        wmdec.adaln_fused_projection(c, w, None, out)
    assert e.value.status == wmdec.ERR_UNSUPPORTED


# ------------------------------------------------------------------ measurement helper: the plain copy of known traffic
@pytest.mark.parametrize("nbytes", [16, 16 * 255, (1 << 20) + 16 * 7, 256 << 20])
def test_measure_copy_bit_exact(nbytes):
    """wmdec_measure_copy moves exactly the bytes it is given (counter passes are scaled by its traffic) and nothing
    next to them; sizes and pointers that are not multiples of 16, and overlapping ranges, are refused."""
    g = torch.Generator(device="cuda").manual_seed(nbytes % 9973)
    src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=g)
    big = torch.full((nbytes + 512,), 0x5A, dtype=torch.uint8, device="cuda")
    dst = big[256:256 + nbytes]
    wmdec.measure_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert bool((big[:256] == 0x5A).all()) and bool((big[256 + nbytes:] == 0x5A).all())
    if nbytes >= 64:
        for bad_src, bad_dst in ((src[:24], dst[:24]), (src[8:40], dst[:32]), (big[:64], big[32:96])):
            with pytest.raises(wmdec.WmdecError) as e:
                wmdec.measure_copy(bad_src, bad_dst)
            assert e.value.status == wmdec.ERR_INVALID_ARG
