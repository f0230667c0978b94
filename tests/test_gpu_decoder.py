"""GPU parity of the composed path: the workload stages (ResBlock, upsample stage)
and decoder_run against the fp64 oracle, plus properties that hold at any size."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2602_00608_amd import synth, wmdec
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def resblock_gpu(xd, p, dtype, groups, eps, out_dtype):
    """ResBlock through the per-op entry points; intermediates stored as `dtype`, last output as out_dtype."""
    n, h, w, cin = xd.shape
    cout = p["conv1.w"].shape[0]
    t = G.TORCH[dtype]
    m1, r1 = G.gn_stats(xd, groups, eps)
    hbuf = torch.empty((n, h, w, cout), dtype=t, device="cuda")
    wmdec.gn_silu_conv3x3(xd, m1, r1, G.dev_f32(p["norm1.gamma"]), G.dev_f32(p["norm1.beta"]), groups, True,
                          G.pack(p["conv1.w"], dtype), G.dev_f32(p["conv1.b"]), None, hbuf)
    m2, r2 = G.gn_stats(hbuf, groups, eps)
    res = xd
    if "shortcut.w" in p:
        res = torch.empty((n, h, w, cout), dtype=t, device="cuda")
        wmdec.gn_conv1x1(xd, None, None, None, None, groups, False, G.pack(p["shortcut.w"], dtype),
                         G.dev_f32(p["shortcut.b"]), None, res)
    y = torch.empty((n, h, w, cout), dtype=G.TORCH[out_dtype], device="cuda")
    wmdec.gn_silu_conv3x3(hbuf, m2, r2, G.dev_f32(p["norm2.gamma"]), G.dev_f32(p["norm2.beta"]), groups, True,
                          G.pack(p["conv2.w"], dtype), G.dev_f32(p["conv2.b"]), res, y)
    return y


def resblock_params(seed, cin, cout, sixteen):
    spec = synth.resblock_spec("rb", cin, cout)
    p = synth.draw_params(spec, seed, sixteen_bit=sixteen)
    return {k[3:]: v for k, v in p.items()}


def test_workload1_resblock_fp32():
    """Single decoder ResBlock, fp32, x[1,64,32,32], GN(32, eps 1e-6, gamma 1, beta 0)."""
    x = synth.activation(0, (1, 64, 32, 32), False)
    p = resblock_params(synth.weight_seed(0), 64, 64, False)
    y = resblock_gpu(G.dev_nhwc(x, "f32"), p, "f32", 32, 1e-6, "f32")
    want = ref.resblock(x, p, 32, 1e-6)
    err = ref.rel_err(G.host_nchw(y), want)
    assert err <= 1e-4, err


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_workload3_resblock_reduced(dtype):
    """The full-resolution ResBlock (128 ch, GN 32) on a 96x136 crop-sized input: spans many tiles, ragged tail."""
    x = synth.activation(2, (1, 128, 96, 136), True)
    p = resblock_params(synth.weight_seed(2), 128, 128, True)
    y = resblock_gpu(G.dev_nhwc(x, dtype), p, dtype, 32, 1e-6, "f32")
    err = ref.rel_err(G.host_nchw(y), ref.resblock(x, p, 32, 1e-6))
    assert err <= G.TOL[dtype], err


def test_resblock_channel_change_shortcut():
    x = synth.activation(7, (2, 64, 20, 28), True)
    p = resblock_params(synth.weight_seed(7), 64, 32, True)
    y = resblock_gpu(G.dev_nhwc(x, "f16"), p, "f16", 32, 1e-6, "f32")
    err = ref.rel_err(G.host_nchw(y), ref.resblock(x, p, 32, 1e-6))
    assert err <= G.TOL["f16"], err


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_workload2_upsample_stage_reduced(dtype):
    """x[1,256,h,w] -> nearest-2x -> conv3x3 256->256 -> ResBlock(256) at reduced size."""
    x = synth.activation(1, (1, 256, 30, 44), True)
    r = np.random.default_rng(synth.weight_seed(1))
    wu, bu = synth.conv_params(r, 256, 256, 3, True)
    p = resblock_params(synth.weight_seed(1) + 1, 256, 256, True)
    xd = G.dev_nhwc(x, dtype)
    u = torch.empty((1, 60, 88, 256), dtype=G.TORCH[dtype], device="cuda")
    wmdec.upsample2x_conv3x3(xd, G.pack_upconv(wu, dtype), G.dev_f32(bu), u)
    y = resblock_gpu(u, p, dtype, 32, 1e-6, "f32")
    want = ref.resblock(ref.upconv(x, wu, bu), p, 32, 1e-6)
    err = ref.rel_err(G.host_nchw(y), want)
    assert err <= G.TOL[dtype], err


# ------------------------------------------------------------------ decoder_run
def make_blob(dec, weights):
    """Canonical weight blob (bytes) from name -> float32 array, laid out by the library's own table."""
    blob = np.zeros(dec.weights_bytes(), np.uint8)
    for name, off, nb, dt, shape in dec.weight_table():
        a = weights[name]
        raw = synth.bf16_bits(a).tobytes() if dt == wmdec.BF16 else np.ascontiguousarray(a, np.float32).tobytes()
        assert len(raw) == nb, name
        blob[off:off + nb] = np.frombuffer(raw, np.uint8)
    return torch.from_numpy(blob).cuda()


def run_decoder(cfg, weights, z, batch=None):
    dec = wmdec.Decoder(cfg)
    packed = torch.empty(dec.packed_bytes(), dtype=torch.uint8, device="cuda")
    dec.pack_weights(make_blob(dec, weights), packed)
    n = z.shape[0]
    ws = torch.empty(dec.workspace_bytes(n), dtype=torch.uint8, device="cuda")
    dec.set_workspace(ws)
    zd = torch.from_numpy(synth.bf16_bits(z).view(np.int16)).view(torch.bfloat16).cuda()
    scale = 8 if cfg.num_levels == 4 else 2 ** (cfg.num_levels - 1)
    out = torch.empty((n, cfg.out_c, cfg.latent_h * scale, cfg.latent_w * scale), dtype=torch.float32, device="cuda")
    dec.run(zd, packed, out)
    torch.cuda.synchronize()
    res = out.cpu().numpy().astype(np.float64)
    dec.close()
    return res


def small_cfg(act_dtype):
    cfg = wmdec.decoder_default_config()
    cfg.latent_h, cfg.latent_w = 7, 9
    cfg.level_channels[0], cfg.level_channels[1], cfg.level_channels[2], cfg.level_channels[3] = 512, 128, 64, 32
    cfg.resblocks_per_level = 2
    cfg.act_dtype = act_dtype
    cfg.max_batch = 3
    return cfg


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_decoder_reduced_size(dtype):
    """A narrower, shallower decoder on an odd-sized latent (7x9 -> 56x72), random GroupNorm affine, batch 3."""
    cfg = small_cfg(G.ENUM[dtype])
    chans = (512, 128, 64, 32)
    spec = synth.decoder_weight_spec(level_channels=chans, resblocks_per_level=2)
    weights = synth.draw_params(spec, synth.weight_seed(9), random_affine=True)
    z = synth.latent_sequence(workload=9, frames=3, h=7, w=9)
    got = run_decoder(cfg, weights, z)
    want = ref.decoder(z, weights, level_channels=chans, resblocks_per_level=2, groups=32, eps=1e-6)
    assert got.shape == want.shape == (3, 3, 56, 72)
    err = ref.rel_err(got, want)
    # 20 convolutions deep: bf16 operands and storage accumulate beyond the single-stage bar (see the
    # full-size test); f16 must meet it
    assert err <= (G.TOL["f16"] if dtype == "f16" else 1e-1), err
    # frames are independent: batched result == one-by-one result, bit for bit
    one = run_decoder(cfg, weights, z[1:2])
    assert np.array_equal(one[0], got[1])


@pytest.fixture(scope="module")
def workload4():
    weights = synth.decoder_weights(4)
    z = synth.latent_single(4)
    want = ref.decoder(z, weights)
    return weights, z, want


def test_time_step_repeats_a_step_without_changing_the_frame():
    """decoder_time_step launches one step of the plan several times on whatever the workspace holds; it must not
    disturb anything a later full run depends on (ticket counters, packed weights, the plan itself)."""
    cfg = small_cfg(wmdec.F16)
    spec = synth.decoder_weight_spec(level_channels=(512, 128, 64, 32), resblocks_per_level=2)
    weights = synth.draw_params(spec, synth.weight_seed(9), random_affine=True)
    z = synth.latent_sequence(workload=9, frames=1, h=7, w=9)
    dec = wmdec.Decoder(cfg)
    packed = torch.empty(dec.packed_bytes(), dtype=torch.uint8, device="cuda")
    dec.pack_weights(make_blob(dec, weights), packed)
    ws = torch.empty(dec.workspace_bytes(1), dtype=torch.uint8, device="cuda")
    dec.set_workspace(ws)
    zd = torch.from_numpy(synth.bf16_bits(z).view(np.int16)).view(torch.bfloat16).cuda()
    scale = 2 ** (cfg.num_levels - 1)
    out = torch.empty((1, cfg.out_c, cfg.latent_h * scale, cfg.latent_w * scale), dtype=torch.float32, device="cuda")
    dec.run(zd, packed, out)
    torch.cuda.synchronize()
    first = out.clone()
    info = dec.step_info()
    for i in range(len(info)):
        ms = dec.time_step(zd, packed, out, i, 2)
        assert ms > 0.0, (i, info[i][0])
    dec.run(zd, packed, out)
    torch.cuda.synchronize()
    assert torch.equal(out, first)
    dec.close()


def test_decoder_run_replays_from_a_captured_graph():
    """decoder_run enqueues only kernels (no memset nodes, no allocation, no synchronisation), so a caller can
    capture it in a HIP graph: every replay, with eager runs and synchronisations in between, must reproduce
    the eager frame bit for bit."""
    cfg = small_cfg(wmdec.F16)
    spec = synth.decoder_weight_spec(level_channels=(512, 128, 64, 32), resblocks_per_level=2)
    weights = synth.draw_params(spec, synth.weight_seed(9), random_affine=True)
    z = synth.latent_sequence(workload=9, frames=2, h=7, w=9)
    dec = wmdec.Decoder(cfg)
    packed = torch.empty(dec.packed_bytes(), dtype=torch.uint8, device="cuda")
    dec.pack_weights(make_blob(dec, weights), packed)
    ws = torch.empty(dec.workspace_bytes(2), dtype=torch.uint8, device="cuda")
    dec.set_workspace(ws)
    zd = torch.from_numpy(synth.bf16_bits(z).view(np.int16)).view(torch.bfloat16).cuda()
    out = torch.empty((2, cfg.out_c, 56, 72), dtype=torch.float32, device="cuda")
    dec.run(zd, packed, out)            # eager: also the one-time set-up (kernel attributes, ticket counters)
    torch.cuda.synchronize()
    eager = out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dec.run(zd, packed, out)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        dec.run(zd, packed, out)
    for _ in range(3):
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager)
        dec.run(zd, packed, out)        # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(out, eager)
    del graph
    dec.close()


def test_decoder_full_size_f16(workload4):
    """Workload 4: z[1,4,60,90] -> [1,3,480,720], full decoder, against the fp64 oracle."""
    weights, z, want = workload4
    cfg = wmdec.decoder_default_config()
    cfg.act_dtype = wmdec.F16
    got = run_decoder(cfg, weights, z)
    err = ref.rel_err(got, want)
    print("full decoder f16: max|err|/rms = %.3e" % err)
    assert err <= G.TOL["f16"], err
    again = run_decoder(cfg, weights, z)
    assert np.array_equal(got, again)          # deterministic


def test_decoder_full_size_bf16_reported(workload4):
    """bf16 operands + bf16 storage through ~37 convolutions: forecast ~5e-2 of the output RMS, above the
    2e-2 bar that f16 meets; asserted only against that forecast and printed."""
    weights, z, want = workload4
    cfg = wmdec.decoder_default_config()
    cfg.act_dtype = wmdec.BF16
    got = run_decoder(cfg, weights, z)
    err = ref.rel_err(got, want)
    print("full decoder bf16: max|err|/rms = %.3e" % err)
    assert err <= 1e-1, err


def test_decoder_batched_workload5_properties():
    """Workload 5: 4 temporally correlated latents.  Batched output equals frame-by-frame output bit for bit."""
    weights = synth.decoder_weights(4)
    z = synth.latent_sequence(5)
    cfg = wmdec.decoder_default_config()
    got = run_decoder(cfg, weights, z)
    assert got.shape == (4, 3, 480, 720) and np.all(np.isfinite(got))
    for t in (0, 3):
        one = run_decoder(cfg, weights, z[t:t + 1])
        assert np.array_equal(one[0], got[t]), t
