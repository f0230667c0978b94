"""The C-ABI library loads, exports every symbol the header declares, and its
host-side logic (argument checks, decoder plan, weight table) behaves -- no GPU needed."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2602_00608_amd import synth, wmdec

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b((?:wmdec|decoder)_[a-z0-9_]+)\s*\(", text))


def test_every_declared_symbol_is_exported_and_bound():
    syms = header_symbols()
    assert {"decoder_create", "decoder_run", "wmdec_gn_stats", "wmdec_gn_silu_conv3x3",
            "wmdec_upsample2x_conv3x3", "wmdec_attention"} <= syms
    l = wmdec.lib()
    for s in syms:
        assert hasattr(l, s), s
    assert syms == set(wmdec.SIGNATURES), syms ^ set(wmdec.SIGNATURES)


def test_no_torch_types_in_header():
    text = open(os.path.join(ROOT, "include", "wmdec.h")).read()
    assert "torch" not in text and "at::" not in text and "extern \"C\"" in text


def test_default_config_and_weight_table_match_input_recipe():
    dec = wmdec.Decoder()
    cfg = dec.cfg
    assert (cfg.latent_c, cfg.latent_h, cfg.latent_w) == (4, 60, 90)
    assert list(cfg.level_channels) == [512, 512, 256, 128] and cfg.groups == 32 and cfg.out_c == 3
    table = dec.weight_table()
    spec = synth.decoder_weight_spec()
    assert [t[0] for t in table] == [s[0] for s in spec]
    for (name, off, nb, dt, shape), (_, sshape) in zip(table, spec):
        full = tuple(sshape) + (1,) * (4 - len(sshape))
        assert shape == full, name
        assert dt == (wmdec.BF16 if name.endswith(".w") else wmdec.F32)
        assert nb == int(np.prod(sshape)) * (2 if name.endswith(".w") else 4)
        assert off % 256 == 0
        assert dec.weight_offset(name) == (off, nb)
    offs = [t[1] for t in table]
    assert offs == sorted(offs) and dec.weights_bytes() >= offs[-1] + table[-1][2]
    nparam = sum(int(np.prod(s[1])) for s in spec)
    assert 49_000_000 < nparam < 50_000_000          # ~49.5 M parameters
    # work of one frame: 3329 GFLOP with every convolution priced at nine taps (incl. 59.7 GFLOP attention core);
    # the default (f16) decoder evaluates its three upsampling convolutions per output phase and executes 2820
    assert abs(dec.dense_flops_per_frame() / 1e9 - 3329) < 5
    assert abs(dec.flops_per_frame() / 1e9 - 2820) < 5
    assert dec.workspace_bytes(1) > 3 * 480 * 720 * 256 * 2
    assert dec.workspace_bytes(5) == 0                # beyond max_batch
    dec.close()


def test_flops_independent_count():
    """Recount the decoder's FLOPs from the weight spec: every conv weight contributes 2*k*k*cin*cout per output
    pixel at the resolution its name implies.  Only executed work counts: where an upsampling convolution is
    evaluated per output phase (the f16 decoder) it executes 2x2 taps per output, 4/9 of the nine-tap figure; the
    bf16 decoder keeps the nine-tap form."""
    res = {"conv_in": 1, "mid": 1, "up.0": 1, "up.1": 2, "up.2": 4, "up.3": 8, "conv_out": 8}
    dense = phase = 0.0
    for name, shape in synth.decoder_weight_spec():
        if not name.endswith(".w"):
            continue
        key = name[:-2].split(".res")[0].split(".attn")[0].split(".upsample")[0]
        s = res[key] * (2 if ".upsample" in name else 1)
        f = 2.0 * np.prod(shape) * (60 * s) * (90 * s)
        dense += f
        phase += f * 4.0 / 9.0 if ".upsample" in name else f
    attn = 4.0 * 5400 * 5400 * 512
    for act, executed in ((wmdec.F16, phase + attn), (wmdec.BF16, dense + attn)):
        cfg = wmdec.decoder_default_config()
        cfg.act_dtype = act
        dec = wmdec.Decoder(cfg)
        assert abs(dec.flops_per_frame() - executed) / executed < 1e-12
        assert abs(dec.dense_flops_per_frame() - (dense + attn)) / (dense + attn) < 1e-12
        dec.close()


def test_step_accounting_adds_up():
    """The per-step figures the benchmark prices kernels with: their FLOPs sum to the frame total, every step
    names its kernel, convolutions carry the instantiation, and the byte count of a ResBlock convolution is
    input + residual + output + weights, each once."""
    dec = wmdec.Decoder()
    info = dec.step_info()
    assert abs(sum(f for _, f, _ in info) - dec.flops_per_frame()) / dec.flops_per_frame() < 1e-12
    assert all(k for k, _, _ in info)
    convs = [(k, f, b) for k, f, b in info if k.startswith("conv_mfma_kernel<")]
    # 30 ResBlock convolutions (the two 1x1 shortcuts are folded into their second convolutions), three upsampling
    # convolutions, qkv and output projection: 33 launches of the implicit-GEMM kernel; conv_out (three output
    # channels) runs as a contraction onto (tap, channel) pairs
    assert len(convs) == 33 and all(k.endswith(">") for k, _, _ in convs)
    assert info[-1][0] == "conv_taps_kernel<wmdec::f16_t, 8, 2>"
    # the ten 512 -> 512 layers at 60x90 leave compute units at most one workgroup: whole-chunk weight ring
    assert sum(1 for k, _, _ in convs if k.endswith(", 18>")) == 10
    # the second convolution of the 512 -> 256 block carries its shortcut: K = 9*256 + 512, and reads the block input
    fold_flops = 2.0 * (9 * 256 + 512) * 256 * 240 * 360
    fold_bytes = (2 * 240 * 360 * 256 + 240 * 360 * 512) * 2 + (9 * 256 * 256 + 512 * 256) * 2
    assert any(f == fold_flops and b == fold_bytes for _, f, b in convs)
    # last ResBlock convolution at 480x720: 128 -> 128, f16, with residual
    want_flops = 2.0 * 9 * 128 * 128 * 480 * 720
    want_bytes = 3 * 480 * 720 * 128 * 2 + 9 * 128 * 128 * 2
    assert any(f == want_flops and b == want_bytes for _, f, b in convs)
    # 30 normalisations: each gets its moments from the convolution that produced its input (conv_in's vector-ALU kernel
    # included), none from a statistics pass over the tensor.  Where that producer is a single round of workgroups
    # (conv_in, the 60x90 and 120x180 layers: 22 normalisations) the consumer's prologue merges either the producer's triples
    # themselves (few tiles) or what its last workgroup per tile row merged; the 8 producers of several rounds (240x360,
    # 480x720) keep a small merge launch.
    assert sum(1 for k, _, _ in info if k == "gn_stats_vec") == 0 and sum(1 for k, _, _ in info if k == "gn_finalize") == 8
    cfg = wmdec.decoder_default_config()
    cfg.separate_merge_launch = 1
    d2 = wmdec.Decoder(cfg)
    assert sum(1 for k, _, _ in d2.step_info() if k == "gn_finalize") == 30 and d2.num_launches() - dec.num_launches() == 22
    d2.close()
    dec.close()


def test_argument_errors_are_reported_without_a_gpu():
    l = wmdec.lib()
    assert l.wmdec_gn_stats(None, 0, 1, 1, 1, 32, 32, 1e-6, None, None, None, 0, None) == wmdec.ERR_INVALID_ARG
    assert b"null" in l.wmdec_last_error()
    # fake but aligned non-null addresses: the checks must fire before anything touches them
    p = 0x1000
    assert l.wmdec_gn_stats(p, 0, 1, 4, 4, 30, 32, 1e-6, p, p, p, 1 << 20, None) == wmdec.ERR_SHAPE
    assert l.wmdec_gn_stats(p, 7, 1, 4, 4, 32, 32, 1e-6, p, p, p, 1 << 20, None) == wmdec.ERR_INVALID_ARG
    assert l.wmdec_gn_stats(p, 0, 0, 4, 4, 32, 32, 1e-6, p, p, p, 1 << 20, None) == wmdec.ERR_INVALID_ARG
    assert l.wmdec_gn_stats(p + 4, 0, 1, 4, 4, 32, 32, 1e-6, p, p, p, 1 << 20, None) == wmdec.ERR_INVALID_ARG
    assert l.wmdec_gn_silu_conv3x3(p, 0, p, p, p, p, 32, 1, p, p, None, 2 * p, 0, 1, 4, 4, 48, 8, None) == wmdec.ERR_SHAPE
    assert l.wmdec_gn_silu_conv3x3(p, 1, None, None, None, None, 32, 1, p, p, None, p, 1, 1, 4, 4, 32, 8, None) == wmdec.ERR_INVALID_ARG  # x == y
    assert l.wmdec_gn_silu_conv3x3(p, 1, None, None, None, None, 32, 1, p, p, None, 2 * p, 2, 1, 4, 4, 32, 8, None) == wmdec.ERR_UNSUPPORTED
    assert l.wmdec_attention(p, 1, p, p, p, p, 32, p, p, p, p, 2 * p, 1, 4, 4, 256, p, 1 << 30, None) == wmdec.ERR_UNSUPPORTED
    assert l.wmdec_attention(p, 1, p, p, p, p, 32, p, p, p, p, 2 * p, 1, 4, 4, 512, p, 16, None) == wmdec.ERR_WORKSPACE
    assert l.wmdec_upsample2x_nearest(p, p, 1, 1, 2, 2, 8, None) == wmdec.ERR_INVALID_ARG
    assert l.wmdec_conv_packed_bytes(64, 64, 3, wmdec.F32) == 9 * 64 * 64 * 4
    assert l.wmdec_conv_packed_bytes(3, 4, 3, wmdec.BF16) == 9 * 32 * 16 * 2   # padded to 32 x 16 fragments
    assert l.wmdec_conv_packed_bytes(64, 64, 2, wmdec.F32) == 0
    # upsampling convolution: the 9-tap pack plus the 16-tap phase pack
    assert l.wmdec_upconv_packed_bytes(64, 64, wmdec.F16) == (9 + 16) * 64 * 64 * 2
    assert l.wmdec_upconv_packed_bytes(64, 64, 9) == 0
    assert l.wmdec_pack_upconv_weights(p, wmdec.F16, 64, 64, 2 * p, wmdec.F16, None) == wmdec.ERR_INVALID_ARG   # source type
    assert l.wmdec_pack_upconv_weights(p, wmdec.F32, 64, 64, 2 * p + 8, wmdec.F16, None) == wmdec.ERR_INVALID_ARG   # alignment
    # statistics on the built-in scratch: same argument checks, no workspace argument
    assert l.wmdec_gn_stats_noalloc(None, 0, 1, 1, 1, 32, 32, 1e-6, None, None, None) == wmdec.ERR_INVALID_ARG
    assert l.wmdec_gn_stats_noalloc(p, 0, 1, 4, 4, 30, 32, 1e-6, p, p, None) == wmdec.ERR_SHAPE
    assert l.wmdec_gn_stats_noalloc(p, 1, 65, 2, 2, 32, 32, 1e-6, p, p, None) == wmdec.ERR_WORKSPACE
    assert b"limit" in l.wmdec_last_error()
    # convolution that also emits the moments of its output
    assert l.wmdec_conv_stats_workspace_bytes(wmdec.F16, wmdec.F16, 1, 480, 720, 128, 128, 32) == 32 * 60 * 45 * 12   # one triple per group and 8x16 tile
    assert l.wmdec_conv_stats_workspace_bytes(wmdec.F32, wmdec.F32, 1, 8, 8, 64, 64, 32) == 0
    assert l.wmdec_gn_silu_conv3x3_stats(p, 2, None, None, None, None, 32, 0, p, None, None, 2 * p, 2, 1, 8, 8, 64, 64,
                                         24, 1e-6, p, p, p, 1 << 20, None) == wmdec.ERR_SHAPE
    assert l.wmdec_gn_silu_conv3x3_stats(p, 2, None, None, None, None, 32, 0, p, None, None, 2 * p, 2, 1, 8, 8, 64, 64,
                                         32, 1e-6, p, p, p, 16, None) == wmdec.ERR_WORKSPACE
    assert l.wmdec_gn_silu_conv3x3_stats(p, 0, None, None, None, None, 32, 0, p, None, None, 2 * p, 0, 1, 8, 8, 64, 64,
                                         32, 1e-6, p, p, p, 1 << 20, None) == wmdec.ERR_UNSUPPORTED
    # convolution with the folded shortcut
    assert l.wmdec_gn_silu_conv3x3_shortcut(p, 2, None, None, None, None, 32, 0, p, None, None, 64, p, None, 2 * p, 2,
                                            1, 8, 8, 64, 64, None) == wmdec.ERR_INVALID_ARG       # no x2
    assert l.wmdec_gn_silu_conv3x3_shortcut(p, 2, None, None, None, None, 32, 0, p, None, 3 * p, 0, p, None, 2 * p, 2,
                                            1, 8, 8, 64, 64, None) == wmdec.ERR_INVALID_ARG       # cin2 = 0
    assert l.wmdec_gn_silu_conv3x3_shortcut(p, 2, None, None, None, None, 32, 0, p, None, 2 * p, 64, p, None, 2 * p, 2,
                                            1, 8, 8, 64, 64, None) == wmdec.ERR_INVALID_ARG       # x2 == y
    # fused AdaLN projections
    assert l.wmdec_adaln_max_batch(1920) == 8 and l.wmdec_adaln_max_batch(0) == 0
    assert l.wmdec_adaln_fused_projection(p, 0, None, 1, None, p, 1, 64, 8, 1, None) == wmdec.ERR_INVALID_ARG
    assert l.wmdec_adaln_fused_projection(p, 0, p, 1, None, 2 * p, 1, 60, 8, 1, None) == wmdec.ERR_SHAPE        # 16-byte vectors
    assert l.wmdec_adaln_fused_projection(p, 0, p, 1, None, 2 * p, 17, 64, 8, 1, None) == wmdec.ERR_UNSUPPORTED  # batch
    # latent extrapolation
    assert l.wmdec_latent_extrapolate(p, None, 1, 0.5, 1, p, 1, 16, None) == wmdec.ERR_INVALID_ARG
    assert l.wmdec_latent_extrapolate(p, p, 1, float("nan"), 1, p, 1, 16, None) == wmdec.ERR_INVALID_ARG
    assert l.wmdec_latent_extrapolate(p, p, 1, 0.5, -1, p, 1, 16, None) == wmdec.ERR_INVALID_ARG
    assert l.wmdec_latent_extrapolate(p, p, 1, 0.5, 1, p, 1, 0, None) == wmdec.OK          # nothing to do
    assert l.wmdec_status_string(wmdec.ERR_WORKSPACE) == b"workspace missing or too small"
    cfg = wmdec.decoder_default_config()
    cfg.level_channels[2] = 250
    h = ctypes.c_void_p()
    assert l.decoder_create(ctypes.byref(cfg), ctypes.byref(h)) == wmdec.ERR_SHAPE and not h.value
    cfg = wmdec.decoder_default_config()
    cfg.act_dtype = wmdec.F32
    assert l.decoder_create(ctypes.byref(cfg), ctypes.byref(h)) == wmdec.ERR_UNSUPPORTED
    dec = wmdec.Decoder()
    assert l.decoder_run(dec.handle, p, p, p, 9, None) == wmdec.ERR_INVALID_ARG
    assert l.decoder_run(dec.handle, p, p, p, 1, None) == wmdec.ERR_WORKSPACE
    assert l.decoder_run_extrapolated(dec.handle, p, None, 0.5, p, p, 1, None) == wmdec.ERR_INVALID_ARG
    assert l.decoder_run_extrapolated(dec.handle, p, p, float("inf"), p, p, 1, None) == wmdec.ERR_INVALID_ARG
    assert l.decoder_run_extrapolated(dec.handle, p, p, 0.5, p, p, 1, None) == wmdec.ERR_WORKSPACE
    ms = ctypes.c_float()
    assert l.decoder_time_step(dec.handle, p, p, p, 1, 0, 1, ctypes.byref(ms), None) == wmdec.ERR_INVALID_ARG   # no run yet
    assert l.decoder_time_step(dec.handle, p, p, p, 1, 999, 1, ctypes.byref(ms), None) == wmdec.ERR_INVALID_ARG
    dec.close()


def test_synth_bf16_rounding_matches_torch():
    import torch
    x = np.random.default_rng(3).standard_normal(100000).astype(np.float32) * 37.0
    x[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]     # exact ties: to even
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = synth.bf16_round(x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    bits = synth.bf16_bits(got)
    assert np.array_equal(bits, torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


def test_synth_is_deterministic_and_shaped():
    a = synth.latent_sequence()
    b = synth.latent_sequence()
    assert a.shape == (4, 4, 60, 90) and np.array_equal(a, b)
    # temporally correlated: consecutive differences are nearly the same step d
    d1, d2 = a[1] - a[0], a[2] - a[1]
    assert np.corrcoef(d1.ravel(), d2.ravel())[0, 1] > 0.95
    z = synth.latent_single()
    assert z.shape == (1, 4, 60, 90) and abs(float(z.std()) - 1.0) < 0.02
    w = synth.decoder_weights()
    assert abs(float(w["mid.res1.conv1.w"].std()) * np.sqrt(9 * 512) - 1.0) < 0.01
    assert abs(float(w["conv_in.b"].std()) - 0.01) < 0.002
    assert np.all(w["norm_out.gamma"] == 1) and np.all(w["norm_out.beta"] == 0)
