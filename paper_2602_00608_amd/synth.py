"""Seeded synthetic inputs for the decoder workloads.

This module only draws random tensors and quantises them to the storage type
of a workload; it contains none of the decoder's arithmetic.  Both the HIP
path's callers and the CPU oracle's callers take their inputs from here, so
the two sides see bit-identical values.

Recipe: numpy `default_rng(seed).standard_normal(shape)` in float64, scaled,
cast to float32; tensors a workload stores in 16 bit are then rounded to
bfloat16 (round to nearest even) and handed out as float32 holding those
values.  Conv / linear weights have std 1/sqrt(fan_in) with fan_in = k*k*C_in,
biases have std 0.01, GroupNorm gamma = 1 and beta = 0 unless a test asks for
random ones.  Seeds: SEED_BASE*10 + workload index for activations, +100 for
weights.  Tensors are drawn in the order of `decoder_weight_spec`.
"""
import math

import numpy as np

SEED_BASE = 260200608

LEVEL_CHANNELS = (512, 512, 256, 128)
RESBLOCKS_PER_LEVEL = 3
LATENT_C, LATENT_H, LATENT_W = 4, 60, 90
OUT_C = 3
GROUPS = 32
EPS = 1e-6


def input_seed(workload):
    return SEED_BASE * 10 + int(workload)


def weight_seed(workload):
    return SEED_BASE * 10 + int(workload) + 100


def bf16_round(x):
    """Round float32 values to the nearest bfloat16 (ties to even); result is float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32).reshape(x.shape)


def bf16_bits(x):
    """uint16 bit patterns of float32 values that are already bfloat16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bfloat16-representable"
    return (u >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def normal(rng, shape, std=1.0, sixteen_bit=False):
    a = (rng.standard_normal(shape) * std).astype(np.float32)
    return bf16_round(a) if sixteen_bit else a


def conv_params(rng, cout, cin, k, sixteen_bit):
    """(w[cout,cin,k,k] ~ N(0, std=1/sqrt(k*k*cin)), b[cout] ~ N(0, std=0.01))."""
    w = normal(rng, (cout, cin, k, k), 1.0 / math.sqrt(k * k * cin), sixteen_bit)
    b = normal(rng, (cout,), 0.01, False)
    return w, b


def resblock_spec(prefix, cin, cout):
    spec = [
        (prefix + ".norm1.gamma", (cin,)), (prefix + ".norm1.beta", (cin,)),
        (prefix + ".conv1.w", (cout, cin, 3, 3)), (prefix + ".conv1.b", (cout,)),
        (prefix + ".norm2.gamma", (cout,)), (prefix + ".norm2.beta", (cout,)),
        (prefix + ".conv2.w", (cout, cout, 3, 3)), (prefix + ".conv2.b", (cout,)),
    ]
    if cin != cout:
        spec += [(prefix + ".shortcut.w", (cout, cin, 1, 1)), (prefix + ".shortcut.b", (cout,))]
    return spec


def decoder_weight_spec(level_channels=LEVEL_CHANNELS, resblocks_per_level=RESBLOCKS_PER_LEVEL,
                        latent_c=LATENT_C, out_c=OUT_C):
    """[(name, shape)] of every decoder parameter, in execution order."""
    c0 = level_channels[0]
    spec = [("conv_in.w", (c0, latent_c, 3, 3)), ("conv_in.b", (c0,))]
    spec += resblock_spec("mid.res1", c0, c0)
    spec += [("mid.attn.norm.gamma", (c0,)), ("mid.attn.norm.beta", (c0,))]
    for nm in ("q", "k", "v", "proj"):
        spec += [(f"mid.attn.{nm}.w", (c0, c0, 1, 1)), (f"mid.attn.{nm}.b", (c0,))]
    spec += resblock_spec("mid.res2", c0, c0)
    prev = c0
    for l, c in enumerate(level_channels):
        for i in range(resblocks_per_level):
            spec += resblock_spec(f"up.{l}.res{i}", prev if i == 0 else c, c)
        prev = c
        if l + 1 < len(level_channels):
            spec += [(f"up.{l}.upsample.w", (c, c, 3, 3)), (f"up.{l}.upsample.b", (c,))]
    spec += [("norm_out.gamma", (prev,)), ("norm_out.beta", (prev,)),
             ("conv_out.w", (out_c, prev, 3, 3)), ("conv_out.b", (out_c,))]
    return spec


def draw_params(spec, seed, sixteen_bit=True, random_affine=False):
    """dict name -> float32 array following `spec` order.  '.w' tensors are conv
    weights (std 1/sqrt(fan_in), stored 16 bit when asked), '.b' biases (std 0.01),
    gamma/beta are 1/0 or, with random_affine, 1+0.2*N(0,1) and 0.2*N(0,1)."""
    rng = np.random.default_rng(seed)
    out = {}
    for name, shape in spec:
        if name.endswith(".w"):
            fan_in = shape[1] * shape[2] * shape[3]
            out[name] = normal(rng, shape, 1.0 / math.sqrt(fan_in), sixteen_bit)
        elif name.endswith(".b"):
            out[name] = normal(rng, shape, 0.01)
        elif name.endswith(".gamma"):
            out[name] = (1.0 + normal(rng, shape, 0.2)) if random_affine else np.ones(shape, np.float32)
        elif name.endswith(".beta"):
            out[name] = normal(rng, shape, 0.2) if random_affine else np.zeros(shape, np.float32)
        else:
            raise ValueError(name)
    return out


def decoder_weights(workload=4, **topology):
    return draw_params(decoder_weight_spec(**topology), weight_seed(workload))


def latent_single(workload=4, h=LATENT_H, w=LATENT_W, c=LATENT_C):
    """z[1,c,h,w] ~ N(0,1), 16-bit storage."""
    rng = np.random.default_rng(input_seed(workload))
    return normal(rng, (1, c, h, w), 1.0, True)


def latent_sequence(workload=5, frames=4, h=LATENT_H, w=LATENT_W, c=LATENT_C):
    """z_t = z_0 + t*d + 0.1*eps_t, t = 0..frames-1; draw order z_0, d, eps_0.. ; 16-bit storage.

    Mimics latents produced by first-order extrapolation along a motion vector
    (Alg. 2, Eq. 10): consecutive frames differ by a constant step plus noise."""
    rng = np.random.default_rng(input_seed(workload))
    z0 = rng.standard_normal((c, h, w))
    d = rng.standard_normal((c, h, w))
    z = np.empty((frames, c, h, w), np.float32)
    for t in range(frames):
        z[t] = (z0 + t * d + 0.1 * rng.standard_normal((c, h, w))).astype(np.float32)
    return bf16_round(z)


def adaln_params(seed, d_model, d_cond, sixteen_bit=True):
    """Weights of one AdaLN modulation: 'shift.w', 'scale.w', 'gate.w' ~ N(0, std=1/sqrt(d_cond)) [d_model, d_cond]
    (16-bit storage when asked) and their biases ~ N(0, std=0.01), drawn in that order."""
    rng = np.random.default_rng(seed)
    out = {}
    for name in ("shift", "scale", "gate"):
        out[name + ".w"] = normal(rng, (d_model, d_cond), 1.0 / math.sqrt(d_cond), sixteen_bit)
        out[name + ".b"] = normal(rng, (d_model,), 0.01)
    return out


def activation(workload, shape, sixteen_bit):
    rng = np.random.default_rng(input_seed(workload))
    return normal(rng, shape, 1.0, sixteen_bit)
