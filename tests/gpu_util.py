"""Helpers shared by the GPU parity tests: host <-> device marshalling in the
library's NHWC layout and wrappers that run one op through the C ABI."""
import numpy as np
import torch

from paper_2602_00608_amd import wmdec

TORCH = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
ENUM = {"f32": wmdec.F32, "bf16": wmdec.BF16, "f16": wmdec.F16}
TOL = {"f32": 1e-4, "bf16": 2e-2, "f16": 2e-2}   # max|err| / rms(oracle), the workload's stated bar


def dev_nhwc(x_nchw, dtype):
    """numpy [N,C,H,W] float32 -> device tensor [N,H,W,C] of `dtype` (values must be representable)."""
    t = torch.from_numpy(np.ascontiguousarray(np.transpose(x_nchw, (0, 2, 3, 1)))).to(TORCH[dtype])
    return t.cuda()


def host_nchw(t_nhwc):
    """device [N,H,W,C] -> numpy float64 [N,C,H,W]."""
    return t_nhwc.detach().to(torch.float64).cpu().numpy().transpose(0, 3, 1, 2)


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def stored(x, dtype):
    """The float32 values a tensor holds once stored as `dtype` (what the oracle must consume)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(TORCH[dtype]).to(torch.float32).numpy()


def pack(w_oihw, dtype):
    """Pack logical [cout,cin,k,k] float32 weights for operand type `dtype` through the ABI."""
    cout, cin, k, _ = w_oihw.shape
    src = torch.from_numpy(np.ascontiguousarray(w_oihw, dtype=np.float32)).cuda()
    nbytes = wmdec.conv_packed_bytes(cout, cin, k, ENUM[dtype])
    assert nbytes > 0
    packed = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    wmdec.pack_conv_weights(src, packed, ENUM[dtype])
    return packed


def pack_upconv(w_oihw, dtype):
    """Pack [cout,cin,3,3] float32 weights of an upsampling convolution (9-tap pack + phase pack) through the ABI."""
    cout, cin, _, _ = w_oihw.shape
    src = torch.from_numpy(np.ascontiguousarray(w_oihw, dtype=np.float32)).cuda()
    nbytes = wmdec.upconv_packed_bytes(cout, cin, ENUM[dtype])
    assert nbytes > 0
    packed = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    wmdec.pack_upconv_weights(src, packed, ENUM[dtype])
    return packed


def gn_stats(x_dev, groups, eps):
    n, h, w, c = x_dev.shape
    ws = torch.zeros(max(wmdec.gn_stats_workspace_bytes(n, h, w, c, groups), 256), dtype=torch.uint8, device="cuda")   # ticket counter starts at zero
    mean = torch.empty(n * groups, dtype=torch.float32, device="cuda")
    rstd = torch.empty(n * groups, dtype=torch.float32, device="cuda")
    wmdec.gn_stats(x_dev, groups, eps, mean, rstd, ws)
    return mean, rstd


def canaried(shape, dtype):
    """Output tensor inside a larger allocation filled with a sentinel; returns (view, check)."""
    numel = int(np.prod(shape))
    pad = 256
    big = torch.full((numel + 2 * pad,), 12345.0, dtype=dtype, device="cuda")
    view = big[pad:pad + numel].view(*shape)

    def check():
        assert bool((big[:pad] == 12345.0).all()) and bool((big[pad + numel:] == 12345.0).all()), "out-of-bounds write"
    return view, check
