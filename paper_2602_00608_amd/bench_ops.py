"""Per-operator timing of the C-ABI entry points at the decoder's layer shapes (one MI355X).

    python -m paper_2602_00608_amd.bench_ops [--dtype f16|bf16] [--reps 20]      (or run the file directly)

Prints one line per operator: microseconds per call (HIP events around `reps` back-to-back calls on the current
stream, inputs resident in HBM), algorithmic TFLOP/s or GB/s, and the fraction of the published MI355X peak
(2516.6 TFLOP/s dense f16/bf16 MFMA, 8000 GB/s HBM).  Inputs are seeded N(0,1) tensors and 1/sqrt(fan_in)
weights; real activations toggle fewer bits, so inside decoder_run the same convolutions run somewhat faster.
"""
import argparse
import os
import sys

import torch

if __package__ in (None, ""):   # run as a file (e.g. under a profiler): make the package importable
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    from paper_2602_00608_amd import wmdec
else:
    from . import wmdec

PEAK_TFLOPS, PEAK_GBPS = 2516.6, 8000.0
TORCH = {"f16": torch.float16, "bf16": torch.bfloat16}
ENUM = {"f16": wmdec.F16, "bf16": wmdec.BF16}


def timeit(fn, reps):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(reps):
        fn()
    t1.record()
    torch.cuda.synchronize()
    return t0.elapsed_time(t1) / reps * 1e3   # microseconds


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--reps", type=int, default=20)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_ops: no GPU visible; the HIP path has no CPU fallback")
    torch.manual_seed(260200608)
    dt, en = TORCH[args.dtype], ENUM[args.dtype]
    groups, eps = 32, 1e-6

    def stats_of(x):
        n, h, w, c = x.shape
        ws = torch.zeros(wmdec.gn_stats_workspace_bytes(n, h, w, c, groups), dtype=torch.uint8, device="cuda")
        mean = torch.empty(n * groups, dtype=torch.float32, device="cuda")
        rstd = torch.empty(n * groups, dtype=torch.float32, device="cuda")
        wmdec.gn_stats(x, groups, eps, mean, rstd, ws)
        return mean, rstd, ws

    # cin, cout, h_out, w_out, kernel, upsample
    convs = [(128, 128, 480, 720, 3, 0), (256, 128, 480, 720, 3, 0), (256, 256, 240, 360, 3, 0), (512, 256, 240, 360, 3, 0),
             (512, 512, 120, 180, 3, 0), (512, 512, 60, 90, 3, 0), (256, 256, 480, 720, 3, 1), (512, 512, 240, 360, 3, 1),
             (512, 512, 120, 180, 3, 1), (256, 128, 480, 720, 1, 0), (512, 256, 240, 360, 1, 0), (512, 1536, 60, 90, 1, 0)]
    for cin, cout, h, w, k, ups in convs:
        hi, wi = (h // 2, w // 2) if ups else (h, w)
        x = torch.randn((1, hi, wi, cin), device="cuda").to(dt)
        y = torch.empty((1, h, w, cout), device="cuda", dtype=dt)
        res = torch.randn((1, h, w, cout), device="cuda").to(dt)
        wsrc = torch.randn((cout, cin, k, k), device="cuda") / (cin * k * k) ** 0.5
        bias = 0.01 * torch.randn(cout, device="cuda")
        gamma, beta = torch.ones(cin, device="cuda"), torch.zeros(cin, device="cuda")
        if ups:
            wp = torch.empty(wmdec.upconv_packed_bytes(cout, cin, en), dtype=torch.uint8, device="cuda")
            wmdec.pack_upconv_weights(wsrc, wp, en)
            us = timeit(lambda: wmdec.upsample2x_conv3x3(x, wp, bias, y), args.reps)
            name = "upsample2x_conv3x3"
        else:
            wp = torch.empty(wmdec.conv_packed_bytes(cout, cin, k, en), dtype=torch.uint8, device="cuda")
            wmdec.pack_conv_weights(wsrc, wp, en)
            mean, rstd, _ = stats_of(x)
            fn = wmdec.gn_silu_conv3x3 if k == 3 else wmdec.gn_conv1x1
            us = timeit(lambda: fn(x, mean, rstd, gamma, beta, groups, True, wp, bias, res, y), args.reps)
            name = "gn_silu_conv3x3" if k == 3 else "gn_conv1x1"
        flops = 2.0 * k * k * cin * cout * h * w
        print("%-20s %4d->%4d @%3dx%3d: %8.1f us  %7.1f TFLOP/s  (%4.1f%% of %.1f)"
              % (name, cin, cout, h, w, us, flops / us / 1e6, flops / us / 1e6 / PEAK_TFLOPS * 100, PEAK_TFLOPS), flush=True)

    for c, h, w in [(128, 480, 720), (256, 480, 720), (256, 240, 360), (512, 120, 180), (512, 60, 90)]:
        x = torch.randn((1, h, w, c), device="cuda").to(dt)
        mean, rstd, ws = stats_of(x)
        us = timeit(lambda: wmdec.gn_stats(x, groups, eps, mean, rstd, ws), args.reps)
        nbytes = x.numel() * 2
        print("%-20s %4d       @%3dx%3d: %8.1f us  %7.1f GB/s    (%4.1f%% of %.0f)"
              % ("gn_stats", c, h, w, us, nbytes / us / 1e3, nbytes / us / 1e3 / PEAK_GBPS * 100, PEAK_GBPS), flush=True)

    x = torch.randn((1, 120, 180, 256), device="cuda").to(dt)
    y = torch.empty((1, 240, 360, 256), device="cuda", dtype=dt)
    us = timeit(lambda: wmdec.upsample2x_nearest(x, y), args.reps)
    nbytes = (x.numel() + y.numel()) * 2
    print("%-20s %4d       @%3dx%3d: %8.1f us  %7.1f GB/s    (%4.1f%% of %.0f)"
          % ("upsample2x_nearest", 256, 240, 360, us, nbytes / us / 1e3, nbytes / us / 1e3 / PEAK_GBPS * 100, PEAK_GBPS), flush=True)


if __name__ == "__main__":
    main()
