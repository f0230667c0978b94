"""Per-operator timing of the C-ABI entry points at the decoder's layer shapes (one MI355X).

    python -m paper_2602_00608_amd.bench_ops [--dtype f16|bf16] [--reps 20]      (or run the file directly)

Prints one line per operator: microseconds per call, algorithmic TFLOP/s or GB/s, and the fraction of the
published MI355X peak (2516.6 TFLOP/s dense f16/bf16 MFMA, 8000 GB/s HBM).  Two timings per operator, both with HIP
events on the current stream and inputs resident in HBM:
  warm  `reps` back-to-back calls on the same tensors (tensors up to a few hundred MB partly stay in the last-level
        cache between calls);
  cold  between two calls a 2 GiB buffer is streamed (read and written), which evicts every cache level; the time
        of the streaming kernel alone, measured the same way, is subtracted.
An upsampling convolution that is evaluated per output phase is priced at the 2x2 taps it executes (4/9 of the
nine-tap figure).  Inputs are seeded N(0,1) tensors and 1/sqrt(fan_in) weights; real activations toggle fewer bits,
so inside decoder_run the same convolutions run somewhat faster.
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


def _events(fn, reps):
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(reps):
        fn()
    t1.record()
    torch.cuda.synchronize()
    return t0.elapsed_time(t1) / reps * 1e3   # microseconds


def timeit(fn, reps):
    """(warm, cold) microseconds per call."""
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    warm = _events(fn, reps)
    creps = max(3, reps // 4)
    flush = timeit.flush

    def evict():
        flush.add_(1)          # reads and writes 2 GiB: nothing of the operator's tensors survives in any cache

    def cold_call():
        evict()
        fn()
    evict()
    torch.cuda.synchronize()
    base = _events(evict, creps)
    cold = _events(cold_call, creps) - base
    return warm, cold


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--reps", type=int, default=20)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_ops: no GPU visible; the HIP path has no CPU fallback")
    torch.manual_seed(260200608)
    timeit.flush = torch.zeros(2 << 30, dtype=torch.uint8, device="cuda")
    dt, en = TORCH[args.dtype], ENUM[args.dtype]
    groups, eps = 32, 1e-6

    def stats_of(x):
        n, h, w, c = x.shape
        ws = torch.zeros(wmdec.gn_stats_workspace_bytes(n, h, w, c, groups), dtype=torch.uint8, device="cuda")
        mean = torch.empty(n * groups, dtype=torch.float32, device="cuda")
        rstd = torch.empty(n * groups, dtype=torch.float32, device="cuda")
        wmdec.gn_stats(x, groups, eps, mean, rstd, ws)
        return mean, rstd, ws

    def line(name, shape, us, work, unit, peak):
        warm, cold = us
        print("%-30s %-22s warm %8.1f us %8.1f %s (%4.1f%%)   cold %8.1f us %8.1f %s (%4.1f%% of %.0f)"
              % (name, shape, warm, work / warm / 1e6 if unit == "TFLOP/s" else work / warm / 1e3, unit,
                 (work / warm / 1e6 if unit == "TFLOP/s" else work / warm / 1e3) / peak * 100,
                 cold, work / cold / 1e6 if unit == "TFLOP/s" else work / cold / 1e3, unit,
                 (work / cold / 1e6 if unit == "TFLOP/s" else work / cold / 1e3) / peak * 100, peak), flush=True)

    # cin, cout, h_out, w_out, kernel, upsample, normalise + SiLU on load, residual
    convs = [(128, 128, 480, 720, 3, 0, 1, 1), (256, 128, 480, 720, 3, 0, 1, 0), (256, 256, 240, 360, 3, 0, 1, 1),
             (512, 256, 240, 360, 3, 0, 1, 0), (512, 512, 120, 180, 3, 0, 1, 1), (512, 512, 60, 90, 3, 0, 1, 1),
             (256, 256, 480, 720, 3, 1, 0, 0), (512, 512, 240, 360, 3, 1, 0, 0), (512, 512, 120, 180, 3, 1, 0, 0),
             (256, 128, 480, 720, 1, 0, 0, 0), (512, 256, 240, 360, 1, 0, 0, 0), (512, 1536, 60, 90, 1, 0, 1, 0),
             ]
    for cin, cout, h, w, k, ups, norm, use_res in convs:
        hi, wi = (h // 2, w // 2) if ups else (h, w)
        out_dt = dt
        x = torch.randn((1, hi, wi, cin), device="cuda").to(dt)
        y = torch.empty((1, h, w, cout), device="cuda", dtype=out_dt)
        res = torch.randn((1, h, w, cout), device="cuda").to(dt) if use_res else None
        wsrc = torch.randn((cout, cin, k, k), device="cuda") / (cin * k * k) ** 0.5
        bias = 0.01 * torch.randn(cout, device="cuda")
        gamma, beta = torch.ones(cin, device="cuda"), torch.zeros(cin, device="cuda")
        flops = 2.0 * k * k * cin * cout * h * w
        nbytes = x.numel() * 2 + y.numel() * y.element_size() + (res.numel() * 2 if use_res else 0) + wsrc.numel() * 2
        if ups:
            wp = torch.empty(wmdec.upconv_packed_bytes(cout, cin, en), dtype=torch.uint8, device="cuda")
            wmdec.pack_upconv_weights(wsrc, wp, en)
            us = timeit(lambda: wmdec.upsample2x_conv3x3(x, wp, bias, y), args.reps)
            name = "upsample2x_conv3x3"
            if args.dtype == "f16" and cout % 64 == 0:
                flops *= 4.0 / 9.0        # evaluated per output phase: 2x2 taps executed
        else:
            wp = torch.empty(wmdec.conv_packed_bytes(cout, cin, k, en), dtype=torch.uint8, device="cuda")
            wmdec.pack_conv_weights(wsrc, wp, en)
            mean, rstd, _ = stats_of(x)
            fn = wmdec.gn_silu_conv3x3 if k == 3 else wmdec.gn_conv1x1
            if norm:
                us = timeit(lambda: fn(x, mean, rstd, gamma, beta, groups, True, wp, bias, res, y), args.reps)
            else:
                us = timeit(lambda: fn(x, None, None, None, None, groups, False, wp, bias, res, y), args.reps)
            name = "gn_silu_conv3x3" if k == 3 else "gn_conv1x1"
        shape = "%4d->%4d @%3dx%3d" % (cin, cout, h, w)
        if flops / nbytes >= 315:            # above the ridge point: priced against the matrix cores
            line(name, shape, us, flops, "TFLOP/s", PEAK_TFLOPS)
        else:
            line(name, shape, us, nbytes, "GB/s", PEAK_GBPS)

    for c, h, w in [(128, 480, 720), (256, 480, 720), (256, 240, 360), (512, 120, 180), (512, 60, 90)]:
        x = torch.randn((1, h, w, c), device="cuda").to(dt)
        mean, rstd, ws = stats_of(x)
        us = timeit(lambda: wmdec.gn_stats(x, groups, eps, mean, rstd, ws), args.reps)
        line("gn_stats", "%4d       @%3dx%3d" % (c, h, w), us, x.numel() * 2, "GB/s", PEAK_GBPS)

    x = torch.randn((1, 120, 180, 256), device="cuda").to(dt)
    y = torch.empty((1, 240, 360, 256), device="cuda", dtype=dt)
    us = timeit(lambda: wmdec.upsample2x_nearest(x, y), args.reps)
    line("upsample2x_nearest", "%4d       @%3dx%3d" % (256, 240, 360), us, (x.numel() + y.numel()) * 2, "GB/s", PEAK_GBPS)


    # mid-block attention as one call (qkv projection, V transpose, attention core + combine, output projection with
    # the residual): 5400 tokens, one head of 512
    c, h, w = 512, 60, 90
    x = torch.randn((1, h, w, c), device="cuda").to(dt)
    y = torch.empty_like(x)
    mean, rstd, _ = stats_of(x)
    gamma, beta = torch.ones(c, device="cuda"), torch.zeros(c, device="cuda")
    wq = torch.randn((3 * c, c, 1, 1), device="cuda") / c ** 0.5
    wo = torch.randn((c, c, 1, 1), device="cuda") / c ** 0.5
    bq, bo = 0.01 * torch.randn(3 * c, device="cuda"), 0.01 * torch.randn(c, device="cuda")
    wqp = torch.empty(wmdec.conv_packed_bytes(3 * c, c, 1, en), dtype=torch.uint8, device="cuda")
    wop = torch.empty(wmdec.conv_packed_bytes(c, c, 1, en), dtype=torch.uint8, device="cuda")
    wmdec.pack_conv_weights(wq, wqp, en)
    wmdec.pack_conv_weights(wo, wop, en)
    aws = torch.empty(wmdec.attention_workspace_bytes(1, h, w, c), dtype=torch.uint8, device="cuda")
    us = timeit(lambda: wmdec.attention(x, mean, rstd, gamma, beta, groups, wqp, bq, wop, bo, y, aws), args.reps)
    t = h * w
    line("attention block (5 launches)", "%4d       @%3dx%3d" % (c, h, w), us, 4.0 * t * t * c + 2.0 * t * c * 4 * c, "TFLOP/s", PEAK_TFLOPS)

    # how much of the matrix-core rate is a matter of operand values: the same plain 3x3 convolution (no normalisation,
    # no residual: identical instruction stream and memory traffic) on N(0,1) activations and on zeros
    for cin, cout, h, w in [(256, 256, 240, 360), (512, 512, 120, 180)]:
        y = torch.empty((1, h, w, cout), device="cuda", dtype=dt)
        wsrc = torch.randn((cout, cin, 3, 3), device="cuda") / (cin * 9) ** 0.5
        bias = 0.01 * torch.randn(cout, device="cuda")
        wp = torch.empty(wmdec.conv_packed_bytes(cout, cin, 3, en), dtype=torch.uint8, device="cuda")
        wmdec.pack_conv_weights(wsrc, wp, en)
        flops = 2.0 * 9 * cin * cout * h * w
        for label, x in (("N(0,1) input", torch.randn((1, h, w, cin), device="cuda").to(dt)),
                         ("all-zero input", torch.zeros((1, h, w, cin), device="cuda", dtype=dt))):
            us = timeit(lambda: wmdec.gn_silu_conv3x3(x, None, None, None, None, groups, False, wp, bias, None, y), args.reps)
            line("plain conv3x3, " + label, "%4d->%4d @%3dx%3d" % (cin, cout, h, w), us, flops, "TFLOP/s", PEAK_TFLOPS)

    # horizontally fused AdaLN projections: one launch on [W_shift; W_scale; W_gate] against three launches
    d = 1920
    for batch in (1, 4):
        c = torch.randn((batch, d), device="cuda")
        wf = (torch.randn((3 * d, d), device="cuda") / d ** 0.5).to(torch.bfloat16)
        bf = 0.01 * torch.randn(3 * d, device="cuda")
        out = torch.empty((batch, 3 * d), device="cuda")
        parts = [wf[i * d:(i + 1) * d].contiguous() for i in range(3)]
        outs = [torch.empty((batch, d), device="cuda") for _ in range(3)]
        fused = timeit(lambda: wmdec.adaln_fused_projection(c, wf, bf, out), args.reps)

        def three():
            for i in range(3):
                wmdec.adaln_fused_projection(c, parts[i], bf[i * d:(i + 1) * d], outs[i])
        sep = timeit(three, args.reps)
        nbytes = wf.numel() * 2
        line("adaln fused (1 launch)", "batch %d %d->3x%d" % (batch, d, d), fused, nbytes, "GB/s", PEAK_GBPS)
        line("adaln 3 launches", "batch %d %d->3x%d" % (batch, d, d), sep, nbytes, "GB/s", PEAK_GBPS)


if __name__ == "__main__":
    main()
