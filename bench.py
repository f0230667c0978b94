#!/usr/bin/env python3
"""Benchmark of the decoder hot path on one MI355X.

A step = one decoder_run of the full 720x480 decoder (every GroupNorm statistics
pass, fused norm-SiLU-conv, upsample-conv, 1x1 conv and the mid-block attention)
over one synthetic seeded latent that is already resident in HBM.  Prints one
JSON line: frames/s, the roofline of the dominant kernel measured with HIP
events inside this process, and the fp64 CPU oracle timed on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"mfma": 2516.6, "hbm": 8000.0}   # TFLOP/s dense bf16/f16 MFMA, GB/s HBM3E (published MI355X figures)

# HBM traffic per launch comes from two rocprofv3 counter passes of this same command (counters cannot be collected
# from inside this process); their summary, written by `python -m paper_2602_00608_amd.profile_summary traffic`, is
# read back here and used only if it was taken from the kernel sources this run was built from.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "decoder_full_f16_hbm_traffic.md")


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=1, help="frames per decoder_run (1 = workload 4, 4 = workload 5)")
    ap.add_argument("--dtype", default="f16", choices=["f16", "bf16"],
                    help="storage / MFMA operand type of activations (weights and latents are given in bf16)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-stats", action="store_true",
                    help="ablation: every GroupNorm runs the streaming statistics pass instead of taking the moments from "
                         "the producing convolution's epilogue")
    ap.add_argument("--separate-merge", action="store_true",
                    help="ablation: a small launch merges the moments a convolution emitted, instead of the hand-over "
                         "inside producer and consumer")
    ap.add_argument("--separate-shortcut", action="store_true",
                    help="ablation: the 1x1 shortcuts are launches of their own instead of contraction steps of conv2")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="first copy 256 MiB device to device three times with the library's plain copy kernel: "
                         "launches of known traffic for counter passes")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (frames shard over GPUs with no exchange; "
                 "multi-GPU runs are not part of it); run with --gpus 1")

    import numpy as np
    import torch
    from paper_2602_00608_amd import profile_summary, synth, wmdec

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    if args.calibration_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            wmdec.measure_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst

    cfg = wmdec.decoder_default_config()
    cfg.act_dtype = wmdec.F16 if args.dtype == "f16" else wmdec.BF16
    cfg.max_batch = max(4, args.batch)
    cfg.separate_stats_pass = int(args.separate_stats)
    cfg.separate_shortcut = int(args.separate_shortcut)
    cfg.separate_merge_launch = int(args.separate_merge)
    dec = wmdec.Decoder(cfg)
    weights = synth.decoder_weights(4)
    blob = np.zeros(dec.weights_bytes(), np.uint8)
    for name, off, nb, dt, shape in dec.weight_table():
        a = weights[name]
        raw = synth.bf16_bits(a).tobytes() if dt == wmdec.BF16 else np.ascontiguousarray(a, np.float32).tobytes()
        blob[off:off + nb] = np.frombuffer(raw, np.uint8)
    packed = torch.empty(dec.packed_bytes(), dtype=torch.uint8, device="cuda")
    dec.pack_weights(torch.from_numpy(blob).cuda(), packed)
    ws = torch.empty(dec.workspace_bytes(args.batch), dtype=torch.uint8, device="cuda")
    dec.set_workspace(ws)
    z = synth.latent_single(4) if args.batch == 1 else synth.latent_sequence(5, frames=args.batch)
    zd = torch.from_numpy(synth.bf16_bits(z).view(np.int16)).view(torch.bfloat16).cuda()
    out = torch.empty((args.batch, 3, 480, 720), dtype=torch.float32, device="cuda")

    for _ in range(args.warmup):
        dec.run(zd, packed, out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dec.run(zd, packed, out)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    fps = args.batch * args.steps / elapsed
    assert bool(torch.isfinite(out).all())

    # ---- roofline of the dominant kernel: every graph step again, in plan order, `reps` launches back to back
    # between two HIP events on the stream the kernels run on (each step then sees the tensors of a real run),
    # grouped by the kernel that executes the step
    info = dec.step_info()
    reps = 10
    fam = {}
    per_step = []
    for i, (kernel, flops, nbytes) in enumerate(info):
        ms = dec.time_step(zd, packed, out, i, reps)
        per_step.append({"step": i, "kernel": profile_summary.short_name(kernel), "us": round(ms * 1e3, 2),
                         "gflop": round(flops * args.batch / 1e9, 2), "mb": round(nbytes * args.batch / 1e6, 2),
                         "tflops": round(flops * args.batch / (ms * 1e-3) / 1e12, 1) if ms > 0 else None,
                         "gbps": round(nbytes * args.batch / (ms * 1e-3) / 1e9, 1) if ms > 0 else None})
        f = fam.setdefault(kernel, {"ms": 0.0, "flops": 0.0, "bytes": 0.0, "launches": 0})
        f["ms"] += ms
        f["flops"] += flops * args.batch
        f["bytes"] += nbytes * args.batch
        f["launches"] += 1
    dom = max(fam, key=lambda k: fam[k]["ms"])
    d = fam[dom]
    bound = "mfma" if dom.startswith("conv_mfma") or dom.startswith("flash_attn") else "hbm"
    if bound == "mfma":
        achieved = d["flops"] / (d["ms"] * 1e-3) / 1e12
        unit = "TFLOP/s"
    else:
        achieved = d["bytes"] / (d["ms"] * 1e-3) / 1e9
        unit = "GB/s"
    traffic = traffic_detail = None   # HBM bytes per launch
    digest, table = profile_summary.read_traffic_table(TRAFFIC_SUMMARY)
    short = profile_summary.short_name(dom)
    if args.batch == 1 and args.dtype == "f16" and short in table:
        fetch_mb, write_mb = table[short]
        current = digest == profile_summary.source_digest()
        traffic_detail = {"fetch_mb_per_launch": fetch_mb, "write_mb_per_launch": write_mb,
                          "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes of this command, copy-calibrated "
                                    "(profiles/decoder_full_f16_hbm_traffic.md)",
                          "taken_from_these_kernel_sources": current}
        if current:
            traffic = round((fetch_mb + write_mb) * 1e6)
    roofline = {"kernel": dom, "bound": bound, "achieved": round(achieved, 2), "peak": PEAK[bound], "unit": unit,
                "frac": round(achieved / PEAK[bound], 4), "traffic": traffic, "traffic_detail": traffic_detail,
                "launches_per_step": d["launches"], "avg_launch_us": round(d["ms"] * 1e3 / d["launches"], 2),
                "algorithmic_gflop_per_launch": round(d["flops"] / d["launches"] / 1e9, 3),
                "algorithmic_mb_per_launch": round(d["bytes"] / d["launches"] / 1e6, 3)}
    families = {k: {"ms_per_step": round(v["ms"], 4), "launches": v["launches"],
                    "tflops": round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 1) if v["ms"] > 0 else None,
                    "gbps": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] > 0 else None}
                for k, v in fam.items()}

    # ---- CPU baseline: the fp64 oracle as it stands, one frame of the same workload on the host cores
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ref
        t0 = time.perf_counter()
        want = ref.decoder(z[:1], weights)
        dt = time.perf_counter() - t0
        dec.run(zd, packed, out)
        torch.cuda.synchronize()
        err = ref.rel_err(out[:1].cpu().numpy(), want)
        cpu = {"value": round(1.0 / dt, 5), "unit": "frames/s", "cores": os.cpu_count() if not os.environ.get("OMP_NUM_THREADS")
               else int(os.environ["OMP_NUM_THREADS"]), "cpu_model": cpu_model(), "kind": "oracle",
               "sample": "1 frame of the same workload (full decoder, fp64, %.1f s)" % dt,
               "gpu_vs_oracle_max_abs_err_over_rms": float("%.3e" % err)}

    print(json.dumps({
        "metric": "720x480 frames/s decoded on 1 MI355X", "value": round(fps, 2), "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "%s MFMA operands and activations, bf16 weights/latents as given, fp32 accumulate" % args.dtype,
        "data": "synthetic",
        "config": {"workload": "configs[3]: full decoder, latent z[%d,4,60,90] -> frame [%d,3,480,720], batch %d"
                   % (args.batch, args.batch, args.batch), "frames_per_step": args.batch,
                   "gflop_per_frame": round(dec.flops_per_frame() / 1e9, 1),
                   "gflop_per_frame_if_upsampling_convs_ran_nine_taps": round(dec.dense_flops_per_frame() / 1e9, 1),
                   "launches_per_step": dec.num_launches(),
                   "graph": {"statistics": "separate pass" if args.separate_stats else ("from the producer's epilogue, merged by a launch"
                                            if args.separate_merge else "from the producer's epilogue, no merge launch"),
                             "shortcut": "separate launch" if args.separate_shortcut else "folded into conv2"}},
        "tflops": round(dec.flops_per_frame() * fps / 1e12, 1),
        "roofline": roofline, "cpu_baseline": cpu, "kernel_families": families, "graph_steps": per_step}))


if __name__ == "__main__":
    main()
