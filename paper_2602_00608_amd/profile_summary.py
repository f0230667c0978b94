"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under profiles/.

    python -m paper_2602_00608_amd.profile_summary trace   <dir with *_kernel_stats.csv>  <out.md>  "<command>"
    python -m paper_2602_00608_amd.profile_summary traffic <FETCH_SIZE dir> <WRITE_SIZE dir> <out.md>
    python -m paper_2602_00608_amd.profile_summary counters <out.md> <dir> [<dir> ...]

`traffic` expects the two counter passes of `bench.py --calibration-copy` (three 256 MiB device-to-device copies of
known size run first; what the counters read for them gives the scale of each counter) and writes the table that
`bench.py` reads back for `roofline.traffic`.  Every summary records a digest of the kernel sources it was taken
from, so that a reader (and `bench.py`) can tell whether it still describes the library as built.
"""
import collections
import csv
import glob
import hashlib
import os
import re
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CALIBRATION_KERNEL = "copy_u128_kernel"
CALIBRATION_KIB = 256 * 1024          # one calibration copy reads and writes 256 MiB


def source_digest():
    """sha256 over the library's sources (csrc/*.hip, *.hpp, *.cpp) in name order, first 16 hex digits."""
    h = hashlib.sha256()
    csrc = os.path.join(HERE, "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".hpp", ".cpp")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def short_name(kernel):
    """`void wmdec::(anonymous namespace)::foo<wmdec::f16_t, ...>(args)` -> `foo<f16_t, ...>`."""
    k = re.sub(r"^void\s+", "", kernel)
    depth, cut = 0, len(k)
    for i, ch in enumerate(k):          # drop the argument list: the first '(' outside template brackets that is not
        if ch == "<":                   # part of "(anonymous namespace)"
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0 and not k.startswith("(anonymous namespace)", i):
            cut = i
            break
    k = k[:cut]
    return k.replace("wmdec::(anonymous namespace)::", "").replace("wmdec::", "")


def _one(pattern):
    files = sorted(glob.glob(pattern, recursive=True))
    if not files:
        raise SystemExit("no file matches %s" % pattern)
    return files[0]


def read_counters(directory):
    """{kernel: {counter: [value per dispatch]}} from a rocprofv3 --pmc run."""
    out = collections.defaultdict(lambda: collections.defaultdict(list))
    with open(_one(os.path.join(directory, "**", "*counter_collection.csv"))) as f:
        for r in csv.DictReader(f):
            out[short_name(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return out


def mean(v):
    return sum(v) / len(v) if v else 0.0


def cmd_trace(directory, out_md, command):
    rows = list(csv.DictReader(open(_one(os.path.join(directory, "**", "*kernel_stats.csv")))))
    with open(out_md, "w") as f:
        f.write("# Kernel trace of the benchmark run\n\nCommand (run from /tmp with TMPDIR=/tmp):\n\n    %s\n\n" % command)
        f.write("Source digest of the library: `%s`.  Durations in microseconds, from `*_kernel_stats.csv`.\n\n" % source_digest())
        f.write("| kernel | calls | total us | average us | % of GPU time | min us | max us |\n|---|---:|---:|---:|---:|---:|---:|\n")
        for r in rows:
            f.write("| `%s` | %s | %.0f | %.1f | %s | %.1f | %.1f |\n" % (
                short_name(r["Name"]), r["Calls"], float(r["TotalDurationNs"]) / 1e3, float(r["AverageNs"]) / 1e3,
                r["Percentage"], float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3))


def cmd_traffic(fetch_dir, write_dir, out_md):
    fetch, write = read_counters(fetch_dir), read_counters(write_dir)
    cal_f = mean(fetch[CALIBRATION_KERNEL]["FETCH_SIZE"])
    cal_w = mean(write[CALIBRATION_KERNEL]["WRITE_SIZE"])
    if cal_f <= 0 or cal_w <= 0:
        raise SystemExit("no calibration copies in the counter passes (run bench.py with --calibration-copy)")
    sf, sw = CALIBRATION_KIB / cal_f, CALIBRATION_KIB / cal_w
    with open(out_md, "w") as f:
        f.write("# HBM traffic per launch, full decoder (f16, batch 1, latent 4x60x90 -> frame 3x480x720)\n\n"
                "Two counter passes of the same command, one counter each (run from /tmp with TMPDIR=/tmp):\n\n"
                "    rocprofv3 --pmc FETCH_SIZE -d <out> -o r --output-format csv -- python3 /root/repo/bench.py --steps 3 --warmup 1 --no-cpu-baseline --calibration-copy\n"
                "    rocprofv3 --pmc WRITE_SIZE -d <out> -o r --output-format csv -- python3 /root/repo/bench.py --steps 3 --warmup 1 --no-cpu-baseline --calibration-copy\n\n"
                "summarised by `python -m paper_2602_00608_amd.profile_summary traffic <fetch dir> <write dir> <this file>`.\n\n")
        f.write("Calibration: the three 256 MiB device-to-device copies (`%s`) read FETCH_SIZE = %.1f KiB and WRITE_SIZE = "
                "%.1f KiB per copy against 262144 KiB read and written: scale factors %.3f (fetch) and %.3f (write).\n"
                "Figures are scaled, mean per dispatch over all dispatches of the kernel in the run (MB = 1e6 bytes).\n\n"
                % (CALIBRATION_KERNEL, cal_f, cal_w, sf, sw))
        f.write("source digest: %s\n\n" % source_digest())
        f.write("| kernel | dispatches | fetch MB | write MB |\n|---|---:|---:|---:|\n")
        names = sorted(fetch, key=lambda k: -sum(fetch[k]["FETCH_SIZE"]))
        for k in names:
            if k == CALIBRATION_KERNEL or "at::native" in k:
                continue
            fv, wv = fetch[k]["FETCH_SIZE"], write.get(k, {}).get("WRITE_SIZE", [])
            f.write("| `%s` | %d | %.1f | %.1f |\n" % (k, len(fv), mean(fv) * sf * 1024 / 1e6, mean(wv) * sw * 1024 / 1e6))


def read_traffic_table(path):
    """(digest, {kernel: (fetch MB, write MB)}) from a summary written by cmd_traffic; (None, {}) if absent."""
    if not os.path.exists(path):
        return None, {}
    digest, table = None, {}
    for line in open(path):
        m = re.match(r"source digest: ([0-9a-f]+)", line)
        if m:
            digest = m.group(1)
        m = re.match(r"\| `(.+)` \| (\d+) \| ([0-9.]+) \| ([0-9.]+) \|", line)
        if m:
            table[m.group(1)] = (float(m.group(3)), float(m.group(4)))
    return digest, table


def cmd_counters(out_md, dirs):
    merged = collections.defaultdict(dict)
    names = []
    for d in dirs:
        for k, cs in read_counters(d).items():
            for c, v in cs.items():
                merged[k][c] = (mean(v), len(v))
                if c not in names:
                    names.append(c)
    with open(out_md, "w") as f:
        f.write("# Hardware counters per kernel, full decoder benchmark (f16, batch 1)\n\n"
                "One `rocprofv3 --pmc <counters> -d <out> -o r --output-format csv -- python3 /root/repo/bench.py --steps 3 "
                "--warmup 1 --no-cpu-baseline` run per counter group (run from /tmp with TMPDIR=/tmp), summarised by\n"
                "`python -m paper_2602_00608_amd.profile_summary counters <this file> <dirs>`.  Mean per dispatch.\n\n")
        f.write("source digest: %s\n\n" % source_digest())
        f.write("| kernel | dispatches | " + " | ".join(names) + " |\n|---|---:|" + "---:|" * len(names) + "\n")
        order = sorted(merged, key=lambda k: -merged[k].get(names[0], (0, 0))[0] * merged[k].get(names[0], (0, 0))[1])
        for k in order:
            if "at::native" in k or k == CALIBRATION_KERNEL:
                continue
            n = max(v[1] for v in merged[k].values())
            f.write("| `%s` | %d | " % (k, n) + " | ".join("%.4g" % merged[k][c][0] if c in merged[k] else "" for c in names) + " |\n")


def main(argv):
    if len(argv) >= 5 and argv[1] == "trace":
        cmd_trace(argv[2], argv[3], argv[4])
    elif len(argv) == 5 and argv[1] == "traffic":
        cmd_traffic(argv[2], argv[3], argv[4])
    elif len(argv) >= 4 and argv[1] == "counters":
        cmd_counters(argv[2], argv[3:])
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv)
