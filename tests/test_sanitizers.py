"""AddressSanitizer / UndefinedBehaviorSanitizer builds of the CPU-side code (no GPU): the C oracle on small odd-sized
inputs in exact-size heap buffers, and the library's host logic (plan building, weight table, workspace layout, step
accounting, argument checks) driven without launching a kernel.  Device code is not instrumented."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2602_00608_amd")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-3000:], r.stderr[-3000:])
    return r.stdout + r.stderr


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize_check")
    run(["gcc", "-O1", "-g", "-std=c99", "-fopenmp"] + SAN + ["-static-libasan", "-o", exe,
         os.path.join(ROOT, "oracle", "sanitize_check.c"), "-lm"])
    out = run([exe], env=dict(os.environ, OMP_NUM_THREADS="4"))
    assert "sanitize_check: ok" in out and "runtime error" not in out, out


def test_host_logic_under_address_and_undefined_sanitizers(tmp_path):
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not on PATH")
    objs = [o for o in sorted(glob.glob(os.path.join(PKG, "_build", "kernels_*.o")))]
    if len(objs) < 7:
        pytest.skip("kernel objects not built (run __graft_entry__.build())")
    inc = ["-I" + os.path.join(PKG, "csrc"), "-I" + os.path.join(ROOT, "include")]
    api = str(tmp_path / "api_san.o")
    host = []
    for f in SAN:
        host += ["-Xarch_host", f]
    run(["hipcc", "-x", "hip", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + host + inc +
        ["-c", os.path.join(PKG, "csrc", "api.cpp"), "-o", api])
    drv = str(tmp_path / "drv.o")
    run(["hipcc", "-O1", "-g", "-std=c++17"] + SAN + inc + ["-c", os.path.join(ROOT, "tests", "host_sanitize_check.cpp"), "-o", drv])
    exe = str(tmp_path / "host_sanitize_check")
    run(["hipcc", "--offload-arch=gfx950"] + SAN + ["-o", exe, drv, api] + objs)
    out = run([exe])
    assert "host_sanitize_check: ok" in out and "runtime error" not in out, out
