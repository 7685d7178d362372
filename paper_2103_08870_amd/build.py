"""Builds liblgc.so (HIP, gfx950) in-tree next to this file.  Also builds, when it can, the stand-alone
measurement program hbm_rates beside bench.py at the repository root (streaming rates of plain kernels, for
comparison; bench.py runs it when it is there); the library does not depend on it."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblgc.so")
ROOT = os.path.dirname(HERE)
HBM_RATES = os.path.join(ROOT, "hbm_rates")
SOURCES = ["api.hip", "streaming.hip", "topk.hip", "segmented.hip", "autoencoder.hip", "ae_mfma.hip"]
HEADERS = [os.path.join(CSRC, "lgc_internal.h"), os.path.join(CSRC, "device_helpers.h"),
           os.path.join(os.path.dirname(HERE), "include", "lgc.h")]

FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-ffp-contract=off",
         "-fno-gpu-flush-denormals-to-zero",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-variable", "-Wno-unknown-attributes"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link liblgc.so.  With force=False nothing is
    done when the library is newer than all sources."""
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(p) for p in srcs + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        cmd = [hipcc] + FLAGS + ["-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if verbose or r.returncode != 0:
            sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}")
        return obj

    def build_probe():
        src = os.path.join(ROOT, "hbm_rates.hip")
        if not os.path.exists(src):
            return
        cmd = [hipcc] + [f for f in FLAGS if f != "-fPIC"] + [src, "-o", HBM_RATES]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if verbose or r.returncode != 0:
            sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        if r.returncode != 0:   # the measurement program is optional: the library build goes on without it
            sys.stderr.write("warning: hbm_rates.hip did not build; bench.py will leave out the plain-kernel rates\n")

    with ThreadPoolExecutor(max_workers=len(srcs) + 1) as ex:
        probe = ex.submit(build_probe)
        objs = list(ex.map(compile_one, srcs))
        probe.result()
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("linking liblgc.so failed")
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
