"""Builds libdos.so (HIP kernels + C-ABI) and libdos_probe.so (the benchmark's measurement aids)
in-tree for gfx950 with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
PROBE_SRC = os.path.join(HERE, "probe")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdos.so")
PROBE_LIB = os.path.join(HERE, "libdos_probe.so")

# -ffp-contract=off, correctly rounded divide/sqrt and kept denormals make every
# source-level float operation one IEEE binary32 operation on device and host.
# Packed FP32 instructions are switched off for the device pass.
# -fno-math-errno changes no arithmetic: it lets sqrtf become the (correctly rounded)
# square-root instruction without a libm call for errno, which is what allows the host
# update loop to be vectorised at all.
COMMON = ["-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math", "-fno-math-errno", "-pthread",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", PROBE_SRC, "-Wall", "-Wno-unused-function"]
DEVICE = ["--offload-arch=gfx950", "-fhip-fp32-correctly-rounded-divide-sqrt",
          "-fno-gpu-flush-denormals-to-zero", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))


def probe_sources():
    return sorted(glob.glob(os.path.join(PROBE_SRC, "*.hip")) + glob.glob(os.path.join(PROBE_SRC, "*.cpp")))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    if src.endswith(".hip"):
        cmd = [_hipcc(), *COMMON, *DEVICE, "-c", src, "-o", obj]
    else:
        cmd = [_hipcc(), *COMMON, "-x", "hip", "--offload-host-only", "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("compile failed: " + " ".join(cmd))
    return obj


def _link(objs, lib: str) -> None:
    tmp = lib + ".tmp.%d" % os.getpid()
    cmd = [_hipcc(), "-shared", "-fPIC", "-pthread", "-o", tmp, *objs, "-Wl,--no-undefined"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed: " + " ".join(cmd))
    os.replace(tmp, lib)


def build_library(verbose: bool = False) -> str:
    """Compile every source under csrc/ and probe/ and link libdos.so and
    libdos_probe.so.  Always compiles."""
    os.makedirs(OBJ, exist_ok=True)
    srcs, psrcs = sources(), probe_sources()
    with ThreadPoolExecutor(max_workers=min(8, len(srcs) + len(psrcs))) as ex:
        objs = list(ex.map(_compile, srcs + psrcs))
    _link(objs[:len(srcs)], LIB)
    _link(objs[len(srcs):], PROBE_LIB)
    if verbose:
        print("built", LIB, "and", PROBE_LIB)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
