"""Build libzc.so (HIP, gfx950) in-tree with hipcc.

``python -m paper_2504_09983_amd.build`` compiles every ``csrc/*.hip`` to an
object under ``_build/`` (git-ignored) and links ``paper_2504_09983_amd/libzc.so``, then builds
the stand-alone measurement program ``state_layout_probe`` from ``csrc/probe/``.
hipcc cross-compiles, so no GPU is needed to build.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
BUILD_DIR = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libzc.so")
PROBE_SRC = os.path.join(CSRC, "probe", "state_layout_probe.hip")
PROBE = os.path.join(PKG, "state_layout_probe")      # stand-alone measurement program (tune.py runs it)

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ARCH = "gfx950"

# Packed-fp32 VALU forms are switched off for every device TU.
DEVICE_FLAGS = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
COMMON = ["-O3", "-std=c++17", "-fPIC", f"--offload-arch={ARCH}", "-I", INCLUDE, "-I", CSRC,
          "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _compile(src: str) -> str:
    obj = os.path.join(BUILD_DIR, os.path.basename(src) + ".o")
    cmd = [HIPCC, *COMMON, *DEVICE_FLAGS, "-c", src, "-o", obj]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs: int = 8, verbose: bool = True) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    srcs = sources()
    if not srcs:
        raise RuntimeError("no HIP sources found")
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(srcs)))) as pool:
        objs = list(pool.map(_compile, srcs))
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [HIPCC, "-shared", "-fPIC", f"--offload-arch={ARCH}", *objs, "-o", tmp]
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    tmp = PROBE + f".tmp{os.getpid()}"
    cmd = [HIPCC, "-O3", "-std=c++17", f"--offload-arch={ARCH}", *DEVICE_FLAGS, "-Wno-unused-command-line-argument",
           "-Wno-unknown-warning-option", PROBE_SRC, "-o", tmp]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed on {PROBE_SRC}:\n{proc.stderr}")
    os.replace(tmp, PROBE)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources and {PROBE}")
    return LIB


if __name__ == "__main__":
    build()
