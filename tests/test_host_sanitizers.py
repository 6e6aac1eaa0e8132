"""Host logic under sanitizers: the layout and planner entry points (pure host functions of the
library) are compiled with host-side AddressSanitizer and UndefinedBehaviorSanitizer, linked to a
fuzz driver and fed ~100,000 random, partly invalid argument sets plus sizes near INT64_MAX."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2504_09983_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# sanitizers on the host side only (the device side of these files holds a few stand-in kernels
# that the driver never launches)
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
       "-Xarch_host", "-fno-sanitize-recover=undefined"]
ARCH = "--offload-arch=gfx950"


@pytest.mark.skipif(not (os.path.exists(HIPCC) or shutil.which("hipcc")), reason="hipcc not available")
def test_layouts_and_planners_fuzzed_under_asan_and_ubsan(tmp_path):
    common = [HIPCC, "-O1", "-g", "-std=c++17", ARCH, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC, *SAN]
    objs = []
    for name in ("zc_core.hip", "zc_plan.hip"):
        obj = str(tmp_path / (name + ".o"))
        subprocess.check_call(common + ["-c", os.path.join(CSRC, name), "-o", obj], stderr=subprocess.DEVNULL)
        objs.append(obj)
    drv = str(tmp_path / "fuzz.o")
    subprocess.check_call(common + ["-x", "hip", "-c", os.path.join(ROOT, "tests", "host_fuzz", "fuzz_planners.cpp"),
                                    "-o", drv], stderr=subprocess.DEVNULL)
    exe = str(tmp_path / "fuzz")
    subprocess.check_call([HIPCC, ARCH, "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                           drv, *objs, "-o", exe], stderr=subprocess.DEVNULL)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]
    calls, ok = (int(x) for x in run.stdout.split()[1::2])
    assert calls > 90_000 and 0.2 * calls < ok < 0.9 * calls, run.stdout      # both paths exercised
