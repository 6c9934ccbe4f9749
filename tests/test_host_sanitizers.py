"""The library's host code under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU needed).

bt_api.hip and gemm.hip hold all host logic that takes caller input: the config checks, the
workspace layout, the create path up to its first HIP call, and the GEMM planner.  They are compiled
once more with the sanitizers on the host side only (device code is built as usual), linked with a
small driver (tests/host_san_driver.cpp) and run here, on the CPU.
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2406_02657_amd", "csrc")
OUT = os.path.join(ROOT, "tests", "_host_san")
HIPCC = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else "hipcc"
COMMON = ["-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-math-errno", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
# sanitizers on the host pass only (there is no GPU AddressSanitizer on this pool)
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-fno-sanitize-recover=undefined"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "not a recognized feature for this target" not in l)
    return r.returncode, out


@pytest.mark.timeout(900)
def test_host_code_under_asan_and_ubsan():
    os.makedirs(OUT, exist_ok=True)
    jobs = []
    for src in ("bt_api.hip", "gemm.hip"):
        jobs.append([HIPCC, *COMMON, *SAN, "-c", os.path.join(CSRC, src), "-o", os.path.join(OUT, src.replace(".hip", ".o"))])
    # launchers that the sanitized code links against but never reaches without a GPU: plain objects
    for src in ("elementwise.hip", "attention.hip"):
        jobs.append([HIPCC, *COMMON, "-O3", "-c", os.path.join(CSRC, src), "-o", os.path.join(OUT, src.replace(".hip", ".o"))])
    jobs.append([HIPCC, *COMMON, *SAN, "-x", "hip", "-c", os.path.join(ROOT, "tests", "host_san_driver.cpp"),
                 "-o", os.path.join(OUT, "driver.o")])
    with ThreadPoolExecutor(max_workers=5) as ex:
        for rc, out in ex.map(_run, jobs):
            assert rc == 0, out
    exe = os.path.join(OUT, "host_san_driver")
    objs = [os.path.join(OUT, n) for n in ("bt_api.o", "gemm.o", "elementwise.o", "attention.o", "driver.o")]
    rc, out = _run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", *objs, "-o", exe])
    assert rc == 0, out
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    rc, out = _run([exe], env=env, timeout=600)
    assert rc == 0, out
    assert "checks passed" in out and "AddressSanitizer" not in out and "runtime error" not in out, out
