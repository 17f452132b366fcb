"""The host code of the library (structure compiler, argument checks, table upload, layer loops of the C ABI) under
AddressSanitizer and UndefinedBehaviorSanitizer, in a CPU process: api.cpp and structure.cpp are compiled with g++,
the kernel launchers and the handful of HIP runtime calls are replaced by the stand-ins of tests/host_sanitizer/stubs.cpp,
and tests/host_sanitizer/driver.cpp walks forty random models (the generator of the GPU random-shapes test), the
benchmark structures at a small K, and the error paths through create / sizes / structure / bind / the compute calls /
destroy.  Sanitizers never run on the GPU."""
import os
import shutil
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2004_06231_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "host_sanitizer")


def _line(structure, K, C, family, B, D=0, depth=0, R=0, seed=0, H=0, W=0, deltas=(), axes=3, param=0):
    d = list(deltas) + [0, 0]
    return f"{structure} {K} {C} {family} {B} {D} {depth} {R} {seed} {H} {W} {len(deltas)} {d[0]} {d[1]} {axes} {param}"


def _models():
    from tests.test_gpu_random_shapes import draw_case
    lines = []
    for case in range(40):
        family, param, K, C, B, spec, _, seed = draw_case(case)
        if spec["kind"] == "rat":
            lines.append(_line(0, K, C, family, B, D=spec["D"], depth=spec["depth"], R=spec["R"], seed=seed, param=param))
        else:
            lines.append(_line(1, K, C, family, B, H=spec["H"], W=spec["W"], deltas=spec["deltas"], axes=spec.get("axes", 3),
                               seed=seed, param=param))
    # the benchmark structures (small K: the tables do not depend on it) and shapes that must be refused
    lines.append(_line(0, 4, 1, 0, 64, D=8, depth=3, R=2, seed=1))
    lines.append(_line(0, 2, 1, 0, 10, D=784, depth=8, R=10, seed=2))
    lines.append(_line(1, 8, 1, 1, 16, H=28, W=28, deltas=[7]))
    lines.append(_line(1, 8, 3, 1, 128, H=32, W=32, deltas=[8]))
    lines.append(_line(1, 4, 3, 1, 8, H=64, W=64, deltas=[16, 8]))
    lines.append(_line(1, 40, 3, 1, 4, H=32, W=32, deltas=[8], axes=2))
    lines.append(_line(0, 4, 1, 0, 8, D=4, depth=3, R=1))             # a one-variable scope would have to split
    lines.append(_line(1, 4, 1, 1, 8, H=4, W=4, deltas=[9]))           # no delta cuts the image
    lines.append(_line(0, 65, 1, 0, 8, D=8, depth=1, R=1))            # K out of range
    lines.append(_line(0, 4, 1, 2, 8, D=8, depth=1, R=1, param=0))    # binomial without trials
    lines.append(_line(0, 4, 1, 3, 8, D=8, depth=1, R=1, param=300))  # too many categorical values
    return lines


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"),
                    reason="needs g++ and the HIP headers")
def test_host_code_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "host_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           os.path.join(CSRC, "api.cpp"), os.path.join(CSRC, "structure.cpp"), os.path.join(HERE, "stubs.cpp"),
           os.path.join(HERE, "driver.cpp"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], input="\n".join(_models()) + "\n", capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout[-3000:], run.stderr[-6000:])
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr, run.stderr[-6000:]
    out = run.stdout.strip().splitlines()
    assert out[-1].startswith("models 51 "), out[-1]
    ok = [l for l in out if " ok regions" in l]
    refused = [l for l in out if "create rc=" in l]
    assert len(ok) + len(refused) == 51 and len(refused) >= 5
    assert not any("FAILED" in l for l in out)
