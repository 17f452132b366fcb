"""Builds libeinet.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libeinet.so")
SOURCES = ["csrc/leaf_forward.hip", "csrc/einsum_forward.hip", "csrc/einsum_backward.hip", "csrc/root_layer.hip", "csrc/statistics.hip",
           "csrc/update.hip", "csrc/sampling.hip", "csrc/static_scratch.hip", "csrc/peaks.hip", "csrc/api.cpp", "csrc/structure.cpp"]
# -packed-fp32-ops is switched off for all device code (a target feature of the device compiler only;
# the host pass warns that it does not know it)
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _report(res, verbose):
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))


def build_library(verbose=False):
    """Compiles every translation unit (side by side, at most eight at a time) and links them."""
    with tempfile.TemporaryDirectory(prefix="einet_build_") as tmp:
        jobs = []
        for src in SOURCES:
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            cmd = ["hipcc"] + FLAGS + ["-c", os.path.join(HERE, src), "-o", obj]
            jobs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
        failed = []
        for src, obj, proc in jobs:
            out, err = proc.communicate()
            res = subprocess.CompletedProcess(proc.args, proc.returncode, out, err)
            _report(res, verbose)
            if proc.returncode != 0:
                failed.append(src)
        if failed:
            raise RuntimeError("hipcc failed compiling " + ", ".join(failed))
        link = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] +
                              [obj for _, obj, _ in jobs], capture_output=True, text=True)
        _report(link, verbose)
        if link.returncode != 0:
            raise RuntimeError("hipcc failed linking libeinet.so")
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
