"""Builds libeinet.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libeinet.so")
SOURCES = ["csrc/kernels.hip", "csrc/api.cpp", "csrc/structure.cpp"]
# -packed-fp32-ops is switched off for all device code (a target feature of the device compiler only;
# the host pass warns that it does not know it)
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-shared", "-std=c++17", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(verbose=False):
    cmd = ["hipcc"] + FLAGS + ["-o", LIB_PATH] + [os.path.join(HERE, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libeinet.so")
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
