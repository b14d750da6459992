"""Compile the HIP library (csrc/vps_api.hip) for gfx950 into paper_2605_18815_amd/libvps.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libvps.so")
SRC = os.path.join(HERE, "csrc", "vps_api.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build_library(verbose=False):
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-o", LIB, SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0 or verbose:
        print(res.stdout + res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for " + SRC)
    return LIB


def library_path(build_if_missing=True):
    if not os.path.exists(LIB):
        if not build_if_missing:
            raise FileNotFoundError(LIB + " is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        build_library()
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
