"""Compile the CPU build of the library's per-item code (test infrastructure)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libvps_hostcheck.so")
SRC = os.path.join(HERE, "hostcheck.cpp")
CSRC = os.path.join(HERE, "..", "..", "paper_2605_18815_amd", "csrc")


def build():
    deps = [SRC] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    deps.append(os.path.join(HERE, "..", "..", "include", "vps.h"))
    if os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(d) for d in deps):
        return LIB
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-Wall", "-Wextra",
                    "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-o", LIB, SRC], check=True)
    return LIB
