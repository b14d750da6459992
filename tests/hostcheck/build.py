"""Compile the CPU build of the library's per-item code (test infrastructure)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libvps_hostcheck.so")
SRC = os.path.join(HERE, "hostcheck.cpp")
CSRC = os.path.join(HERE, "..", "..", "paper_2605_18815_amd", "csrc")


LIB_ASAN = os.path.join(HERE, "libvps_hostcheck_asan.so")


def _deps():
    deps = [SRC] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    deps.append(os.path.join(HERE, "..", "..", "include", "vps.h"))
    return deps


def build():
    if os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(d) for d in _deps()):
        return LIB
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-Wall", "-Wextra",
                    "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-o", LIB, SRC], check=True)
    return LIB


def build_asan():
    """The same with AddressSanitizer (heap bounds and lifetimes of the tables).  A process that
    loads it needs the sanitizer runtime preloaded: see asan_env()."""
    if os.path.exists(LIB_ASAN) and os.path.getmtime(LIB_ASAN) >= max(os.path.getmtime(d) for d in _deps()):
        return LIB_ASAN
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-Wall", "-Wextra",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-o", LIB_ASAN, SRC], check=True)
    return LIB_ASAN


def asan_env():
    """Environment for a child process that loads the sanitizer build through ctypes."""
    # the C++ runtime goes along: the sanitizer looks up __cxa_throw when it starts, and the Python
    # executable itself does not link libstdc++
    libs = [subprocess.run(["gcc", "-print-file-name=" + n], capture_output=True, text=True, check=True).stdout.strip()
            for n in ("libasan.so", "libstdc++.so.6")]
    return dict(os.environ, VPSH_LIB=build_asan(), LD_PRELOAD=" ".join(libs), ASAN_OPTIONS="detect_leaks=0:abort_on_error=0")
