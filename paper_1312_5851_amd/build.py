"""Builds the HIP library (and the CPU-only replay of its FFT phases used by tests).

hipcc cross-compiles for gfx950 without a GPU.  The shared objects are written
next to the sources so that they travel with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")

# translation units of the library; they share no device code and compile side by side
HIP_SOURCES = ["fftconv.hip", "fft_fused.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def lib_path() -> str:
    return os.path.join(_HERE, "libfftconv.so")


def replay_lib_path() -> str:
    return os.path.join(_HERE, "libfft_host_replay.so")


def _sources_newer(target: str) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    for d in (CSRC, INCLUDE):
        for name in os.listdir(d):
            if os.path.getmtime(os.path.join(d, name)) > t:
                return True
    return False


def build_library(force: bool = True, extra_flags=()) -> str:
    """Compile the HIP sources under csrc/ for gfx950 and link them into libfftconv.so."""
    out = lib_path()
    if force or _sources_newer(out):
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        objdir = os.path.join(_HERE, "_build")
        os.makedirs(objdir, exist_ok=True)
        jobs = []
        for src in HIP_SOURCES:
            obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
            cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", INCLUDE, "-c", "-o", obj, os.path.join(CSRC, src)]
            jobs.append((obj, cmd, subprocess.Popen(cmd)))
        failed = [cmd for _, cmd, proc in jobs if proc.wait() != 0]
        if failed:
            raise subprocess.CalledProcessError(1, failed[0])
        link = [hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", out, *[obj for obj, _, _ in jobs]]
        subprocess.run(link, check=True)
    return out


def build_host_replay(force: bool = False) -> str:
    """Compile the CPU replay of the FFT kernel phases (plain g++, no HIP)."""
    out = replay_lib_path()
    if force or _sources_newer(out):
        cmd = ["g++", "-std=c++17", "-O1", "-fPIC", "-shared", "-o", out, os.path.join(CSRC, "fft_host_replay.cpp")]
        subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build_library(force=True, extra_flags=sys.argv[1:]))
    print(build_host_replay(force=True))
