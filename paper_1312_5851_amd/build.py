"""Builds the HIP library (and the CPU-only replay of its FFT phases used by tests).

hipcc cross-compiles for gfx950 without a GPU.  The shared objects are written
next to the sources so that they travel with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
import time

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")

# Translation units of the library as (source, extra defines, object name); they share no device
# code and compile side by side.  The longest first, so that a pool of workers ends evenly.
HIP_UNITS = [
    ("fft_fused.hip", ["-DFFTCONV_FUSED_F=4"], "fft_fused_f4.o"),
    ("fft_fused.hip", ["-DFFTCONV_FUSED_F=3"], "fft_fused_f3.o"),
    ("fft_fused.hip", ["-DFFTCONV_FUSED_F=2"], "fft_fused_f2.o"),
    ("fft_fused.hip", ["-DFFTCONV_FUSED_F=1"], "fft_fused_f1.o"),
    ("fft_inv.hip", [], "fft_inv.o"),
    ("fft_inv_small.hip", [], "fft_inv_small.o"),
    ("fft_fwd_small.hip", [], "fft_fwd_small.o"),
    ("fft_fwd.hip", [], "fft_fwd.o"),
    ("contract.hip", [], "contract.o"),
    ("fft_inv_tiled.hip", [], "fft_inv_tiled.o"),
    ("fft_inv_quad.hip", [], "fft_inv_quad.o"),
    ("skinny.hip", [], "skinny.o"),
    ("fftconv.hip", [], "fftconv.o"),
]
MAX_JOBS = 8

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


def build_library(force: bool = True, extra_flags=(), only_units=None) -> str:
    """Compile the HIP sources under csrc/ for gfx950 and link them into libfftconv.so.

    ``only_units``: names of sources to recompile; the other units reuse their objects if present."""
    out = lib_path()
    if force or _sources_newer(out):
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        objdir = os.path.join(_HERE, "_build")
        os.makedirs(objdir, exist_ok=True)
        only = set(only_units) if only_units else None   # (after a change to one source: recompile just its units)
        pending, running, objs, failed = list(HIP_UNITS), [], [], []
        while pending or running:
            while pending and len(running) < MAX_JOBS:
                src, defines, objname = pending.pop(0)
                obj = os.path.join(objdir, objname)
                objs.append(obj)
                if only is not None and src not in only and os.path.exists(obj):
                    continue
                cmd = [hipcc, *HIPCC_FLAGS, *defines, *extra_flags, "-I", INCLUDE, "-c", "-o", obj, os.path.join(CSRC, src)]
                running.append((cmd, subprocess.Popen(cmd)))
            if running:   # free the slot of whichever compile ends first
                done = [i for i, (_, proc) in enumerate(running) if proc.poll() is not None]
                if not done:
                    time.sleep(0.2)
                    continue
                cmd, proc = running.pop(done[0])
                if proc.returncode != 0:
                    failed.append(cmd)
        if failed:
            raise subprocess.CalledProcessError(1, failed[0])
        link = [hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", out, *objs]
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
    # python -m paper_1312_5851_amd.build [--only a.hip,b.hip] [extra hipcc flags]
    argv = sys.argv[1:]
    only = None
    if argv and argv[0] == "--only":
        only, argv = argv[1].split(","), argv[2:]
    print(build_library(force=True, extra_flags=argv, only_units=only))
    print(build_host_replay(force=True))
