"""Build the HIP shared library for gfx950 with hipcc (no JIT, in-tree output)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libscout.so")
SOURCES = ["score.hip", "append.hip", "fetch.hip", "topk.hip", "attn.hip", "api.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep hipcc from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


CALIB_LIB = os.path.join(HERE, "libscout_calib.so")


def _hipcc(sources, out, verbose):
    cmd = ["hipcc", *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in sources], "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in res.stderr.splitlines() if noise not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return out


def build(verbose: bool = False) -> str:
    """Compile every kernel source into libscout.so next to this file (and the measurement aids into
    libscout_calib.so, a library of their own); returns the path of libscout.so."""
    _hipcc(["calib.hip"], CALIB_LIB, verbose)
    return _hipcc(SOURCES, LIB, verbose)


HOST_LIB = os.path.join(HERE, "libscout_host.so")


def build_host(verbose: bool = False) -> str:
    """Compile the host-side worker (plain C++17, threads) into libscout_host.so next to this file."""
    cmd = ["g++", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra", "-Wno-psabi",
           "-I", os.path.join(ROOT, "include"), os.path.join(CSRC, "host_worker.cpp"), "-o", HOST_LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("g++ failed:\n" + res.stderr)
    if verbose and res.stderr.strip():
        print(res.stderr)
    return HOST_LIB


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_host(verbose=True))
