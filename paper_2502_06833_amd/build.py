"""Compile the HIP library (csrc/ead.hip) for gfx950 into paper_2502_06833_amd/libead.so."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libead.so")
SOURCES = ["ead.hip"]
HEADERS = ["common.hpp", "linear.hpp", "attention.hpp", "entropy.hpp", "state.hpp", "fused.hpp", "stream.hpp"]


def _newest_source() -> float:
    files = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    files.append(os.path.join(os.path.dirname(HERE), "include", "ead.h"))
    return max(os.path.getmtime(f) for f in files)


def is_stale() -> bool:
    return not os.path.exists(LIB) or os.path.getmtime(LIB) < _newest_source()


def build(force: bool = True, verbose: bool = False) -> str:
    """hipcc cross-compiles for gfx950; no GPU is needed to build."""
    if not force and not is_stale():
        return LIB
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", LIB] + [os.path.join(CSRC, f) for f in SOURCES]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
