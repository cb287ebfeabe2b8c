"""Compile libmics.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libmics.so")
SOURCES = [os.path.join(HERE, "csrc", "api.cpp"), os.path.join(HERE, "csrc", "kernels.hip")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
    # reproducible arithmetic: no FMA contraction, IEEE division/sqrt, denormals kept
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-gpu-flush-denormals-to-zero",
    # no packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build(extra_flags=(), out: str = LIB, verbose: bool = False) -> str:
    tmp = out + f".tmp{os.getpid()}"
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", tmp, *SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    log = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    os.replace(tmp, out)
    return out


EXAMPLE_SRC = os.path.join(HERE, "examples", "step_from_c.cpp")
EXAMPLE_BIN = os.path.join(HERE, "examples", "step_from_c")


def build_example(out: str = EXAMPLE_BIN) -> str:
    """The plain host program that drives libmics.so through its C ABI (no Python, no PyTorch)."""
    tmp = out + f".tmp{os.getpid()}"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O2", "-std=c++17", EXAMPLE_SRC,
           "-I" + os.path.join(HERE, "..", "include"), "-L" + HERE, "-lmics", "-Wl,-rpath,$ORIGIN/..", "-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    import sys
    # usage: build.py [out.so] [-DNAME=VALUE ...]   (variants for measurements)
    out = next((a for a in sys.argv[1:] if not a.startswith("-")), LIB)
    print(build([a for a in sys.argv[1:] if a.startswith("-")], out=out, verbose=True))
