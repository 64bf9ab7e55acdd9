"""Builds the HIP library in-tree: paper_2601_20309_amd/libduplexkv.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
SRCS = [os.path.join(CSRC, n) for n in ("duplexkv.hip", "kv_table.cpp", "kv_sched.cpp")]
DEPS = SRCS + [os.path.join(CSRC, "kv_kernels.hpp"), os.path.join(CSRC, "kv_engine.hpp"),
               os.path.join(ROOT, "include", "duplexkv.h")]
LIB = os.path.join(HERE, "libduplexkv.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # The tile draws of the move kernel are one atomic per wave whose result is
    # wanted a whole step later.  The compiler's atomic optimizer would rewrite
    # each into "one lane adds for all active lanes, then broadcast", and the
    # broadcast waits for the atomic (and every access before it) on the spot.
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in DEPS)


def build(force: bool = True, verbose: bool = False) -> str:
    if force or stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-o", LIB] + SRCS
        if verbose:
            print(" ".join(cmd))
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines()
                        if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + err)
        if verbose and err.strip():
            print(err, file=sys.stderr)
    return LIB


PROBE_SRC = os.path.join(CSRC, "pack_probe.hip")
PROBE_BIN = os.path.join(HERE, "pack_probe")


def build_probe(out: str = PROBE_BIN) -> str:
    """The stand-alone measurement program that compares shapes of pack / unpack kernel
    (`python -m paper_2601_20309_amd.experiments packshapes` runs it)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wall", "-Wextra",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", out, PROBE_SRC]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("building pack_probe failed:\n" + r.stderr)
    return out


EXAMPLE_SRC = os.path.join(ROOT, "examples", "duplex_demo.c")
EXAMPLE_BIN = os.path.join(ROOT, "examples", "duplex_demo")


def build_example(out: str = EXAMPLE_BIN) -> str:
    """The plain-C example against the built library: a C compiler, the public
    header and the HIP runtime's C API are all it needs."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-O2", "-Wall", "-Wextra", "-Werror", EXAMPLE_SRC, "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(rocm, "include"), "-L", os.path.dirname(LIB), "-lduplexkv",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2601_20309_amd", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the C example failed:\n" + r.stderr)
    return out


if __name__ == "__main__":
    print(build(force=True, verbose=True))
