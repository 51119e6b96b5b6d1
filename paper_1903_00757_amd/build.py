"""Compile the HIP library for gfx950 into paper_1903_00757_amd/libgvhot.so.

hipcc cross-compiles without a GPU, so this runs anywhere the ROCm toolchain is
installed.  Objects go to ``_build/`` (ignored by git); the shared library stays
in-tree next to the binding that loads it.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgvhot.so")
# (source, extra flags, object): the kernels are compiled twice, side by side (see the head of gv_kernels.hip)
SOURCES = [("gv_kernels.hip", [], "gv_kernels.o"), ("gv_kernels.hip", ["-DGV_TRACK_LOSS=1"], "gv_kernels_tracked.o"),
           ("gv_api.cpp", [], "gv_api.o"), ("gv_augment.cpp", [], "gv_augment.o")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-munsafe-fp-atomics", "-Wall", "-Wextra", "-Wno-unused-parameter",
          # packed-fp32 instructions are kept out of the generated code on purpose
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose: bool = False, extra_flags=(), lib: str = LIB, out_dir: str = "", csrc: str = CSRC) -> str:
    """Compile and link; ``extra_flags``, ``lib`` and ``out_dir`` let a caller build a variant
    (other -D settings) beside the product library without touching it."""
    out_dir = out_dir or os.path.join(HERE, "_build")
    os.makedirs(out_dir, exist_ok=True)
    objects = []
    procs = []
    for src, flags, name in SOURCES:
        obj = os.path.join(out_dir, name)
        cmd = [HIPCC, *COMMON, "-I", csrc, *extra_flags, *flags, "-c", os.path.join(csrc, src), "-o", obj]
        if src == "gv_api.cpp":  # uses the HIP vector types in its interface to the kernels
            cmd.insert(1, "-x")
            cmd.insert(2, "hip")
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objects.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + out)
        if verbose and out:
            print(out)
    tmp = lib + f".{os.getpid()}.tmp"
    subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp, *objects, "-lpthread"])
    os.replace(tmp, lib)
    return lib


MICROBENCH = os.path.join(HERE, "microbench_rows")


def build_microbench() -> str:
    """The stand-alone microbenchmark of row operations (csrc/microbench_rows.hip): an executable beside the library."""
    tmp = MICROBENCH + f".{os.getpid()}.tmp"
    cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-munsafe-fp-atomics", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", os.path.join(CSRC, "microbench_rows.hip"), "-o", tmp]
    done = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if done.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + done.stdout)
    os.replace(tmp, MICROBENCH)
    return MICROBENCH


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
    print(build_microbench())
