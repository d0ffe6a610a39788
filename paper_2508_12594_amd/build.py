"""Compile libflare.so and libflare_rates.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2508_12594_amd.build

hipcc cross-compiles without a GPU.  The libraries are written next to this file so that
they travel with the source tree; nothing is installed.  libflare.so is the operator;
libflare_rates.so holds the machine-rate micro-benchmarks of include/flare_rates.h, which the
operator does not link.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libflare.so")
RATES_LIB = os.path.join(HERE, "libflare_rates.so")
RATES_SOURCES = {"machine_rates.hip": []}
# source -> extra flags.  The matrix-core files never produce NaNs (masked scores are -inf and
# are only ever compared, exponentiated or shifted by finite values), so they are compiled with
# -fno-honor-nans: fmaxf chains then become v_max3_f32 without canonicalising moves.
SOURCES = {"flare_api.hip": [], "flare_valu.hip": [], "flare_mfma_fwd.hip": ["-fno-honor-nans"],
           "flare_mfma_bwd.hip": ["-fno-honor-nans"], "flare_mfma_proj.hip": ["-fno-honor-nans"],
           "flare_spectral.hip": []}

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_library(verbose=True, extra_flags=()):
    """Both libraries; returns the path of libflare.so."""
    _build(RATES_LIB, RATES_SOURCES, verbose, extra_flags)
    return _build(LIB, SOURCES, verbose, extra_flags)


def _build(lib, sources, verbose, extra_flags):
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs, procs = [], []
    for src, flags in sources.items():
        obj = os.path.join(objdir, src.replace(".hip", ".%d.o" % os.getpid()))
        cmd = ["hipcc"] + FLAGS + flags + list(extra_flags) + inc + ["-c", "-o", obj, os.path.join(CSRC, src)]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd)))
        objs.append(obj)
    for cmd, proc in procs:
        if proc.wait() != 0:
            raise subprocess.CalledProcessError(proc.returncode, cmd)
    tmp = lib + ".tmp.%d" % os.getpid()
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, lib)
    for obj in objs:
        os.remove(obj)
    return lib


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
