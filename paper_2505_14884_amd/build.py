"""Compile the HIP library for gfx950 in-tree (``paper_2505_14884_amd/libpolar.so``)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
LIB_PATH = os.path.join(_PKG, "libpolar.so")
SOURCES = ["polar_abi.hip", "polar_router.hip", "polar_sha.hip", "polar_sha_gqa.hip", "polar_label.hip", "polar_probe.hip", "polar_gemm.hip", "polar_gemm_down.hip"]

# Packed-fp32 instructions are switched off for all device code of this library.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]

# Per-file additions.  The router's fp64 matrix-core loop keeps five accumulator tiles live across
# iterations; with the default register classes the compiler copies all 40 registers between the
# vector and the accumulation file around every iteration, the VGPR form of MFMA avoids that.
FILE_FLAGS = {"polar_router.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the library cannot be built")
    return exe


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    # hipcc's host pass does not know the packed-fp32 feature switch and says so once per
    # compile step; that notice is harmless, everything else is passed through
    noise = "is not a recognized feature for this target"
    rest = [ln for ln in proc.stderr.splitlines() if noise not in ln]
    if rest:
        print("\n".join(rest), file=sys.stderr, flush=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed with exit code %d" % proc.returncode)


def build_library(verbose: bool = False, defines=(), out_path: str = LIB_PATH) -> str:
    """Compile every HIP source (each with its own flags, in parallel) and link one shared object;
    always recompiles.  `defines` (e.g. ["POLAR_SHA_LOADS=8"]) and `out_path` serve tuning sweeps."""
    from concurrent.futures import ThreadPoolExecutor

    tmp = out_path + ".tmp.%d" % os.getpid()
    objdir = tempfile.mkdtemp(prefix="polar_build_")
    try:
        common = [hipcc()] + HIPCC_FLAGS + ["-D" + d for d in defines]
        common += ["-I", os.path.join(_ROOT, "include"), "-I", CSRC]
        jobs = []
        for src in SOURCES:
            obj = os.path.join(objdir, src + ".o")
            jobs.append((common + FILE_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj], obj))
        with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
            list(pool.map(lambda j: _run(j[0], verbose), jobs))
        _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [obj for _, obj in jobs], verbose)
        os.replace(tmp, out_path)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    return out_path


if __name__ == "__main__":
    print(build_library(verbose=True))
