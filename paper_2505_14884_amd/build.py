"""Compile the HIP library for gfx950 in-tree (``paper_2505_14884_amd/libpolar.so``)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
LIB_PATH = os.path.join(_PKG, "libpolar.so")
SOURCES = ["polar_abi.hip", "polar_router.hip", "polar_sha.hip", "polar_sha_gqa.hip", "polar_label.hip", "polar_probe.hip", "polar_gemm.hip"]

# Packed-fp32 instructions are switched off for all device code of this library.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the library cannot be built")
    return exe


def build_library(verbose: bool = False, defines=(), out_path: str = LIB_PATH) -> str:
    """Compile every HIP source into one shared object; always recompiles.
    `defines` (e.g. ["POLAR_SHA_LOADS=8"]) and `out_path` serve tuning sweeps."""
    tmp = out_path + ".tmp.%d" % os.getpid()
    cmd = [hipcc()] + HIPCC_FLAGS + ["-D" + d for d in defines]
    cmd += ["-I", os.path.join(_ROOT, "include"), "-I", CSRC, "-o", tmp]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
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
    os.replace(tmp, out_path)
    return out_path


if __name__ == "__main__":
    print(build_library(verbose=True))
