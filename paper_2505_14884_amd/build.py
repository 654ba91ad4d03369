"""Compile the HIP libraries for gfx950 in-tree: ``paper_2505_14884_amd/libpolar.so`` (the product,
``include/polar.h``) and ``paper_2505_14884_amd/libpolar_probe.so`` (read yardsticks for the bench,
``include/polar_probe.h``)."""
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
PROBE_LIB_PATH = os.path.join(_PKG, "libpolar_probe.so")
SOURCES = ["polar_abi.hip", "polar_router.hip", "polar_sha.hip", "polar_sha_gqa.hip", "polar_label.hip",
           "polar_gemm.hip", "polar_gemm_down.hip"]
PROBE_SOURCES = ["polar_probe.hip"]
HEADERS = [os.path.join(_ROOT, "include", "polar.h"), os.path.join(_ROOT, "include", "polar_probe.h"),
           os.path.join(CSRC, "polar_internal.h")]

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


def build_library(verbose: bool = False, defines=(), out_path: str = LIB_PATH,
                  probe_path: str = PROBE_LIB_PATH, extra_flags=()) -> str:
    """Compile every HIP source (each with its own flags, in parallel) and link the two shared
    objects; always recompiles.  `defines` (e.g. ["POLAR_SHA_LOADS=8"]) and `out_path` serve tuning
    sweeps; `extra_flags` go to every compile and link line (the host-sanitizer build passes
    `-Xarch_host -fsanitize=...` pairs).  Returns the path of the product library."""
    from concurrent.futures import ThreadPoolExecutor

    objdir = tempfile.mkdtemp(prefix="polar_build_")
    try:
        common = [hipcc()] + HIPCC_FLAGS + list(extra_flags) + ["-D" + d for d in defines]
        common += ["-DPOLAR_SOURCE_HASH=\"%s\"" % source_hash()]
        common += ["-I", os.path.join(_ROOT, "include"), "-I", CSRC]
        jobs = []
        for src in SOURCES + PROBE_SOURCES:
            obj = os.path.join(objdir, src + ".o")
            jobs.append((common + FILE_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj], obj))
        with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
            list(pool.map(lambda j: _run(j[0], verbose), jobs))
        for srcs, path in ((SOURCES, out_path), (PROBE_SOURCES, probe_path)):
            tmp = path + ".tmp.%d" % os.getpid()
            objs = [os.path.join(objdir, src + ".o") for src in srcs]
            _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + list(extra_flags) + ["-o", tmp] + objs, verbose)
            os.replace(tmp, path)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    return out_path


def source_hash() -> str:
    """Hash of every source and header the libraries are built from.  It is compiled into the
    product library (polar_source_hash), so a loader can tell a binary built from other sources
    than the ones on disk whatever the files' time stamps say."""
    import hashlib

    h = hashlib.sha256()
    for path in [os.path.join(CSRC, s) for s in SOURCES + PROBE_SOURCES] + HEADERS:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


if __name__ == "__main__":
    import argparse

    ap = argparse.ArgumentParser(description="Build libpolar.so and libpolar_probe.so for gfx950.")
    ap.add_argument("--define", action="append", default=[], metavar="NAME=VALUE",
                    help="extra preprocessor definition (tuning and timing-only variants), repeatable")
    ap.add_argument("--out", default=LIB_PATH, help="path of the product library (default: in-tree); load a "
                                                    "variant with the environment variable POLAR_LIBRARY")
    ap.add_argument("--probe-out", default="", help="path of the yardstick library (default: beside --out)")
    a = ap.parse_args()
    probe = a.probe_out or (PROBE_LIB_PATH if a.out == LIB_PATH else a.out + ".probe.so")
    print(build_library(verbose=True, defines=a.define, out_path=a.out, probe_path=probe))
