"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU needed).

Device sanitizers are not available on the test machines, so what can be checked this way is the
host side: the C oracle (every loop the parity tests trust) and the argument checking and launch
planning of the C ABI.  Each test builds a separate, instrumented shared object into a temporary
directory and runs the ordinary `-m "not gpu"` test file against it in a child interpreter with
the sanitizer runtime preloaded; any report aborts the child (halt_on_error) and fails the test.
"""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN_ENV = {"ASAN_OPTIONS": "detect_leaks=0:halt_on_error=1:abort_on_error=1",
           "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"}


def run_pytest_under(runtime, env_extra, test_file):
    env = dict(os.environ, **SAN_ENV, **env_extra)
    env["LD_PRELOAD"] = runtime + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")
    proc = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", test_file), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (proc.stdout + proc.stderr)[-3000:]
    assert proc.returncode == 0, tail
    assert "passed" in proc.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail


def test_oracle_pins_pass_under_asan_and_ubsan(tmp_path):
    from oracle import polar_oracle

    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    so = polar_oracle.build(force=True, out_path=str(tmp_path / "libpolar_oracle_san.so"),
                            extra_flags=("-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                                         "-fno-sanitize-recover=undefined"))
    run_pytest_under(runtime, {"POLAR_ORACLE_LIBRARY": so}, "test_oracle_pins.py")


def test_abi_host_checks_pass_under_asan_and_ubsan(tmp_path):
    from paper_2505_14884_amd import build

    hits = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not hits:
        pytest.skip("clang's AddressSanitizer runtime is not installed")
    # host passes only: each -fsanitize= directly after -Xarch_host (device code is not instrumented)
    flags = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    lib = build.build_library(out_path=str(tmp_path / "libpolar_san.so"), probe_path=str(tmp_path / "libpolar_probe_san.so"),
                              extra_flags=flags)
    run_pytest_under(hits[0], {"POLAR_LIBRARY": lib, "POLAR_PROBE_LIBRARY": str(tmp_path / "libpolar_probe_san.so")},
                     "test_abi_host.py")
