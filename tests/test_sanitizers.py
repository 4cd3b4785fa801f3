"""The host code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

Two child processes, each with the sanitizer runtime preloaded: (1) the oracle's C file built with
gcc's sanitizers runs all of its pin tests; (2) libqqq's host side (argument validation, workspace
arithmetic, dispatch) built with clang's sanitizers for the host pass only runs the C-ABI tests.
No GPU is involved: kernels are compiled but never launched.  Any report aborts the child
(-fno-sanitize-recover), which fails the test.
"""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(env_extra, args, timeout):
    env = dict(os.environ)
    env.update(env_extra)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider", *args],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=timeout)
    assert r.returncode == 0, (r.stdout[-3000:] + r.stderr[-3000:])
    assert "passed" in r.stdout


def test_oracle_pins_under_asan_ubsan(tmp_path):
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc's libasan is not installed")
    _run({"QQQ_ORACLE_SANITIZE": str(tmp_path), "LD_PRELOAD": asan},
         ["tests/test_oracle.py", "tests/test_oracle_f16scale.py", "tests/test_oracle_frontend.py"], 900)
    assert os.path.exists(tmp_path / "libqqq_oracle_san.so")


def test_library_host_side_under_asan_ubsan(tmp_path):
    rt = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not rt:
        pytest.skip("clang's shared asan runtime is not installed")
    from paper_2406_09904_amd import build
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-g"]
    lib = build.build(extra_flags=san, out_dir=str(tmp_path))
    _run({"QQQ_LIB_PATH": lib, "LD_PRELOAD": rt[-1]}, ["tests/test_abi.py"], 600)
