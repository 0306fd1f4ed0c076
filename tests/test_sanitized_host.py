"""The oracle and the host side of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (CPU
only): the oracle is rebuilt with -fsanitize=address,undefined into a temporary library, and the oracle
pins plus the host-only ABI checks run against it in a child process (the sanitizer runtime has to be
loaded before Python's own allocator work, hence LD_PRELOAD in a fresh interpreter)."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _asan_runtime():
    out = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return out if out and os.path.sep in out and os.path.exists(out) else None


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_pins_and_abi_host_checks_under_asan_ubsan(tmp_path):
    rt = _asan_runtime()
    if rt is None:
        pytest.skip("gcc has no shared AddressSanitizer runtime here")
    lib = tmp_path / "liboracle_asan.so"
    subprocess.run(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                    os.path.join(ROOT, "oracle", "gsa_oracle.c"), "-o", str(lib), "-lm"], check=True)
    env = dict(os.environ)
    env["LD_PRELOAD"] = (rt + " " + env.get("LD_PRELOAD", "")).strip()
    # Python itself is not leak-clean; every other report aborts the child
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["GSA_ORACLE_LIB"] = str(lib)
    env["OMP_NUM_THREADS"] = "2"
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                          os.path.join(ROOT, "tests", "test_abi_host.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
