"""Host code under the address and undefined-behaviour sanitizers, on the CPU only:
the oracle's C source (the oracle pin tests re-run against a sanitized build in a child
process), and the library's host-side logic (chunk tables and claim arithmetic of the
self-scheduling kernels, workgroup maps, policy search) through tests/host/host_logic_check.cpp."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def _asan_runtime():
    path = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        pytest.skip("no address-sanitizer runtime for gcc here")
    return path


def test_host_logic_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_logic_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Wextra"] + SAN +
                   [os.path.join(ROOT, "tests", "host", "host_logic_check.cpp"), "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host logic ok" in r.stdout


def test_oracle_under_sanitizers(tmp_path):
    """tests/test_oracle_pins.py once more, in a child process whose oracle library is built with
    the sanitizers (the runtime has to be preloaded into the Python process)."""
    asan = _asan_runtime()
    lib = str(tmp_path / "libhylra_oracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"] + SAN +
                   ["-o", lib, os.path.join(ROOT, "oracle", "hylra_oracle.c"), "-lm"], check=True)
    env = dict(os.environ, HYLRA_ORACLE_LIB=lib, ASAN_OPTIONS="detect_leaks=0",
               LD_PRELOAD=":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "passed" in r.stdout
