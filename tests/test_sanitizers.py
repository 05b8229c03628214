"""AddressSanitizer / UndefinedBehaviorSanitizer legs, host code only.

* the oracle's C source, compiled with -fsanitize=undefined, must pass its pins (the pin
  tests run in a child process against that build);
* a C driver calls every oracle entry point on heap buffers of exactly the documented sizes;
  built with -fsanitize=address,undefined it must finish without a report and print the same
  hashes as a plain build;
* the plain-C client of the GPU library (tests/native/zpp_client.c) must compile and link with
  the same flags (it needs a GPU to run; tests/test_gpu_native_client.py runs it there).
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_SRC = os.path.join(ROOT, "oracle", "zpp_oracle.c")
DRIVER_SRC = os.path.join(ROOT, "tests", "native", "oracle_sanitize.c")
BASE = ["gcc", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-Wall", "-Wextra"]
SAN = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
       "-static-libasan"]
SAN_ENV = {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0:halt_on_error=1", "UBSAN_OPTIONS": "print_stacktrace=1:halt_on_error=1"}


def test_oracle_pins_pass_under_ubsan(tmp_path):
    lib = tmp_path / "liboracle_ubsan.so"
    subprocess.run([*BASE, "-O1", "-g", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-fPIC", "-shared",
                    ORACLE_SRC, "-o", str(lib), "-lm"], check=True)
    env = dict(os.environ, ZPP_ORACLE_LIB=str(lib), UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_codec.py"), os.path.join(ROOT, "tests", "test_oracle_qgz.py")],
                       env=env, cwd=ROOT, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "runtime error" not in r.stdout + r.stderr


def test_oracle_driver_is_clean_under_asan_and_ubsan(tmp_path):
    plain, san = tmp_path / "driver_plain", tmp_path / "driver_san"
    subprocess.run([*BASE, "-O2", DRIVER_SRC, ORACLE_SRC, "-o", str(plain), "-lm"], check=True)
    subprocess.run([*BASE, *SAN, DRIVER_SRC, ORACLE_SRC, "-o", str(san), "-lm"], check=True)
    a = subprocess.run([str(plain)], capture_output=True, text=True)
    b = subprocess.run([str(san)], capture_output=True, text=True, env=dict(os.environ, **SAN_ENV))
    assert a.returncode == 0, a.stdout[-2000:] + a.stderr[-2000:]
    assert b.returncode == 0, b.stdout[-2000:] + b.stderr[-4000:]
    assert "ERROR: AddressSanitizer" not in b.stderr and "runtime error" not in b.stderr, b.stderr[-4000:]
    assert a.stdout == b.stdout and a.stdout.count("\n") > 30


def test_c_client_builds_with_sanitizers(tmp_path):
    """Compile and link the GPU library's plain-C client with ASan + UBSan (host code only; the
    GPU kernels it calls live in the shared library, which is not instrumented)."""
    sys.path.insert(0, os.path.join(ROOT, "tests", "native"))
    import importlib.util
    spec = importlib.util.spec_from_file_location("zpp_client_build", os.path.join(ROOT, "tests", "native", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    out = mod.build(force=True, sanitize=True, out=str(tmp_path / "zpp_client_san"))
    assert os.path.exists(out)
