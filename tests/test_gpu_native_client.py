"""The C ABI used from a plain C program (tests/native/zpp_client.c): no Python or
torch between the caller and the library.  The program compares every output byte of
the five operations with the oracle it is linked against and exits 0 if all agree."""
import importlib.util
import os
import subprocess

import pytest


def client_builder():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "build.py")
    spec = importlib.util.spec_from_file_location("zpp_client_build", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.mark.gpu
def test_plain_c_client_gets_the_oracle_bytes():
    exe = client_builder().build(force=False)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(run.stdout)
    print(run.stderr)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "ALL EQUAL" in run.stdout
    assert run.stdout.count("ok   ") >= 13


@pytest.mark.gpu
def test_plain_c_client_under_host_sanitizers():
    """The same program with its own (host) code instrumented by ASan + UBSan: heap misuse or
    undefined arithmetic in how a C caller prepares buffers and pointer tables would be
    reported here.  The GPU kernels are in the library, which is not instrumented."""
    exe = client_builder().build(force=False, sanitize=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:protect_shadow_gap=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=180, env=env)
    print(run.stdout)
    print(run.stderr[-3000:])
    assert run.returncode == 0, run.stdout + run.stderr[-3000:]
    assert "ALL EQUAL" in run.stdout
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr


def test_header_is_plain_c_and_the_client_links():
    """no GPU needed: the header passes a strict C11 compiler on its own, and the C client
    compiles without warnings and links against the two libraries"""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for name in ("zpp.h", "zpp_diagnostics.h"):
        header = os.path.join(root, "include", name)
        subprocess.run(["gcc", "-std=c11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c", header],
                       check=True)
    exe = client_builder().build(force=True)
    assert os.access(exe, os.X_OK)
