"""Host-side sanitizer builds (no GPU): the CPU oracle, and the host code of
libadt, compiled with -fsanitize=address,undefined and driven through edge
tables (empty layers, byte counts 1,3,1,3,..., ragged sizes, invalid tables).
A sanitizer report aborts the driver, so a zero exit status means none."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = tmp_path / "oracle_san"
    subprocess.check_call(["gcc", "-std=c99", "-O1", "-g", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-Wall", "-Wextra", "-Werror",
                           os.path.join(ROOT, "oracle", "adt_oracle.c"),
                           os.path.join(SAN, "oracle_driver.c"), "-o", str(exe), "-lm"])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120, env=ENV)
    assert out.returncode == 0 and "oracle sanitizer driver ok" in out.stdout, (out.stdout, out.stderr)


def test_library_host_code_under_sanitizers(tmp_path):
    """The library's sources plus the driver in one executable; the sanitizers
    instrument the host code only (device code cannot be sanitized here)."""
    from paper_2004_02297_amd import _build
    try:
        hipcc = _build.hipcc()
    except RuntimeError:
        pytest.skip("no hipcc")
    exe = tmp_path / "host_san"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    flags = [f for f in _build.HIPCC_FLAGS if f not in ("-shared", "-fPIC", "-O3")]
    cmd = [hipcc, *flags, "-O1", "-g", *san, "-I", os.path.join(ROOT, "include"), "-o", str(exe),
           os.path.join(SAN, "host_driver.cpp")] + [os.path.join(_build.CSRC, s) for s in _build.SOURCES]
    subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120, env=ENV)
    assert out.returncode == 0 and "host sanitizer driver ok" in out.stdout, (out.stdout, out.stderr)
