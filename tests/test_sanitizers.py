"""Sanitizer leg (no GPU): the CPU oracle and the host side of the C ABI, each built with
-fsanitize=address,undefined into a small program that walks its edge cases.  A memory
error or undefined behaviour aborts the program, so a zero exit status is the check."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}"
    return r.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=all", os.path.join(SAN, "oracle_driver.cpp"),
          os.path.join(ROOT, "oracle", "ivfpq_oracle.cpp"), "-o", exe])
    out = _run([exe], env=ENV)
    assert "cases clean" in out


def test_abi_host_side_under_sanitizers(tmp_path):
    """The host code of csrc/api.hip, with stubs in place of the kernel launchers: argument
    validation, index description checks and the workspace planner run without a GPU."""
    exe = str(tmp_path / "api_san")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    csrc = os.path.join(ROOT, "paper_2312_01712_amd", "csrc")
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
          "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
          "-Xarch_host", "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "include"), "-I", csrc,
          os.path.join(csrc, "api.hip"), "-x", "hip", os.path.join(SAN, "launch_stubs.cpp"),
          os.path.join(SAN, "api_driver.cpp"), "-o", exe])
    out = _run([exe], env=ENV)
    assert "api_driver: clean" in out
