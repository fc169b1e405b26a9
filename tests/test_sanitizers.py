"""The CPU oracle and the library's host-only entry points built under AddressSanitizer and
UndefinedBehaviorSanitizer and driven over the extremes of their argument ranges (longest
reduction with the extreme codes, every shift, special floats).  A signed overflow of an
accumulator, a shift out of range or an access beyond a buffer aborts the driver."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)  # the sanitizer runtime must come first in the driver's own process


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    err = "\n".join(ln for ln in res.stderr.splitlines() if "packed-fp32-ops" not in ln)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout}\n{err}"
    return res.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-fopenmp",
          "-o", exe, os.path.join(HERE, "oracle_driver.c"), os.path.join(ROOT, "oracle", "qnn_oracle.c"), "-lm"])
    assert _run([exe], env=ENV, timeout=600).strip().endswith("ok")


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
def test_host_helpers_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "host_san")
    csrc = os.path.join(ROOT, "paper_1806_08342_amd", "csrc")
    host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
            "-fno-sanitize-recover=all"]
    _run(["hipcc", "-O1", "-g", "--offload-arch=gfx950", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", *host, "-I" + os.path.join(ROOT, "include"), "-I" + csrc, "-o", exe,
          os.path.join(HERE, "host_helpers_driver.cpp"), os.path.join(csrc, "host_helpers.hip"),
          os.path.join(csrc, "elementwise.hip")], timeout=900)
    assert _run([exe], env=ENV, timeout=600).strip().endswith("ok")
