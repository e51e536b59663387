"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host side of the library
(loader, reordering, packer: mgk_host.cpp, mgk_reorder.cpp on a host-only context) and of
the C oracle, each with a small driver under tests/sanitize/.  Host code only; no GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600, **kw)
    assert res.returncode == 0, " ".join(cmd) + "\n" + res.stdout[-4000:]
    return res.stdout


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.exists("/opt/rocm/lib/libamdhip64.so"),
                    reason="needs g++ and the HIP runtime library to link against")
def test_host_code_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "host_driver")
    csrc = os.path.join(ROOT, "paper_1910_06310_amd", "csrc")
    _run(["g++", "-std=c++17", "-pthread", "-D__HIP_PLATFORM_AMD__=1", "-I/opt/rocm/include",
          "-I" + os.path.join(ROOT, "include"), "-I" + csrc] + SAN +
         [os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), os.path.join(csrc, "mgk_host.cpp"),
          os.path.join(csrc, "mgk_reorder.cpp"), "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib",
          "-o", exe])
    out = _run([exe], env=ENV)
    assert "host sanitizer driver: ok" in out and "runtime error" not in out and "AddressSanitizer" not in out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_c_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-std=c99", "-fopenmp"] + SAN +
         [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "mgk_oracle.c"),
          "-lm", "-o", exe])
    out = _run([exe], env=ENV)
    assert "oracle sanitizer driver: ok" in out and "runtime error" not in out and "AddressSanitizer" not in out
