"""CPU builds of the C oracle and of the host half of the C ABI (csrc/cf_api.cpp with stand-in launchers, no
device) under AddressSanitizer and UndefinedBehaviorSanitizer, each driven by a small program of its own
(tests/host_sanitize/).  A sanitizer report makes the program exit non-zero."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "host_sanitize")
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)         # the sanitizer runtime must come first in the program it is linked into


def _run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout[-4000:]}"
    return res.stdout


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-std=c11", "-ffp-contract=off", *SAN, "-I", os.path.join(ROOT, "oracle"),
          os.path.join(ROOT, "oracle", "cf_oracle.c"), os.path.join(HERE, "oracle_driver.c"), "-o", exe, "-lm"])
    out = _run([exe], env=ENV)
    assert "ran clean" in out


def test_abi_host_half_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "abi_san")
    inc = ["-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2507_17511_amd", "csrc")]
    _run(["g++", "-std=c++17", *SAN, *inc, os.path.join(ROOT, "paper_2507_17511_amd", "csrc", "cf_api.cpp"),
          os.path.join(HERE, "stubs.cpp"), os.path.join(HERE, "host_driver.cpp"), "-o", exe])
    out = _run([exe], env=ENV)
    assert "all expectations hold" in out
