"""The fp64 oracle and the C ABI's host layer (argument validation, workspace plan, dispatch) built for the CPU with
AddressSanitizer and UndefinedBehaviorSanitizer and run on small inputs.  Host code only: the ABI layer is compiled
without its device side and linked against stand-ins for the kernel launch sequences (tests/sanitize/)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)   # a preloaded library would have to come after the sanitizer runtime


def _run(exe):
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=ENV)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr
    return r.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           os.path.join(ROOT, "oracle", "deltanet_oracle.c"), os.path.join(SAN, "oracle_main.c"), "-o", exe, "-lm"])
    assert "rc=0" in _run(exe)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_c_abi_host_layer_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "abi_san")
    cmd = ["hipcc", "--offload-host-only", "-x", "hip", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
           os.path.join(ROOT, "paper_2406_06484_amd", "csrc", "dn_api.hip"), os.path.join(SAN, "abi_stubs.cpp"),
           os.path.join(SAN, "abi_main.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-3000:]
    assert "host layer under sanitizers: ok" in _run(exe)
