"""Debug target: the CPU oracle and the host side of the HIP library built
with AddressSanitizer and UndefinedBehaviorSanitizer and run on the host.
The drivers under ``tests/host_sanitize/`` call every oracle function on
corner-case inputs and every host-side path of the library that returns
before its first kernel launch (sizing, geometry, argument checks); any
report from a sanitizer fails the run. No GPU is involved: sanitizers run on
host code only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "host_sanitize")
SAN_ENV = {"ASAN_OPTIONS": "abort_on_error=0:halt_on_error=1",
           "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"}


def _run(exe, extra_env=None):
    env = dict(os.environ)
    env.update(SAN_ENV)
    env.update(extra_env or {})
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                         env=env, timeout=300)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "runtime error" not in res.stdout and "AddressSanitizer" not in res.stdout, res.stdout[-4000:]
    assert "0 failures" in res.stdout, res.stdout[-2000:]


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_driver")
    cmd = [gcc, "-O1", "-g", "-std=c11", "-fno-fast-math", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-Wall", "-Wextra",
           "-o", exe, os.path.join(HERE, "oracle_driver.c"),
           os.path.join(ROOT, "oracle", "rtopk_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    _run(exe)                                     # leak detection stays on: the oracle frees what it takes


def test_library_host_side_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from paper_2005_10761_amd import build as hip_build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    exe = str(tmp_path / "abi_driver")
    flags = [f for f in hip_build.HIPCC_FLAGS if f not in ("-O3", "-fPIC", "-shared")]
    san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"):
        san += ["-Xarch_host", f]                 # host code only: the device code is built as always
    cmd = [hipcc, "-O1", "-g"] + flags + san + ["-o", exe, os.path.join(HERE, "abi_driver.cpp")] \
        + hip_build.sources()
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-4000:]
    # the HIP runtime keeps its own allocations until the process ends
    _run(exe, {"ASAN_OPTIONS": SAN_ENV["ASAN_OPTIONS"] + ":detect_leaks=0"})
