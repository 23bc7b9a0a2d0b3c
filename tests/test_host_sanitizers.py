"""Address / undefined-behaviour sanitizers over the host code (CPU only): the oracle's C source under its own
pins, and the C ABI's validation, planning and workspace carving in a host-only program."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True, check=True).stdout.strip()
    if not os.path.isabs(path):
        pytest.skip(f"{name} is not installed")
    return path


def test_abi_host_layer_under_asan_ubsan(tmp_path):
    exe = tmp_path / "plan_sanitize"
    src = os.path.join(ROOT, "tests", "host", "plan_sanitize.cpp")
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", *SAN, "-o", str(exe), src], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.startswith("ok:"), res.stdout
    planned = int(res.stdout.split(",")[1].split()[0])
    assert planned > 2000


def test_oracle_pins_under_asan_ubsan(tmp_path):
    """The pins of tests/test_oracle_pins.py once more, against an instrumented build of oracle/helix_oracle.c."""
    lib = tmp_path / "libhelix_oracle_san.so"
    subprocess.run(["gcc", "-std=c11", "-Wall", "-fopenmp", "-fPIC", "-shared", *SAN, "-o", str(lib),
                    os.path.join(ROOT, "oracle", "helix_oracle.c"), "-lm"], check=True)
    preload = [_runtime("libasan.so"), _runtime("libubsan.so")]
    if os.environ.get("LD_PRELOAD"):
        preload.append(os.environ["LD_PRELOAD"])
    env = dict(os.environ, HELIX_ORACLE_LIB=str(lib), LD_PRELOAD=":".join(preload),
               # python itself is not instrumented: its allocations are not leaks of the code under test
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT)
    tail = res.stdout[-3000:] + res.stderr[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "runtime error" not in tail and "AddressSanitizer" not in tail, tail
