"""CPU sanitizer builds (no GPU): the oracle under AddressSanitizer + UndefinedBehaviorSanitizer with every
pin run on it, and the library's host-side arithmetic (argument checks, launch plan, workspace layout, page
addressing) swept up to the documented limits under the same sanitizers."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]


def _runtime(name):
    path = subprocess.run(["gcc", "-print-file-name=" + name], check=True, capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(path):
        pytest.skip(name + " is not installed")
    return path


def test_oracle_pins_under_asan_ubsan(tmp_path):
    asan = _runtime("libasan.so")
    so = tmp_path / "libsr_oracle_san.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off"] + SAN +
                   [os.path.join(ROOT, "oracle", "sr_oracle.c"), "-o", str(so), "-lm"], check=True)
    code = ("import sys; sys.path[:0] = [%r, %r]\n"
            "import oracle_pins\n"
            "for pin in oracle_pins.ALL_PINS:\n"
            "    pin(%r); print('pinned', pin.__name__, flush=True)\n" % (ROOT, os.path.join(ROOT, "tests"), str(so)))
    env = dict(os.environ)
    # the sanitizer runtime has to be loaded before the interpreter; whatever is preloaded already stays
    env["LD_PRELOAD"] = " ".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    res = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=900)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-4000:]
    assert res.stdout.count("pinned") >= 14


def test_host_side_arithmetic_under_asan_ubsan(tmp_path):
    _runtime("libasan.so")
    exe = tmp_path / "host_sweep"
    subprocess.run(["g++", "-O1", "-std=c++17", "-Wall", "-Wextra", "-Werror"] + SAN +
                   ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2604_16883_amd", "csrc"),
                    os.path.join(ROOT, "tests", "host_sweep.cpp"), "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    res = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert res.stdout.startswith("ok ") and int(res.stdout.split()[1]) > 5000
    assert "runtime error" not in res.stderr
