"""CPU sanitizer runs (AddressSanitizer + UndefinedBehaviorSanitizer, gcc): the C oracle under its pins, and the host
side of the C-ABI library -- handles, contexts, argument checks, copies, scratch layout -- on a fake device that lives
on the host heap (tests/hip_stub).  Each runs in a child process with the sanitizer runtime preloaded; a report makes
the child fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
STUB = os.path.join(ROOT, "tests", "hip_stub")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def _runtime(name):
    path = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(path):
        pytest.skip("gcc has no %s here" % name)
    return path


def _env(**extra):
    env = dict(os.environ)
    env["LD_PRELOAD"] = " ".join(x for x in (_runtime("libasan.so"), env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=66"      # python itself leaks by design
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=67"
    env["OMP_NUM_THREADS"] = "4"
    env.update(extra)
    return env


def test_host_side_of_the_library_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "liblite_attn_hostcheck.so")
    csrc = os.path.join(ROOT, "paper_2511_11062_amd", "csrc")
    cmd = ["g++", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra"] + SAN + [
        "-I" + STUB, "-I" + os.path.join(ROOT, "include"), "-I" + csrc,
        os.path.join(csrc, "lite_attn.cpp"), os.path.join(csrc, "lite_attn_host.cpp"),
        os.path.join(STUB, "fake_launches.cpp"), "-o", lib]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    res = subprocess.run([sys.executable, os.path.join(STUB, "lifecycle.py"), lib], capture_output=True, text=True,
                         env=_env(), timeout=600)
    assert res.returncode == 0 and "lifecycle ok" in res.stdout, res.stdout[-2000:] + res.stderr[-6000:]
    # the argument-error tests of the ABI suite, against the same build
    res = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_abi.py"), "-k", "bad_arguments_are_rejected"],
                         capture_output=True, text=True, env=_env(LITE_ATTN_TEST_LIB=lib), timeout=600, cwd=ROOT)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]


def test_oracle_under_asan_and_ubsan_passes_its_pins():
    """The pins of the oracle run against a sanitizer build of the same C source (both precisions)."""
    res = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         capture_output=True, text=True, env=_env(LA_ORACLE_SANITIZE="1"), timeout=1500, cwd=ROOT)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-6000:]
    assert "passed" in res.stdout
