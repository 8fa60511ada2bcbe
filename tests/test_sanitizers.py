"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; nothing of the kind runs on
the GPU): the oracle on small inputs through every entry point, and the library's planning and argument
validation, which return before anything is launched."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
SAN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="4")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    sys.stdout.write(r.stdout[-4000:])
    return r


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-o", exe,
           os.path.join(HERE, "oracle_driver.c"), os.path.join(ROOT, "oracle", "fsd_oracle.c"), "-lm"]
    r = _run(cmd)
    assert r.returncode == 0, "the sanitizer build of the oracle failed"
    r = _run([exe], env=SAN_ENV, timeout=600)
    assert r.returncode == 0 and "0 failing calls" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc is needed to build the library's host side")
def test_abi_validation_under_sanitizers(tmp_path):
    from paper_2502_20704_amd import build as hip_build

    exe = str(tmp_path / "abi_san")
    flags = [f for f in hip_build.FLAGS if f not in ("-shared", "-O3")]
    cmd = ["hipcc", "-O1", "-g", *flags, "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-o", exe, os.path.join(HERE, "abi_driver.cpp"), hip_build.SRC]
    r = _run(cmd)
    assert r.returncode == 0, "the sanitizer build of the library's host side failed"
    r = _run([exe], env=SAN_ENV, timeout=300)
    assert r.returncode == 0 and "0 unexpected results" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout
