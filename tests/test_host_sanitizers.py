"""The host side of the library (encoder, validator) under AddressSanitizer and UndefinedBehaviorSanitizer: a small C++
driver (sanitize_driver.cpp) is built with g++ from the library's two host-only sources and run on random matrices with
every option, carried dictionaries, and corrupted or truncated containers.  No GPU involved."""
import os
import shutil
import subprocess
import tempfile

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2509_22951_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_encoder_and_validator_are_clean_under_asan_and_ubsan():
    folder = tempfile.mkdtemp(prefix="tq_san_")
    exe = os.path.join(folder, "driver")
    build = subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-pthread",
                            os.path.join(HERE, "sanitize_driver.cpp"), os.path.join(CSRC, "tq_encode.cpp"),
                            os.path.join(CSRC, "tq_blob.cpp"), "-o", exe], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "containers encoded and validated" in run.stdout
