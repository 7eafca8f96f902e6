"""The library's host code (packer, assignment, selection, export, stride-2 parity form) and the C oracle, built
with -fsanitize=address,undefined and run on seeded layers (tests/host_sanitize_main.cpp).  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no g++")
def test_host_code_and_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    csrc = os.path.join(ROOT, "paper_2001_07710_amd", "csrc")
    common = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-O1", "-g"]
    obj = str(tmp_path / "conv_oracle.o")
    subprocess.run(["gcc", *common, "-c", os.path.join(ROOT, "oracle", "conv_oracle.c"), "-o", obj], check=True)
    subprocess.run(["g++", "-std=c++17", *common, "-static-libasan", "-static-libubsan", "-ffp-contract=off",
                    "-I" + os.path.join(ROOT, "include"), "-I" + csrc,
                    os.path.join(ROOT, "tests", "host_sanitize_main.cpp"), os.path.join(csrc, "pconv_host.cpp"), obj,
                    "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "clean under the sanitizers" in run.stdout
