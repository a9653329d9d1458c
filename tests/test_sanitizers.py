"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the C++ planner on seeded
random operator lists and the C oracle on small operators.  The drivers are compiled here, with the host
compilers, and run as child processes."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-g", "-O1"]
# (the sanitizer runtime is linked statically and told not to insist on being the first library loaded)
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout}\n{res.stderr}"
    return res.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_planner_under_sanitizers(tmp_path):
    exe = str(tmp_path / "planner_driver")
    _run(["g++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"),
          "-I", os.path.join(ROOT, "paper_1901_10008_amd", "csrc"),
          os.path.join(ROOT, "tests", "sanitize", "planner_driver.cpp"),
          os.path.join(ROOT, "paper_1901_10008_amd", "csrc", "planner.cpp"), "-o", exe])
    assert "planner_driver: ok" in _run([exe], env=ENV)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no host C compiler")
def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-std=c11", *SAN, "-fopenmp", os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
          os.path.join(ROOT, "oracle", "sk_oracle.c"), "-lm", "-o", exe])
    assert "oracle_driver: ok" in _run([exe], env=dict(ENV, OMP_NUM_THREADS="2"))
