"""The host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the planner (deft_plan.cpp holds
no device call and builds with plain g++) and the C oracle are compiled with -fsanitize=address,undefined together
with small drivers that run them over random and damaged inputs; any out-of-bounds access, use after free, leak,
signed overflow or misaligned access makes the driver exit non-zero."""

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)  # the sanitizer runtime wants to come first


def run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=ENV, timeout=600)
    assert p.returncode == 0, " ".join(cmd) + "\n" + p.stdout[-4000:]
    return p.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "plan_driver")
    run(["g++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"),
         "-I", os.path.join(ROOT, "paper_2404_00242_amd", "csrc"),
         os.path.join(ROOT, "paper_2404_00242_amd", "csrc", "deft_plan.cpp"),
         os.path.join(ROOT, "tests", "sanitize", "plan_driver.cpp"), "-lpthread", "-o", exe])
    out = run([exe])
    assert "plans" in out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_c_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    run(["gcc", "-std=c11", "-fopenmp", *SAN, os.path.join(ROOT, "oracle", "tree_attention_oracle.c"),
         os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-lm", "-o", exe])
    assert "oracle ok" in run([exe])
