"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle (random round trips of every format),
the library's host-side code construction (random histograms) and its container validation (damaged containers).
GPU code is not involved."""
import os
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
FLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def _build_and_run(tmp_path, compiler, args, exe):
    if shutil.which(compiler) is None:
        pytest.skip(compiler + " not found")
    out = str(tmp_path / exe)
    built = subprocess.run([compiler] + FLAGS + args + ["-o", out], capture_output=True, text=True)
    if built.returncode != 0 and ("asan" in built.stderr.lower() or "ubsan" in built.stderr.lower()):
        pytest.skip("sanitizer runtime not installed")
    assert built.returncode == 0, built.stderr
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)                      # the sanitizer runtime must come first in the process
    ran = subprocess.run([out], capture_output=True, text=True, env=env, timeout=600)
    assert ran.returncode == 0 and ran.stdout.startswith("ok"), (ran.stdout, ran.stderr[-2000:])


def test_oracle_round_trips_under_sanitizers(tmp_path):
    _build_and_run(tmp_path, "gcc", ["-std=c99", os.path.join(HERE, "sanitize", "oracle_round_trips.c"),
                                     os.path.join(ROOT, "oracle", "zc_oracle.c"), "-lm"], "oracle_round_trips")


def test_host_code_construction_under_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2508_19263_amd", "csrc")
    _build_and_run(tmp_path, "g++", ["-std=c++17", "-I" + csrc, os.path.join(HERE, "sanitize", "host_code_lengths.cpp"),
                                     os.path.join(csrc, "zc_codebook.cpp")], "host_code_lengths")


def test_host_container_validation_under_sanitizers(tmp_path):
    # the validator and the code construction it links against are the library's; the containers are the oracle's
    csrc = os.path.join(ROOT, "paper_2508_19263_amd", "csrc")
    _build_and_run(tmp_path, "g++", ["-std=c++17", "-I" + csrc, "-I" + os.path.join(ROOT, "include"),
                                     os.path.join(HERE, "sanitize", "host_container_validation.cpp"),
                                     os.path.join(csrc, "zc_container.cpp"), os.path.join(csrc, "zc_codebook.cpp"),
                                     "-x", "c", os.path.join(ROOT, "oracle", "zc_oracle.c"), "-lm"], "host_container_validation")
