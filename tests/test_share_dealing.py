"""The dealing of a call's units to the persistent grid (host + device inline functions of the
library) checked on the CPU: the header is compiled into a small host program that walks many
(units, workers, skew) combinations and checks the properties the kernels and the merge pass
rely on.  No GPU, no oracle: this is host logic of the product."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(os.path.dirname(HERE), "paper_2405_01814_amd", "csrc")


def test_shares_cover_the_stream_and_owners_match(tmp_path):
    cxx = shutil.which("g++") or shutil.which("c++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "share_dealing_check")
    build = subprocess.run([cxx, "-std=c++17", "-O2", "-Wall", "-Wextra", "-Werror",
                            "-fsanitize=undefined", "-fno-sanitize-recover=all", "-I", CSRC,
                            os.path.join(HERE, "share_dealing_check.cpp"), "-o", exe],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stdout + build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.startswith("ok "), run.stdout
    assert int(run.stdout.split()[1]) > 10000
