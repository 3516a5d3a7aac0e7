"""The policy generator (Algorithm 3) is host code: build it as plain C++ with the address and undefined-behaviour
sanitizers and run it over random networks (sizes 2 to 64, sparse and full graphs, feasible and infeasible)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_policy_generator_under_sanitizers(tmp_path):
    src = os.path.join(ROOT, "paper_2009_05766_amd", "csrc", "policy.hip")
    drv = os.path.join(ROOT, "tests", "policy_sanitizer_driver.cpp")
    exe = str(tmp_path / "drive")
    flags = ["-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
    subprocess.run(["g++", *flags, "-x", "c++", src, drv, "-o", exe], check=True, cwd=ROOT)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    if r.returncode != 0 and "runtime does not come first" in r.stderr:
        pytest.skip("the sanitizer runtime cannot be loaded first in this environment")
    assert r.returncode == 0, r.stderr[-2000:]
    assert "invalid 0" in r.stdout and "ERROR" not in r.stderr
