"""The host-side work decomposition (csrc/dppf_walk.h: tile lists, the split of the tiles over
thread blocks, the walk a block makes, the on-demand counter) compiled with a plain host compiler
and AddressSanitizer + UndefinedBehaviorSanitizer, one host thread per simulated thread block: every
work item visited exactly once, every row of partial sums written exactly once, counter back at zero."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_walk_simulation_under_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    exe = tmp_path / "walk_sim"
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-static-libubsan", "-pthread",
           "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "paper_2507_20424_amd", "csrc"),
           os.path.join(ROOT, "tests", "host", "walk_sim.cpp"), "-o", str(exe)]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    res = subprocess.run([str(exe), "400"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300,
                         env=env)
    assert res.returncode == 0, res.stdout
    assert "all checks passed" in res.stdout
