"""The launches' work maps (which tile and which piece of the token axis a workgroup owns, how a Gram call is cut
into pieces, the sweep's super-block widths and far-update tiles) are plain integer logic in csrc/planner.hpp, shared
by kernels and launchers.  tests/planner_check.cpp enumerates them on the host for every supported width (d_in in
steps of 16 up to 32768, 256 compute units, token counts and workspace sizes around the plan's thresholds) and
requires that every tile, and every piece of a split tile, is owned exactly once and lies inside the matrix."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def test_work_maps_are_bijections(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no C++ compiler")
    exe = tmp_path / "planner_check"
    subprocess.run([gxx, "-O2", "-std=c++17", "-Wall", "-Wextra", "-Werror", os.path.join(HERE, "planner_check.cpp"),
                    "-o", str(exe)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
    out = r.stdout.split()
    assert out[0] == "ok" and int(out[1]) > 100000


def test_work_maps_under_sanitizers(tmp_path):
    """The same enumeration, on a thinned set of widths, built with AddressSanitizer and UBSan: the maps index
    nothing out of range and overflow no integer on the way."""
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no C++ compiler")
    exe = tmp_path / "planner_check_san"
    cmd = [gxx, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-DPLANNER_CHECK_THIN",
           os.path.join(HERE, "planner_check.cpp"), "-o", str(exe)]
    if subprocess.run(cmd, capture_output=True).returncode != 0:
        pytest.skip("sanitizer runtime not available to this compiler")
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)       # the sanitizer runtime has to come first in the link order
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.split()[0] == "ok"
