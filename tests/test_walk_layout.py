"""Launch arithmetic of the level-walk kernels, on the host: the LDS layouts they carve
(csrc/lc_walk_layout.h) are enumerated over every shape the launchers can produce by a small C++
program built with the host compiler, and the limits the library reports are the layout's."""
import os
import subprocess

import pytest

from paper_2603_08453_amd import binding as lc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_walk_layouts_over_every_launch_shape(tmp_path):
    exe = tmp_path / "walk_layout_check"
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Werror", "-I",
                    os.path.join(ROOT, "paper_2603_08453_amd", "csrc"),
                    os.path.join(ROOT, "tests", "cpp", "walk_layout_check.cpp"), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.startswith("ok "), out.stdout + out.stderr
    assert int(out.stdout.split()[1]) > 10000


def test_reported_limits_match_the_layout():
    L = lc.lib()
    L.lc_walk_limits.argtypes = [lc.ctypes.POINTER(lc.ctypes.c_int32), lc.ctypes.POINTER(lc.ctypes.c_int32)]
    L.lc_walk_limits.restype = None
    exact, beam = lc.ctypes.c_int32(), lc.ctypes.c_int32()
    L.lc_walk_limits(lc.ctypes.byref(exact), lc.ctypes.byref(beam))
    # 13 bytes per node slot + 16 per staging slot (>= node slots) + 12 per probe slot (>= 64) within 150 KiB
    assert 5000 <= exact.value <= 5400 and exact.value % 64 == 0
    assert 13 * exact.value + 16 * exact.value + 12 * 64 <= 150 * 1024 < 29 * (exact.value + 64) + 12 * 64
    assert beam.value == 65536
