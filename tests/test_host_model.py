"""Host model of the decode kernel's schedule and hand-out of work items (one OS thread per wavefront, the kernel's
own schedule header): built with the host C++ compiler and run on the CPU.  See
tests/host_model/decode_schedule.cpp for what it checks."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "host_model", "decode_schedule.cpp")
INC = os.path.join(ROOT, "paper_2502_15294_amd", "csrc")


def _build(tmp_path, name, *defines):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / name)
    r = subprocess.run([gxx, "-std=c++17", "-O1", "-Wall", "-Werror", "-pthread", *defines, "-I", INC, SRC, "-o", exe],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_every_wave_exits_every_tile_streamed_once_every_cut_sequence_has_its_records(tmp_path, seed):
    exe = _build(tmp_path, "model")
    r = subprocess.run([exe, str(seed), "150"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr


@pytest.mark.parametrize("plant", ["-DPLANT_SKIP_LAST_ITEM", "-DPLANT_RECORD_BY_RANGE"])
def test_the_model_fails_when_a_mistake_is_planted(tmp_path, plant):
    exe = _build(tmp_path, "planted", plant)
    r = subprocess.run([exe, "1", "150"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 1, "the planted mistake went unnoticed:\n" + r.stdout + r.stderr
