"""Host sanitizer run of the C oracle: oracle/tbn_oracle.c and tests/oracle_sanitize_driver.c are compiled with
AddressSanitizer and UndefinedBehaviorSanitizer and the driver's pins (the hand-worked example of
tests/golden/hand_worked_pack.txt, agreement of the oracle's independent code paths on ragged shapes) run on heap
buffers of exactly the documented sizes."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCES = [os.path.join(ROOT, "oracle", "tbn_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitize_driver.c")]
FLAGS = ["-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra"]


def _build(tmp_path, name, extra=()):
    exe = str(tmp_path / name)
    res = subprocess.run(["gcc", *FLAGS, *extra, *SOURCES, "-lm", "-o", exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return exe


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="2")
    return subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)


def test_oracle_pins_under_address_and_undefined_sanitizers(tmp_path):
    res = _run(_build(tmp_path, "oracle_san"))
    assert res.returncode == 0 and "ok" in res.stdout, res.stdout + res.stderr


def test_sanitizer_build_sees_a_planted_overrun(tmp_path):
    # the same driver with a tile buffer one word short: the run must not pass silently
    res = _run(_build(tmp_path, "oracle_san_planted", ["-DPLANT_SHORT_TILE"]))
    assert res.returncode != 0 and "heap-buffer-overflow" in res.stderr, res.stdout + res.stderr
