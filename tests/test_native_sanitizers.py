"""Host components under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU.

tests/native/planner_vs_oracle.cpp drives the GPU library's planner (pure C++) and the C oracle
through the same random operation sequences in one instrumented executable; see its header.
"""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("native")
    obj = str(out / "kv_oracle.o")
    exe = str(out / "planner_vs_oracle")
    subprocess.check_call(["gcc", "-std=c99", "-c"] + SAN + ["-o", obj, os.path.join(ROOT, "oracle", "kv_oracle.c")])
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra"] + SAN +
                          ["-o", exe, os.path.join(HERE, "native", "planner_vs_oracle.cpp"), obj])
    return exe


@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5, 6])
def test_planner_and_oracle_agree_under_sanitizers(driver, seed):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([driver, str(seed), "4000"], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "calls agreed" in r.stdout
