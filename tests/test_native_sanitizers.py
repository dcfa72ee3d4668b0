"""Host components under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU, and the C ABI from plain C.

tests/native/planner_vs_oracle.cpp drives the GPU library's planner (pure C++) and the C oracle
through the same random operation sequences in one instrumented executable; tests/native/sched_stress.cpp
does the same for the scheduler and the metrics (invariants instead of an oracle: the oracle is Python);
tests/native/abi_from_c.c is a C99 client of both headers against the built library, in plan-only mode.
See their headers.
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


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_scheduler_under_sanitizers(tmp_path_factory, seed):
    out = tmp_path_factory.mktemp("sched")
    exe = str(out / "sched_stress")
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra"] + SAN +
                          ["-I", os.path.join(ROOT, "include"), "-o", exe, os.path.join(HERE, "native", "sched_stress.cpp"),
                           os.path.join(ROOT, "paper_2510_02758_amd", "csrc", "scheduler.cpp")])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe, str(seed), "3000"], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "rounds ok" in r.stdout


def test_c_abi_from_plain_c(tmp_path):
    """Both headers are valid C99 and the library can be driven from C without a GPU (KV_PLAN_ONLY)."""
    pkg = os.path.join(ROOT, "paper_2510_02758_amd")
    exe = str(tmp_path / "abi_from_c")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                           os.path.join(HERE, "native", "abi_from_c.c"), "-o", exe, "-L", pkg, "-l:libkvswap.so",
                           "-Wl,-rpath," + pkg, "-Wl,-rpath,/opt/rocm/lib"])
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "C ABI ok" in r.stdout, r.stdout + r.stderr
