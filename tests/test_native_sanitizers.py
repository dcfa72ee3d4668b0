"""Host components under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU, and the C ABI from plain C.

tests/native/planner_vs_oracle.cpp drives the GPU library's planner (pure C++) and the C oracle
through the same random operation sequences in one instrumented executable; tests/native/sched_stress.cpp
does the same for the scheduler and the metrics (invariants instead of an oracle: the oracle is Python);
tests/native/abi_from_c.c is a C99 client of both headers against the built library, in plan-only mode;
tests/native/runtime_on_mock_hip.cpp runs the library's host runtime and its kernel source, unchanged, on a
host-only stand-in for the HIP runtime (tests/native/mockhip) whose executor decides which stream lags, and
compares random serving histories with the oracle; the same driver injects HIP errors and allocation failures,
and runs with a second thread under ThreadSanitizer.  See their headers.
"""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
# stack-use-after-return detection gives every fiber of the stand-in's workgroups a fake stack of its own (an mmap
# each): switched off, or a launch of a thousand workgroups takes seconds
ASAN_OPTS = "detect_leaks=1:abort_on_error=0:detect_stack_use_after_return=0"
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
    env = dict(os.environ, ASAN_OPTIONS=ASAN_OPTS, UBSAN_OPTIONS="print_stacktrace=1")
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
    env = dict(os.environ, ASAN_OPTIONS=ASAN_OPTS, UBSAN_OPTIONS="print_stacktrace=1")
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


# ---- the real runtime and the real kernel source on a stand-in HIP runtime, on the CPU ----
CLANGXX = os.environ.get("HOST_CLANGXX", "/opt/rocm/llvm/bin/clang++")   # the kernel source uses clang builtins
CSRC = os.path.join(ROOT, "paper_2510_02758_amd", "csrc")
MOCK = os.path.join(HERE, "native", "mockhip")


_COMMON = {}   # flags -> objects of everything but the library: built once per flag set


def _common_objects(flags):
    key = tuple(flags)
    if key not in _COMMON:
        import tempfile
        from concurrent.futures import ThreadPoolExecutor
        d = tempfile.mkdtemp(prefix="mockhip_obj_")
        jobs = [(["gcc", "-std=c99", "-c"] + flags, os.path.join(ROOT, "oracle", "kv_oracle.c"), os.path.join(d, "kv_oracle.o"))]
        for src in (os.path.join(MOCK, "mockhip.cpp"), os.path.join(HERE, "native", "runtime_on_mock_hip.cpp")):
            jobs.append(([CLANGXX, "-std=c++17", "-Wall", "-pthread", "-c"] + flags +
                         ["-I", MOCK, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "native")],
                         src, os.path.join(d, os.path.basename(src) + ".o")))
        with ThreadPoolExecutor(max_workers=len(jobs)) as pool:     # three translation units, three compilers
            list(pool.map(lambda j: subprocess.check_call(j[0] + [j[1], "-o", j[2]]), jobs))
        _COMMON[key] = [j[2] for j in jobs]
    return _COMMON[key]


def _build_on_mock(out_dir, name, csrc_dir, flags):
    from concurrent.futures import ThreadPoolExecutor
    exe = os.path.join(out_dir, name)
    lib = os.path.join(out_dir, name + "_kvswap.o")
    with ThreadPoolExecutor(max_workers=1) as pool:   # the library compiles while the common objects do (if they still have to)
        compiling = pool.submit(subprocess.check_call, [CLANGXX, "-std=c++17", "-Wall", "-pthread", "-c"] + flags +
                                ["-I", MOCK, "-I", os.path.join(ROOT, "include"), "-x", "c++",
                                 os.path.join(csrc_dir, "kvswap.hip"), "-o", lib])
        common = _common_objects(flags)
        compiling.result()
    subprocess.check_call([CLANGXX, "-pthread"] + flags + [lib] + common + ["-o", exe])
    return exe


@pytest.fixture(scope="module")
def mock_driver(tmp_path_factory):
    if not os.path.exists(CLANGXX):
        pytest.skip("no host clang++ for the kernel source")
    return _build_on_mock(str(tmp_path_factory.mktemp("mockhip")), "runtime_on_mock_hip", CSRC, SAN)


@pytest.mark.parametrize("first", [0, 48, 96, 144])
def test_runtime_and_kernels_on_the_stand_in_hip_runtime(mock_driver, first):
    """Seeds first .. first+47 cover every geometry x padding x path x events combination under one lag policy
    (0: random progress, 48: the evict stream starved, 96: the load stream starved, 144: nothing runs until a wait)."""
    env = dict(os.environ, ASAN_OPTIONS=ASAN_OPTS, UBSAN_OPTIONS="print_stacktrace=1")
    for seed in range(first, first + 48):
        r = subprocess.run([mock_driver, str(seed), "6"], capture_output=True, text=True, timeout=300, env=env)
        assert r.returncode == 0, "seed %d\n%s%s" % (seed, r.stdout[-2000:], r.stderr[-4000:])
        assert "equal to the oracle" in r.stdout


def test_kernel_arithmetic_on_geometries_nobody_wrote_down(mock_driver):
    """Seeds from 192 on draw L, H, D, B, element size, scales and the kernel's unroll variant at random (chunks of 16
    bytes to 20 KiB): every access of every lane of the real kernel source stays inside its buffers (AddressSanitizer)
    and the bytes equal the oracle's."""
    env = dict(os.environ, ASAN_OPTIONS=ASAN_OPTS, UBSAN_OPTIONS="print_stacktrace=1")
    for seed in range(192, 288):
        r = subprocess.run([mock_driver, str(seed), "4"], capture_output=True, text=True, timeout=300, env=env)
        assert r.returncode == 0, "seed %d\n%s%s" % (seed, r.stdout[-2000:], r.stderr[-4000:])
        assert "equal to the oracle" in r.stdout


@pytest.mark.parametrize("what", ["hipfail", "nomem"])
def test_a_failure_inside_a_call_leaves_a_handle_that_refuses_work_and_can_be_destroyed(mock_driver, what):
    """hipfail: some HIP call made by the library returns an error; nomem: some allocation made while a library
    call runs throws.  No exception leaves the C boundary, the call returns KV_EHIP / KV_ENOMEM, every later call
    that would change state returns KV_EHIP, queries still answer, kv_pool_destroy releases every event and
    buffer (LeakSanitizer); a failure the library can absorb leaves the history equal to the oracle."""
    env = dict(os.environ, ASAN_OPTIONS=ASAN_OPTS, UBSAN_OPTIONS="print_stacktrace=1")
    handled = 0
    for seed in range(0, 96):
        r = subprocess.run([mock_driver, str(seed), "4", what], capture_output=True, text=True, timeout=300, env=env)
        assert r.returncode == 0, "seed %d\n%s%s" % (seed, r.stdout[-2000:], r.stderr[-4000:])
        assert "equal to the oracle" in r.stdout or "failure handled" in r.stdout
        handled += "failure handled" in r.stdout
    assert handled >= 40, handled


# One ordering rule of the runtime is taken out at a time (in a copy of the sources); the same histories must then
# end in a byte difference for some seed: the harness above is able to see what it is meant to see.
RUNTIME_MUTANTS = [
    ("reserved_extent_forgets_the_pending_reader",
     "  if (dep)\n    if (kvswap::Req* r = p->planner.find_mut(req_id)) r->in_seq = dep;\n", "  (void)dep;\n"),
    ("device_block_hazards_off", "  if (p->blk_reader.empty() || n == 0) return nullptr;", "  return nullptr;"),
    ("staging_slot_waits_off", "  if (wait_seq) {", "  if (false && wait_seq) {"),
    ("callers_event_ignored", "  if (wait_event) HIPCHK(p, hipStreamWaitEvent(st, (hipEvent_t)wait_event, 0));", ""),
    ("stale_error_of_the_application_taken_for_a_failed_launch",
     "  (void)hipGetLastError();\n  const bool pipe = kind != 1 && pipelined_variant(p);",
     "  const bool pipe = kind != 1 && pipelined_variant(p);"),
    ("newest_call_hides_the_other_stream",
     "s = std::max(s, cross_stream(p, stream, q.seq));", "s = std::max(s, q.seq);"),
    ("allocation_free_move_not_ordered_after_the_load_stream",
     "  HIPCHK(p, hipStreamWaitEvent(st, p->na_fence_ev, 0));", ""),
    ("load_stream_does_not_wait_for_an_allocation_free_move",
     "      HIPCHK(p, hipStreamWaitEvent(st, p->na_done_ev, 0));", ""),
    ("load_phase_forgets_the_eviction_phase_that_frees_its_blocks",
     "    if (it != reader.end()) need[i / m] = std::max(need[i / m], it->second);", "    (void)it;"),
    ("write_through_that_moves_nothing_forgets_the_pending_reader",
     "        if (kvswap::Req* r = p->planner.find_mut(id)) r->in_seq = std::max(r->in_seq, fresh_dep);", "        (void)id;"),
]


def _mutated_sources(tmp_path, name, find, repl):
    import shutil
    src = tmp_path / "csrc"
    shutil.copytree(CSRC, src)
    hits = 0
    for f in ("runtime.hip.inc", "kvswap.hip", "kernels.hip.inc"):
        text = open(src / f).read()
        hits += text.count(find)
        open(src / f, "w").write(text.replace(find, repl))
    assert hits == 1, "mutation site of %s found %d times" % (name, hits)
    # planner.hpp names the public header by a relative path: keep that path valid for the copy
    text = open(src / "planner.hpp").read().replace('"../../include/kvswap.h"', '"kvswap.h"')
    open(src / "planner.hpp", "w").write(text)
    return str(src)


@pytest.mark.parametrize("name,find,repl", RUNTIME_MUTANTS, ids=[m[0] for m in RUNTIME_MUTANTS])
def test_a_missing_ordering_rule_is_noticed(name, find, repl):
    if not os.path.exists(CLANGXX):
        pytest.skip("no host clang++ for the kernel source")
    exe = _mutant_exe(name)
    failed_at = None
    for seed in range(48, 400):
        r = subprocess.run([exe, str(seed), "6"], capture_output=True, text=True, timeout=300)
        if r.returncode != 0:
            assert "MISMATCH" in r.stderr, r.stderr[-2000:]
            failed_at = seed
            break
    assert failed_at is not None, "no history notices the planted mistake '%s'" % name


# The same for the kernels' arithmetic: a planted mistake in the kernel source must show as a byte difference (or
# end the process, where it sends a store far outside every buffer).
KERNEL_MUTANTS = [
    ("ragged_last_piece_not_clipped", "        const int mine = left - lane0;", "        const int mine = left;"),
    ("k_and_v_planes_swapped", "      const int64_t plane = (int64_t)(k >> 1) * a.ls + (int64_t)(k & 1) * a.ks;",
     "      const int64_t plane = (int64_t)(k >> 1) * a.ls + (int64_t)((k & 1) ^ 1) * a.ks;"),
    ("small_chunks_k_and_v_planes_swapped", "  auto plane_of = [&](int k) { return (int64_t)(k >> 1) * a.ls + (int64_t)(k & 1) * a.ks; };",
     "  auto plane_of = [&](int k) { return (int64_t)(k >> 1) * a.ls + (int64_t)((k & 1) ^ 1) * a.ks; };"),
    ("scale_jobs_launched_from_the_wrong_job", "    side.first_job = a.n_data_jobs;", "    side.first_job = a.n_data_jobs + 1;"),
    ("plane_by_plane_scatter_in_the_wrong_plane", "        k = (int)(job / a.per_plane);", "        k = (int)(job / a.per_plane) ^ 1;"),
    ("half_the_scale_vectors", "      const int vecs = a.scale_words >> 2;", "      const int vecs = a.scale_words >> 3;"),
    ("staging_slot_of_the_wrong_block", "        dst = a.contig + (int64_t)(uint32_t)ds.b * a.S + (int64_t)k * a.chunk;",
     "        dst = a.contig + (int64_t)(uint32_t)ds.a * a.S + (int64_t)k * a.chunk;"),
]


_MUTANT_EXES = {}   # name -> path of the executable, or the exception its build raised


def _mutant_exe(name):
    """All mutants are built on first use, several compilers at a time (one translation unit each, seconds apiece)."""
    if not _MUTANT_EXES:
        import pathlib
        import tempfile
        from concurrent.futures import ThreadPoolExecutor
        top = pathlib.Path(tempfile.mkdtemp(prefix="mockhip_mutants_"))
        _common_objects(["-O1"])      # once, before the workers would race for it

        def build(m):
            d = top / m[0]
            d.mkdir()
            try:
                return m[0], _build_on_mock(str(d), "mutant", _mutated_sources(d, *m), ["-O1"])
            except Exception as e:    # reported by the test of this mutant, not by whichever test came first
                return m[0], e
        with ThreadPoolExecutor(max_workers=max(1, min(6, os.cpu_count() or 1))) as pool:
            _MUTANT_EXES.update(pool.map(build, RUNTIME_MUTANTS + KERNEL_MUTANTS))
    exe = _MUTANT_EXES[name]
    if isinstance(exe, Exception):
        raise exe
    return exe


@pytest.mark.parametrize("name,find,repl", KERNEL_MUTANTS, ids=[m[0] for m in KERNEL_MUTANTS])
def test_a_mistake_in_the_kernel_arithmetic_is_noticed(name, find, repl):
    if not os.path.exists(CLANGXX):
        pytest.skip("no host clang++ for the kernel source")
    exe = _mutant_exe(name)
    for seed in list(range(0, 48)) + list(range(192, 240)):
        r = subprocess.run([exe, str(seed), "4"], capture_output=True, text=True, timeout=300)
        if r.returncode != 0:   # a byte difference, or the wild access ended the process
            assert "MISMATCH" in r.stderr or r.returncode < 0, r.stderr[-2000:]
            return
    raise AssertionError("no history notices the planted mistake '%s'" % name)


# ---- the same harness under ThreadSanitizer, with a second thread that polls the handle ----
TSAN = ["-fsanitize=thread", "-g", "-O1"]


def test_entry_points_from_two_threads_under_tsan(tmp_path):
    """A reader thread (kv_req_poll / kv_req_wait / kv_req_query / kv_io_stats_get / kv_last_stats / kv_wq_pending)
    runs beside the serving history: no data race, and the history still ends equal to the oracle."""
    if not os.path.exists(CLANGXX):
        pytest.skip("no host clang++ for the kernel source")
    exe = _build_on_mock(str(tmp_path), "runtime_tsan", CSRC, TSAN)
    for seed in range(0, 192, 8):
        r = subprocess.run([exe, str(seed + seed // 8 % 4), "4", "poller"], capture_output=True, text=True, timeout=300)
        assert r.returncode == 0, "seed %d\n%s%s" % (seed, r.stdout[-2000:], r.stderr[-4000:])
        assert "equal to the oracle" in r.stdout


def test_tsan_notices_an_entry_point_without_the_lock(tmp_path):
    if not os.path.exists(CLANGXX):
        pytest.skip("no host clang++ for the kernel source")
    import shutil
    src = tmp_path / "csrc"
    shutil.copytree(CSRC, src)
    text = open(src / "kvswap.hip").read()
    at = text.index("int kv_req_query(")
    lock = "std::lock_guard<std::mutex> g(p->mu);"
    at = text.index(lock, at)
    open(src / "kvswap.hip", "w").write(text[:at] + text[at + len(lock):])
    text = open(src / "planner.hpp").read().replace('"../../include/kvswap.h"', '"kvswap.h"')
    open(src / "planner.hpp", "w").write(text)
    exe = _build_on_mock(str(tmp_path), "mutant_tsan", str(src), TSAN)
    for seed in range(0, 64):
        r = subprocess.run([exe, str(seed), "4", "poller"], capture_output=True, text=True, timeout=300)
        if r.returncode != 0:
            assert "ThreadSanitizer: data race" in r.stderr, r.stderr[-3000:]
            return
    raise AssertionError("the unlocked kv_req_query was not reported")
