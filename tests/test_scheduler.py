"""The buffer-aware scheduler and the streaming metrics (include/kvsched.h), on the CPU.

Oracle pins (oracle/sched_oracle.py against facts outside of it): Eq. 1 values, closed forms of
the reader model under constant generation rates, hand-computed reader traces, the effective-
throughput thresholds of Section 7.1, Eq. 2 arithmetic, and the timeline of the paper's motivating
example (tests/golden/toy_example_timeline.txt).  Parity: the C++ implementation must reach the
oracle's decisions on thousands of random scheduler states and reader traces (decisions are
integers: exact; weights and estimates: equal to 1e-12 relative).
"""
import math
import os

import numpy as np
import pytest

from oracle import sched_oracle as so
from paper_2510_02758_amd import kvsched as ks

HERE = os.path.dirname(os.path.abspath(__file__))

BASE = dict(mem_blocks=2, ws_blocks=1000, max_running=2, interval=1.0, gen_rate=40.0, capacity=1e9, gamma=1.0,
            safety=1.0, w_adjust=0.0, t_critical=1.0, tau_schedule=2.5, weight_tau=1e9, weight_alpha=0.0,
            evict_gbps=1e6, load_gbps=1e6, io_fixed=0.005, evict_queue=0.0, load_queue=0.0, block_bytes=1.0,
            prefill_per_token=0.0)


def both(cfg, reqs):
    rc, mode, out = ks.kv_sched_step(ks.make_config(**cfg), reqs)
    assert rc == ks.KVS_OK
    omode, oout = so.sched_step(cfg, reqs)
    assert mode == omode
    for a, b in zip(out, oout):
        assert a["decision"] == b["decision"] and a["how"] == b["how"]
        for k in ("priority_buffer", "value", "t_overhead"):
            assert a[k] == pytest.approx(b[k], rel=1e-12, abs=1e-300)
    return mode, out


def req(state, rate, buffer, arrival=0.0, blocks=1, dirty=0, tokens=16):
    return dict(state=state, arrival=arrival, rate=rate, buffer=buffer, blocks=blocks, dirty_blocks=dirty, tokens=tokens)


# ------------------------------------------------------------------ metrics pins
def test_token_weight_eq1():
    for impl in (so.token_weight, ks.kv_metric_token_weight):
        assert impl(0, 10, 0.1) == 1.0 and impl(10, 10, 0.1) == 1.0
        assert impl(15, 10, 0.1) == pytest.approx(0.5)
        assert impl(20, 10, 0.1) == pytest.approx(0.0, abs=1e-15) and impl(1000, 10, 0.1) == 0.0


@pytest.mark.parametrize("g,r", [(41.7, 20.3), (40.1, 29.7), (25.3, 24.9), (10.3, 7.1)])  # no exact ties
def test_reader_closed_form_fast_generation(g, r):
    """Generation at a constant rate g >= r: no stall; token k is read at k/r; the buffer when token j
    appears is j minus the tokens read by then."""
    L = 200
    t_gen = [j / g for j in range(L)]
    want = [j - min(j, math.floor(j * r / g) + 1) for j in range(L)]
    for buf, t_read, ttft, reb in (so.stream(t_gen, -0.5, r), ):
        assert buf == want and ttft == 0.5 and reb == 0.0
        assert t_read == pytest.approx([k / r for k in range(L)])
    rc, m = ks.kv_metric_stream(t_gen, -0.5, r)
    assert rc == 0 and m["buffer"].tolist() == want and m["ttft"] == 0.5 and m["rebuffer"] == 0.0


@pytest.mark.parametrize("g,r", [(10.0, 20.0), (3.0, 4.0)])
def test_reader_closed_form_slow_generation(g, r):
    """Generation slower than reading: every token after the first is late by 1/g - 1/r, the buffer is
    always empty."""
    L = 50
    t_gen = [2.0 + j / g for j in range(L)]
    buf, t_read, ttft, reb = so.stream(t_gen, 0.0, r)
    assert buf == [0] * L and ttft == 2.0 and t_read == pytest.approx(t_gen)
    assert reb == pytest.approx((L - 1) * (1 / g - 1 / r))
    rc, m = ks.kv_metric_stream(t_gen, 0.0, r)
    assert m["buffer"].tolist() == buf and m["rebuffer"] == pytest.approx(reb, rel=1e-12)


def test_reader_hand_trace():
    """Worked by hand: rate 2/s (one token every 0.5 s).
    generated at   0.0  0.1  0.2  0.3  2.5  2.6  4.0
    read at        0.0  0.5  1.0  1.5  2.5  3.0  4.0     (token 4 is 0.5 s late, token 6 is 0.5 s late)
    buffer         0    0    1    2    0    0    0
    """
    t_gen = [0.0, 0.1, 0.2, 0.3, 2.5, 2.6, 4.0]
    for buf, t_read, ttft, reb in (so.stream(t_gen, -1.0, 2.0),):
        assert buf == [0, 0, 1, 2, 0, 0, 0]
        assert t_read == pytest.approx([0.0, 0.5, 1.0, 1.5, 2.5, 3.0, 4.0])
        assert ttft == 1.0 and reb == pytest.approx(1.0)
    rc, m = ks.kv_metric_stream(t_gen, -1.0, 2.0)
    assert m["buffer"].tolist() == [0, 0, 1, 2, 0, 0, 0] and m["rebuffer"] == pytest.approx(1.0)


def test_effective_throughput_thresholds():
    """Section 7.1 with L = 100: full weight up to a buffer of 10, half at 15, nothing from 20 on."""
    L = 100
    buf = [0] * 50 + [10] * 10 + [15] * 10 + [20] * 10 + [60] * 20
    assert len(buf) == L
    want = 50 + 10 + 10 * 0.5 + 0 + 0
    assert so.effective_sum(buf) == pytest.approx(want)
    rc, s = ks.kv_metric_effective_sum(buf)
    assert rc == 0 and s == pytest.approx(want)


def test_qos_eq2():
    w, t, r = [100.0, 50.0], [1.0, 4.0], [0.0, 2.0]
    want = ((100 - 0.5 * 1 - 3 * 0) + (50 - 0.5 * 4 - 3 * 2)) / 20.0
    assert so.qos(w, t, r, 0.5, 3.0, 20.0) == pytest.approx(want)
    rc, q = ks.kv_metric_qos(w, t, r, 0.5, 3.0, 20.0)
    assert rc == 0 and q == pytest.approx(want)
    assert ks.kv_metric_qos(w, t, r, 0.5, 3.0, 0.0)[0] == ks.KVS_EINVAL


@pytest.mark.parametrize("seed", range(5))
def test_metrics_parity_random(seed):
    rng = np.random.default_rng(seed)
    for _ in range(60):
        L = int(rng.integers(1, 120))
        t_gen = np.cumsum(rng.exponential(0.05, size=L) * rng.choice([0.2, 1.0, 5.0], size=L))
        rate = float(rng.uniform(5, 40))
        buf, t_read, ttft, reb = so.stream(list(t_gen), -0.3, rate)
        rc, m = ks.kv_metric_stream(t_gen, -0.3, rate)
        assert rc == 0 and m["buffer"].tolist() == buf
        assert m["t_read"] == pytest.approx(t_read, rel=1e-12) and m["rebuffer"] == pytest.approx(reb, rel=1e-9, abs=1e-12)
        assert ks.kv_metric_effective_sum(buf)[1] == pytest.approx(so.effective_sum(buf), rel=1e-12)
        tau, alpha = float(rng.uniform(0, 10)), float(rng.uniform(0.01, 1))
        assert ks.kv_metric_weight_sum(buf, tau, alpha)[1] == pytest.approx(so.weight_sum(buf, tau, alpha), rel=1e-12)


# ------------------------------------------------------------------ scheduler
def _toy_timeline(step):
    """Drive one scheduler implementation through the paper's example; returns {time: running names}."""
    rate = {"R1": 20.0, "R2": 30.0, "R3": 25.0}
    arrival = {"R1": 0.0, "R2": 0.0, "R3": 2.0}
    state = {"R1": so.RUNNING, "R2": so.RUNNING}       # both start at t = 0 (two free slots)
    buf = {"R1": 0.0, "R2": 0.0}
    seen = {0: sorted(state)}
    for t in range(1, 6):
        for k in list(state):                           # one second passes
            if state[k] == so.RUNNING:
                buf[k] += BASE["gen_rate"] - rate[k]
            elif state[k] == so.PREEMPTED:
                buf[k] -= rate[k]
        if t == 2:
            state["R3"], buf["R3"] = so.NEW, 0.0
        names = sorted(state)
        reqs = [req(state[k], rate[k], buf[k], arrival[k]) for k in names]
        mode, out = step(BASE, reqs)
        for k, o in zip(names, out):
            if o["decision"] == so.RUN:
                state[k] = so.RUNNING
            elif o["decision"] == so.PREEMPT:
                state[k] = so.PREEMPTED
        seen[t] = sorted(k for k in state if state[k] == so.RUNNING)
    return seen, buf


@pytest.mark.parametrize("impl", ["oracle", "library"])
def test_motivating_example_timeline(impl):
    step = so.sched_step if impl == "oracle" else (lambda cfg, reqs: ks.kv_sched_step(ks.make_config(**cfg), reqs)[1:])
    seen, buf = _toy_timeline(step)
    want = {}
    for line in open(os.path.join(HERE, "golden", "toy_example_timeline.txt")):
        line = line.split("#")[0].split()
        if line:
            want[int(line[0])] = sorted(line[1:])
    assert seen == want
    assert buf == {"R1": 20.0, "R2": 50.0, "R3": 30.0}   # the buffers at t = 5, before the round takes effect


def test_idle_when_nothing_waits_and_nothing_is_critical():
    mode, out = both(BASE, [req(so.RUNNING, 20, 100), req(so.RUNNING, 30, 90)])
    assert mode == so.IDLE and all(o["decision"] == so.KEEP for o in out)


def test_fcfs_fallback_when_not_schedulable():
    cfg = dict(BASE, capacity=60.0, mem_blocks=3, max_running=3)
    reqs = [req(so.RUNNING, 30, 5, arrival=3.0), req(so.PREEMPTED, 30, 0, arrival=1.0), req(so.RUNNING, 30, 50, arrival=2.0),
            req(so.PREEMPTED, 30, 1, arrival=0.5, blocks=2), req(so.NEW, 30, 0, arrival=0.1)]
    mode, out = both(cfg, reqs)
    assert mode == so.FCFS
    # arrival order 3 (2 blocks), 1, 2, 0: memory of 3 blocks holds requests 3 and 1; the new one is not admitted
    assert [o["decision"] for o in out] == [so.PREEMPT, so.RUN, so.PREEMPT, so.RUN, so.KEEP]


def test_load_or_recompute():
    cfg = dict(BASE, evict_gbps=50.0, load_gbps=50.0, block_bytes=2.0 * 2**20, prefill_per_token=1e-4, io_fixed=5e-5)
    short = req(so.PREEMPTED, 20, 0, blocks=4, tokens=64)        # load 0.22 ms, recompute 6.4 ms
    long_ = req(so.PREEMPTED, 20, 0, blocks=256, tokens=4096)    # load 10.8 ms, recompute 410 ms
    mode, out = both(cfg, [short, long_])
    assert out[0]["how"] == so.BY_LOAD and out[1]["how"] == so.BY_LOAD
    cfg2 = dict(cfg, load_queue=0.05, prefill_per_token=1e-5)     # a long load queue: recomputing 64 tokens is quicker
    mode, out = both(cfg2, [short, long_])
    assert out[0]["how"] == so.BY_RECOMPUTE and out[0]["t_overhead"] == pytest.approx(64e-5)
    assert out[1]["how"] == so.BY_RECOMPUTE or out[1]["t_overhead"] == pytest.approx(0.05 + 5e-5 + 256 * 2 * 2**20 / 50e9)


def test_working_set_rule_limits_admission():
    """W_static = floor(ws_blocks / mean blocks); W_scheduled = W_static - w_adjust (W_static - N_running)."""
    reqs = [req(so.RUNNING, 20, 1000, blocks=4)] + [req(so.NEW, 20, 0, arrival=1.0 + i, blocks=4) for i in range(9)]
    cfg = dict(BASE, mem_blocks=400, max_running=64, ws_blocks=24, w_adjust=0.0)      # W_static = 6
    mode, out = both(cfg, reqs)
    assert sum(o["decision"] == so.RUN for o in out) == 5                              # 1 running + 5 admitted
    cfg = dict(cfg, w_adjust=0.4)                                                      # 6 - 0.4*(6-1) = 4
    mode, out = both(cfg, reqs)
    assert sum(o["decision"] == so.RUN for o in out) == 3
    assert [o["decision"] for o in out][1:4] == [so.RUN] * 3                           # in arrival order


def test_adjacent_swap_prefers_the_starving_request():
    """Greedy takes the emptier buffer first; if that request is slow to come back (large overhead)
    and its neighbour is about to starve, the swap pass exchanges them."""
    cfg = dict(BASE, mem_blocks=1, max_running=1, gamma=100.0, t_critical=0.0, load_queue=0.99, io_fixed=0.0)
    a = req(so.PREEMPTED, 1.0, 3.0)     # emptier, but nearly the whole interval goes into its load queue
    b = req(so.RUNNING, 30.0, 3.5)      # reads fast: starves within the interval if it is stopped
    mode, out = both(cfg, [a, b])
    assert [o["decision"] for o in out] == [so.KEEP, so.KEEP]     # b keeps running, a stays out


def _objective(cfg, reqs, s, overhead=None):
    """Section 4.2 objective of running subset s for one interval, written out from the formulation: tokens
    gained by the selected in what the context switch leaves of the interval, gamma * exp(-predicted buffer)
    charged for every candidate."""
    j = 0.0
    for i, r in enumerate(reqs):
        got = cfg["gen_rate"] * (cfg["interval"] - (overhead[i] if overhead else 0.0)) if i in s else 0.0
        j += got - cfg["gamma"] * math.exp(-max(r["buffer"] + got - r["rate"] * cfg["interval"], 0.0))
    return j


def _brute_force_best(cfg, reqs):
    """Exhaustive maximum of the objective over every feasible subset: (subset, value)."""
    import itertools
    best, best_j = None, -math.inf
    for k in range(len(reqs) + 1):
        for s in itertools.combinations(range(len(reqs)), k):
            if k > cfg["max_running"] or sum(reqs[i]["blocks"] for i in s) > cfg["mem_blocks"]:
                continue
            j = _objective(cfg, reqs, set(s))
            if j > best_j:
                best, best_j = set(s), j
    return best, best_j


@pytest.mark.parametrize("seed", range(6))
def test_selection_matches_exhaustive_search_when_greedy_is_optimal(seed):
    """Equal values and sizes, no overheads, buffers that all outlast the interval: the penalty saved by
    running a request, exp(-(b - rT)) * (1 - exp(-gT)), falls with its buffer, so the optimum is the k
    emptiest buffers, which is exactly what the priority order picks first."""
    rng = np.random.default_rng(400 + seed)
    n, k = int(rng.integers(3, 9)), int(rng.integers(1, 4))
    cfg = dict(BASE, mem_blocks=k, max_running=k + int(rng.integers(0, 2)), gamma=float(rng.uniform(0.5, 50)),
               io_fixed=0.0, t_critical=1e9)
    buffers = rng.permutation(np.arange(n)) * 0.37 + 25.0                       # distinct, all above rate * interval
    reqs = [req(int(rng.choice([so.RUNNING, so.PREEMPTED])), 20.0, float(b)) for b in buffers]
    reqs[0]["state"] = so.PREEMPTED                                             # someone is waiting: the round triggers
    mode, out = both(cfg, reqs)
    assert mode == so.BUFFER_AWARE
    chosen = {i for i, (r, o) in enumerate(zip(reqs, out))
              if o["decision"] == so.RUN or (r["state"] == so.RUNNING and o["decision"] == so.KEEP)}
    assert chosen == _brute_force_best(cfg, reqs)[0] == set(np.argsort(buffers)[:k].tolist())


def test_swap_pass_reaches_the_exhaustive_optimum_on_two_candidates():
    """With two candidates and one slot the adjacent-swap pass sees every alternative, so the decision must
    be the exhaustive optimum whichever of the two greedy took first."""
    rng = np.random.default_rng(77)
    flips = 0
    for _ in range(300):
        cfg = dict(BASE, mem_blocks=1, max_running=1, gamma=float(rng.uniform(0, 80)), io_fixed=0.0, t_critical=1e9)
        # buffers of a few tokens around rate * interval keep the two alternatives' objectives well apart
        reqs = [req(so.RUNNING, float(rng.choice([15.0, 30.0])), float(rng.uniform(10, 40))),
                req(so.PREEMPTED, float(rng.choice([15.0, 30.0])), float(rng.uniform(10, 40)))]
        mode, out = both(cfg, reqs)
        chosen = {i for i, (r, o) in enumerate(zip(reqs, out))
                  if o["decision"] == so.RUN or (r["state"] == so.RUNNING and o["decision"] == so.KEEP)}
        assert _objective(cfg, reqs, chosen) >= _brute_force_best(cfg, reqs)[1] - 1e-9
        flips += chosen != {int(np.argmin([r["buffer"] for r in reqs]))}
    assert flips > 5            # the pass did overturn greedy's choice in some of them


def test_swap_pass_weighs_the_context_switch_cost():
    """Two full buffers (no starvation either way), one slot: the waiting request would spend half the
    interval in the load queue, so keeping the running one yields twice the tokens and must win although
    the waiting one has the (slightly) emptier buffer and is taken first by the priority order."""
    cfg = dict(BASE, mem_blocks=1, max_running=1, io_fixed=0.0, load_queue=0.5, t_critical=1e9, prefill_per_token=1.0)
    reqs = [req(so.PREEMPTED, 20.0, 100.0), req(so.RUNNING, 20.0, 101.0)]
    mode, out = both(cfg, reqs)
    assert out[0]["t_overhead"] == pytest.approx(0.5, rel=1e-9) and out[0]["how"] == so.BY_LOAD
    assert [o["decision"] for o in out] == [so.KEEP, so.KEEP]
    over = [0.5, 0.0]
    assert _objective(cfg, reqs, {1}, over) > _objective(cfg, reqs, {0}, over)


@pytest.mark.parametrize("seed", range(8))
def test_scheduler_parity_random(seed):
    rng = np.random.default_rng(100 + seed)
    modes = {}
    for _ in range(250):
        n = int(rng.integers(0, 14))
        cfg = dict(BASE, mem_blocks=int(rng.integers(1, 60)), ws_blocks=int(rng.integers(1, 200)),
                   max_running=int(rng.integers(0, 8)), interval=float(rng.uniform(0.2, 1.5)),
                   gen_rate=float(rng.uniform(10, 60)), capacity=float(rng.choice([1e9, 150.0, 60.0])),
                   gamma=float(rng.uniform(0, 20)), safety=float(rng.uniform(1, 3)), w_adjust=float(rng.uniform(0, 1)),
                   t_critical=float(rng.uniform(0, 2)), tau_schedule=float(rng.uniform(0, 1)),
                   weight_tau=float(rng.uniform(0, 40)), weight_alpha=float(rng.uniform(0.01, 0.2)),
                   evict_gbps=float(rng.uniform(10, 60)), load_gbps=float(rng.uniform(10, 60)),
                   io_fixed=float(rng.uniform(0, 1e-3)), evict_queue=float(rng.uniform(0, 0.1)),
                   load_queue=float(rng.uniform(0, 0.1)), block_bytes=float(2 * 2**20),
                   prefill_per_token=float(rng.choice([0.0, 1e-5, 1e-3])))
        reqs = [req(int(rng.integers(0, 3)), float(rng.choice([15.0, 20.0, 25.0, 30.0])),
                    float(rng.choice([0.0, rng.uniform(0, 5), rng.integers(0, 200)])), arrival=float(rng.integers(0, 6)),
                    blocks=int(rng.integers(0, 20)), dirty=int(rng.integers(0, 5)), tokens=int(rng.integers(0, 4000)))
                for _ in range(n)]
        for r in reqs:
            if r["state"] == so.NEW:
                r["buffer"] = 0.0
        mode, out = both(cfg, reqs)
        modes[mode] = modes.get(mode, 0) + 1
        # invariants of any decision: memory and slots respected
        run = [i for i, o in enumerate(out) if (reqs[i]["state"] == so.RUNNING and o["decision"] == so.KEEP)
               or o["decision"] == so.RUN]
        if mode != so.IDLE:
            assert len(run) <= cfg["max_running"] and sum(reqs[i]["blocks"] for i in run) <= cfg["mem_blocks"]
    assert len(modes) == 3, modes


def test_scheduler_rejects_bad_input():
    cfg = ks.make_config(**BASE)
    assert ks.kv_sched_step(cfg, [req(7, 20, 0)])[0] == ks.KVS_EINVAL
    assert ks.kv_sched_step(cfg, [req(so.RUNNING, 0.0, 0)])[0] == ks.KVS_EINVAL
    assert ks.kv_sched_step(cfg, [req(so.RUNNING, 20, -1.0)])[0] == ks.KVS_EINVAL
    assert ks.kv_sched_step(cfg, [req(so.RUNNING, 20, float("nan"))])[0] == ks.KVS_EINVAL
    assert ks.kv_sched_step(cfg, [req(so.RUNNING, 20, 1.0, arrival=float("nan"))])[0] == ks.KVS_EINVAL
    bad = ks.make_config(**dict(BASE, interval=0.0))
    assert ks.kv_sched_step(bad, [req(so.RUNNING, 20, 1)])[0] == ks.KVS_EINVAL
    cfg.struct_size = 8
    assert ks.kv_sched_step(cfg, [req(so.RUNNING, 20, 1)])[0] == ks.KVS_EINVAL


# Pins of the oracle (everything above except the random parity sweeps), for tests/test_sched_oracle_mutants.py.
PINS = ([(test_token_weight_eq1, ())]
        + [(test_reader_closed_form_fast_generation, a) for a in [(41.7, 20.3), (40.1, 29.7), (25.3, 24.9), (10.3, 7.1)]]
        + [(test_reader_closed_form_slow_generation, a) for a in [(10.0, 20.0), (3.0, 4.0)]]
        + [(test_reader_hand_trace, ()), (test_effective_throughput_thresholds, ()), (test_qos_eq2, ()),
           (test_motivating_example_timeline, ("oracle",)), (test_idle_when_nothing_waits_and_nothing_is_critical, ()),
           (test_fcfs_fallback_when_not_schedulable, ()), (test_load_or_recompute, ()),
           (test_working_set_rule_limits_admission, ()), (test_adjacent_swap_prefers_the_starving_request, ()),
           (test_swap_pass_reaches_the_exhaustive_optimum_on_two_candidates, ()),
           (test_swap_pass_weighs_the_context_switch_cost, ())]
        + [(test_selection_matches_exhaustive_search_when_greedy_is_optimal, (k,)) for k in range(6)])
