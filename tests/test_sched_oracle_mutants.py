"""Are the scheduler oracle's pins sharp?  Plant one plausible mistake at a time in a copy of
oracle/sched_oracle.py (a dropped term, a flipped comparison, a wrong sort key, a forgotten rule) and
require that at least one pin of test_scheduler.py fails on it.  CPU only; the mutated source is compiled
into a module object of its own and the pins run against it instead of the real oracle (the comparison
with the C++ library is switched off for that run: a mutant must be caught by the paper's facts alone).
"""
import os
import types

import pytest

import test_scheduler as T

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "sched_oracle.py")

# (name, text to find, replacement)
MUTANTS = [
    ("weight_threshold_strict", "    if B <= tau:\n        return 1.0", "    if B < tau:\n        return 1.0 - alpha"),
    ("weight_not_clamped", "return max(1.0 - alpha * (B - tau), 0.0)", "return 1.0 - alpha * (B - tau)"),
    ("weight_slope_dropped", "return max(1.0 - alpha * (B - tau), 0.0)", "return max(1.0 - alpha * B, 0.0)"),
    ("reader_never_waits", "            t_read.append(t_gen[j])\n        else:", "            t_read.append(due)\n        else:"),
    ("reader_ignores_pace", "        else:\n            t_read.append(due)", "        else:\n            t_read.append(t_gen[j])"),
    ("rebuffer_counts_first_token", "t_read, rebuffer = [], 0.0", "t_read, rebuffer = [], (t_gen[0] if t_gen else 0.0)"),
    ("buffer_counts_own_token", "for k in range(j):            # tokens", "for k in range(j + 1):            # tokens"),
    ("buffer_read_test_inverted", "if t_read[k] > t_gen[j]:", "if t_read[k] <= t_gen[j]:"),
    ("ttft_from_zero", "ttft = (t_gen[0] - t_arrival) if L else 0.0", "ttft = t_gen[0] if L else 0.0"),
    ("effective_threshold_20", "tau1 = 0.1 * L", "tau1 = 0.2 * L"),
    ("effective_no_decay", "return weight_sum(buffer, tau1, 1.0 / tau1)", "return weight_sum(buffer, tau1, 0.0)"),
    ("qos_lambda_mu_swapped", "s += w - lam * t - mu * r", "s += w - mu * t - lam * r"),
    ("qos_penalty_sign", "s += w - lam * t - mu * r", "s += w + lam * t + mu * r"),
    ("qos_not_normalised", "    return s / T", "    return s"),
    ("recompute_never", "if t_re < t_io:", "if False:"),
    ("recompute_always", "if t_re < t_io:", "if True:"),
    ("load_queue_forgotten", '+ cfg["load_queue"] + tl', "+ tl"),
    ("overhead_not_charged", 'tp = max(cfg["interval"] - overhead, 0.0)', 'tp = cfg["interval"]'),
    ("trigger_ignores_waiting", "waiting = bool(preempted or fresh)", "waiting = False"),
    ("trigger_always", "if not waiting and not critical:", "if False:"),
    ("schedulable_test_dropped", 'if ws_rate > cfg["capacity"]:', "if False:"),
    ("fcfs_by_index", 'key=lambda i: (reqs[i]["arrival"], i))\n        sel, used = set(), 0', "key=lambda i: i)\n        sel, used = set(), 0"),
    ("w_static_ceil", 'w_static = math.floor(cfg["ws_blocks"] / max(beta, 1.0))', 'w_static = math.ceil(cfg["ws_blocks"] / max(beta, 1.0)) + 1'),
    ("w_adjust_ignored", 'w_sched = w_static - cfg["w_adjust"] * (w_static - n_run) if n_run < w_static else w_static', "w_sched = w_static"),
    ("safety_test_dropped", 'if r["buffer"] >= cfg["safety"] * r["rate"] * (t_evict[i] + t_load[i] + cfg["tau_schedule"]):', "if True:"),
    ("tau_schedule_forgotten", '(t_evict[i] + t_load[i] + cfg["tau_schedule"])', "(t_evict[i] + t_load[i])"),
    ("admit_latest_first", 'for i in sorted(fresh, key=lambda i: (reqs[i]["arrival"], i)):', 'for i in sorted(fresh, key=lambda i: (-reqs[i]["arrival"], i)):'),
    ("fullest_buffer_first", 'key=lambda i: (reqs[i]["buffer"], -value[i]', 'key=lambda i: (-reqs[i]["buffer"], -value[i]'),
    ("memory_limit_ignored", 'if len(sel) < cfg["max_running"] and used + reqs[i]["blocks"] <= cfg["mem_blocks"]:\n            sel.add(i)\n            used += reqs[i]["blocks"]\n\n    def objective',
     'if len(sel) < cfg["max_running"]:\n            sel.add(i)\n            used += reqs[i]["blocks"]\n\n    def objective'),
    ("penalty_only_for_selected", "            pen += math.exp(-max(b, 0.0))", "            pen += math.exp(-max(b, 0.0)) if i in s else 0.0"),
    ("gain_sign", "                gain += value[i]", "                gain -= value[i]"),
    ("drain_forgotten", 'b = reqs[i]["buffer"] - reqs[i]["rate"] * cfg["interval"]', 'b = reqs[i]["buffer"]'),
    ("swap_pass_dropped", "if objective(trial) > objective(sel) + 1e-12:", "if False:"),
    ("running_unselected_kept", 'out[i]["decision"] = KEEP if i in selected else PREEMPT', 'out[i]["decision"] = KEEP'),
]


def _mutant(find, repl):
    src = open(SRC).read()
    assert src.count(find) == 1, "mutation site not found exactly once: %r" % find
    mod = types.ModuleType("sched_oracle_mutant")
    exec(compile(src.replace(find, repl), "sched_oracle_mutant", "exec"), mod.__dict__)
    return mod


def _run_pins(mod):
    """Name of the first pin that fails against `mod`, or None."""
    saved = T.so, T.both
    T.so, T.both = mod, (lambda cfg, reqs: mod.sched_step(cfg, reqs))
    try:
        for fn, args in T.PINS:
            try:
                fn(*args)
            except Exception:
                return fn.__name__
        return None
    finally:
        T.so, T.both = saved


def test_the_real_oracle_passes_every_pin():
    src = open(SRC).read()
    mod = types.ModuleType("sched_oracle_copy")
    exec(compile(src, "sched_oracle_copy", "exec"), mod.__dict__)
    assert _run_pins(mod) is None


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, find, repl):
    assert _run_pins(_mutant(find, repl)) is not None, "no pin notices the planted mistake '%s'" % name
