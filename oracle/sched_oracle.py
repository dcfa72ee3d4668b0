"""Plain-Python oracle of the buffer-aware scheduler and the streaming metrics.
TEST INFRASTRUCTURE ONLY: imported by tests, never by the product path; shares no code with
paper_2510_02758_amd/csrc/scheduler.cpp.

Each function restates, in the order the paper gives them, the rules of
  * Section 3.2: reader model, token weight (Eq. 1), QoS (Eq. 2);
  * Section 7.1: effective throughput (10 % / 20 % of the output length);
  * Section 4.2: working set (W_static, W_scheduled), admission test, priority order
    (phi(b) = exp(-b), v*t', r), greedy selection with one pass of adjacent swaps,
    load-or-recompute (t_IO against the prefill estimate);
  * Section 4.3: schedulability test and FCFS fallback.
Where the paper leaves a detail open the reading is the one documented for kv_sched_step.

Parity status: pinned by tests/test_scheduler.py — closed forms for the metrics, hand-computed
reader traces, exhaustive search over every feasible subset on tiny inputs for the selection, and
the timeline of the paper's motivating example (Section 4.1), which the scheduler must reproduce
decision by decision.  tests/test_sched_oracle_mutants.py plants one mistake at a time in a copy of
this file and requires a pin to notice each.
"""
import math

NEW, RUNNING, PREEMPTED = 0, 1, 2
KEEP, RUN, PREEMPT = 0, 1, 2
BY_LOAD, BY_RECOMPUTE = 0, 1
IDLE, BUFFER_AWARE, FCFS = 0, 1, 2


# ------------------------------------------------------------------ metrics
def token_weight(B, tau, alpha):
    """Eq. 1."""
    if B <= tau:
        return 1.0
    return max(1.0 - alpha * (B - tau), 0.0)


def stream(t_gen, t_arrival, rate):
    """Reader of Section 3.2: starts at the first token, one token every 1/rate seconds, waits when
    the next token is late.  Returns (buffer, t_read, ttft, rebuffer)."""
    L = len(t_gen)
    t_read, rebuffer = [], 0.0
    for j in range(L):
        if j == 0:
            t_read.append(t_gen[0])
            continue
        due = t_read[j - 1] + 1.0 / rate
        if t_gen[j] > due:
            rebuffer += t_gen[j] - due
            t_read.append(t_gen[j])
        else:
            t_read.append(due)
    buffer = []
    for j in range(L):
        unread = 0
        for k in range(j):            # tokens generated before j ...
            if t_read[k] > t_gen[j]:  # ... and not read by the time token j appears
                unread += 1
        buffer.append(unread)
    ttft = (t_gen[0] - t_arrival) if L else 0.0
    return buffer, t_read, ttft, rebuffer


def weight_sum(buffer, tau, alpha):
    s = 0.0
    for B in buffer:
        s += token_weight(float(B), tau, alpha)
    return s


def effective_sum(buffer):
    """Section 7.1: full weight below 10 % of the output length, linear to zero at 20 %."""
    L = len(buffer)
    if L == 0:
        return 0.0
    tau1 = 0.1 * L
    return weight_sum(buffer, tau1, 1.0 / tau1)


def qos(weight_sums, ttfts, rebuffers, lam, mu, T):
    """Eq. 2."""
    s = 0.0
    for w, t, r in zip(weight_sums, ttfts, rebuffers):
        s += w - lam * t - mu * r
    return s / T


# ---------------------------------------------------------------- scheduler
def sched_step(cfg, reqs):
    """cfg: dict with the kv_sched_config fields; reqs: list of dicts with the kv_sched_req fields.
    Returns (mode, list of dict(decision, how, priority_buffer, value, t_overhead))."""
    n = len(reqs)
    out = []
    t_evict, t_load, tprime, value = [], [], [], []
    for r in reqs:
        te = cfg["io_fixed"] + r["dirty_blocks"] * cfg["block_bytes"] / (cfg["evict_gbps"] * 1e9) if r["dirty_blocks"] > 0 else 0.0
        tl = cfg["io_fixed"] + r["blocks"] * cfg["block_bytes"] / (cfg["load_gbps"] * 1e9)
        overhead, how = 0.0, BY_LOAD
        if r["state"] == PREEMPTED:
            t_io = ((cfg["evict_queue"] + te) if r["dirty_blocks"] > 0 else 0.0) + cfg["load_queue"] + tl
            t_re = r["tokens"] * cfg["prefill_per_token"]
            if t_re < t_io:
                overhead, how = t_re, BY_RECOMPUTE
            else:
                overhead = t_io
        elif r["state"] == NEW:
            overhead = r["tokens"] * cfg["prefill_per_token"]
        tp = max(cfg["interval"] - overhead, 0.0)
        v = cfg["gen_rate"] * token_weight(r["buffer"], cfg["weight_tau"], cfg["weight_alpha"]) * tp
        t_evict.append(te)
        t_load.append(tl)
        tprime.append(tp)
        value.append(v)
        out.append(dict(decision=KEEP, how=how, priority_buffer=math.exp(-r["buffer"]), value=v, t_overhead=overhead))

    running = [i for i in range(n) if reqs[i]["state"] == RUNNING]
    preempted = [i for i in range(n) if reqs[i]["state"] == PREEMPTED]
    fresh = [i for i in range(n) if reqs[i]["state"] == NEW]
    waiting = bool(preempted or fresh)
    critical = any(reqs[i]["buffer"] / reqs[i]["rate"] < cfg["t_critical"] for i in running)
    if not waiting and not critical:
        return IDLE, out

    def finish(mode, selected):
        for i in range(n):
            if reqs[i]["state"] == RUNNING:
                out[i]["decision"] = KEEP if i in selected else PREEMPT
            else:
                out[i]["decision"] = RUN if i in selected else KEEP
        return mode, out

    # Section 4.3: the working set must be schedulable, else first come first served
    ws_rate = 0.0
    for i in range(n):
        if reqs[i]["state"] != NEW:
            ws_rate += reqs[i]["rate"]
    if ws_rate > cfg["capacity"]:
        order = sorted(running + preempted, key=lambda i: (reqs[i]["arrival"], i))
        sel, used = set(), 0
        for i in order:
            if len(sel) < cfg["max_running"] and used + reqs[i]["blocks"] <= cfg["mem_blocks"]:
                sel.add(i)
                used += reqs[i]["blocks"]
        return finish(FCFS, sel)

    # working set size
    beta = sum(float(r["blocks"]) for r in reqs) / n if n else 1.0
    w_static = math.floor(cfg["ws_blocks"] / max(beta, 1.0))
    n_run = len(running)
    w_sched = w_static - cfg["w_adjust"] * (w_static - n_run) if n_run < w_static else w_static
    # admission: a new request needs a slot and memory, or a running request that can afford a round trip
    safe = 0
    for i in running:
        r = reqs[i]
        if r["buffer"] >= cfg["safety"] * r["rate"] * (t_evict[i] + t_load[i] + cfg["tau_schedule"]):
            safe += 1
    free_blocks = cfg["mem_blocks"] - sum(reqs[i]["blocks"] for i in running)
    free_slots = cfg["max_running"] - n_run
    w_current = n_run + len(preempted)
    admitted = []
    for i in sorted(fresh, key=lambda i: (reqs[i]["arrival"], i)):
        if not (w_current < w_sched):
            break
        if free_slots > 0 and reqs[i]["blocks"] <= free_blocks:
            free_slots -= 1
            free_blocks -= reqs[i]["blocks"]
        elif safe > 0:
            safe -= 1
        else:
            continue
        admitted.append(i)
        w_current += 1

    # buffer balancing: emptiest buffer first, then weighted tokens, then rate
    cand = sorted(running + preempted + admitted,
                  key=lambda i: (reqs[i]["buffer"], -value[i], -reqs[i]["rate"], i))
    sel, used = set(), 0
    for i in cand:
        if len(sel) < cfg["max_running"] and used + reqs[i]["blocks"] <= cfg["mem_blocks"]:
            sel.add(i)
            used += reqs[i]["blocks"]

    def objective(s):
        gain, pen = 0.0, 0.0
        for i in cand:
            b = reqs[i]["buffer"] - reqs[i]["rate"] * cfg["interval"]
            if i in s:
                gain += value[i]
                b += cfg["gen_rate"] * tprime[i]
            pen += math.exp(-max(b, 0.0))
        return gain - cfg["gamma"] * pen

    for k in range(len(cand) - 1):
        a, b = cand[k], cand[k + 1]
        if (a in sel) == (b in sel):
            continue
        on, off = (a, b) if a in sel else (b, a)
        if used - reqs[on]["blocks"] + reqs[off]["blocks"] > cfg["mem_blocks"]:
            continue
        trial = (sel - {on}) | {off}
        if objective(trial) > objective(sel) + 1e-12:
            sel = trial
            used += reqs[off]["blocks"] - reqs[on]["blocks"]
    return finish(BUFFER_AWARE, sel)
