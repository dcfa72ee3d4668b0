"""A small serving-loop simulator that puts the pieces together: synthetic request arrivals, a
synthetic decode-time model, the buffer-aware scheduler (kvsched) deciding who runs, and the swap
library (kvswap) moving real KV blocks when a request is preempted, written through or resumed.

It exists to exercise the library the way the paper's system uses it (Section 3.1 workflow,
Section 4.2 scheduler, Section 5 memory manager) without a model: every running request produces
one token per decode iteration, an iteration takes step_time(batch) seconds, a prefill takes
prompt_len * prefill_per_token seconds.  The simulated clock advances by these model times and
by the transfer estimates (bytes / configured link rate); on a GPU the transfers are also really
executed, so that the KV content of every request can be checked at the end.  Without a GPU the
swap library runs under KV_PLAN_ONLY (bookkeeping only).

Policies: "tokenflow" (buffer-aware preemptive scheduling with write-through) and "fcfs" (requests
run to completion in arrival order, no preemption: the conventional baseline).
"""
from dataclasses import dataclass, field

import numpy as np

from . import kvsched as ks
from . import kvswap as kv
from . import workloads as W


@dataclass
class SimRequest:
    rid: int
    arrival: float
    prompt_len: int
    out_len: int
    rate: float
    # dynamic state
    state: str = "pending"        # pending -> new -> running <-> preempted -> done
    generated: int = 0
    t_gen: list = field(default_factory=list)
    table: list = field(default_factory=list)   # device blocks, logical order
    ready_at: float = 0.0                       # a resumed request decodes again from this time on
    preemptions: int = 0
    recomputes: int = 0


@dataclass
class SimConfig:
    geom: W.Geometry
    gpu_blocks: int
    arena_blocks: int
    max_running: int = 8
    interval: float = 1.0
    step_base: float = 0.020          # decode iteration = step_base + step_per_req * batch
    step_per_req: float = 0.0005
    prefill_per_token: float = 2e-5
    link_gbps: float = 55.0
    io_fixed: float = 5e-5
    policy: str = "tokenflow"
    write_through: bool = True
    safety: float = 1.5
    gamma: float = 1.0
    w_adjust: float = 0.0
    t_critical: float = 1.0
    tau_schedule: float = 0.0005
    qos_lambda: float = 1.0
    qos_mu: float = 1.0
    sync_io: bool = False             # True: the host waits for every eviction and load (the simple serving loop);
                                      # False: nothing waits on the host, the streams are ordered by events alone

    def step_time(self, batch):
        return self.step_base + self.step_per_req * batch


class Simulator:
    def __init__(self, cfg, requests, pool=None, staging=None, seed=0):
        """pool / staging: torch tensors for a real run on the GPU; None runs the library plan-only."""
        self.cfg, self.g = cfg, cfg.geom
        self.reqs = sorted(requests, key=lambda r: (r.arrival, r.rid))
        self.real = pool is not None
        self.pool, self.staging, self.seed = pool, staging, seed
        g = W.Geometry(self.g.L, self.g.H, self.g.D, self.g.B, self.g.dtype, cfg.gpu_blocks, scales=False)
        self.g = g
        if self.real:
            import torch
            # the library's two streams, known to torch so that the "model" can order itself after them
            self.s_evict, self.s_load = torch.cuda.Stream(), torch.cuda.Stream()
            self.kp = kv.KVPool(g, pool, staging, flags=kv.KV_REQ_EVENTS, evict_stream=self.s_evict,
                                load_stream=self.s_load)
        else:
            self.kp = kv.KVPool(g, flags=kv.KV_PLAN_ONLY, staging_bytes=cfg.arena_blocks * g.S)
        self.free = list(range(cfg.gpu_blocks - 1, -1, -1))
        self.t = 0.0
        self.log = []                   # (time, event, rid)
        self.moved_blocks = {"evict": 0, "write_through": 0, "load": 0}
        self.sched_calls = 0

    # ---- KV content: block j of request r is filled with a pattern only (r, j) determines ----
    def _pattern_offset(self, rid, j):
        return ((rid << 20) + j) * self.g.block_bytes

    def _pattern(self, rid, j0, n):
        """Pattern of logical blocks j0..j0+n of request rid as a [L, 2, n, chunk] uint8 tensor."""
        import torch
        g = self.g
        words = g.chunk // 8
        dev = self.pool.device
        base = torch.tensor([self._pattern_offset(rid, j0 + k) // 8 for k in range(n)], dtype=torch.int64, device=dev)
        plane = torch.arange(2 * g.L, dtype=torch.int64, device=dev) * words
        col = torch.arange(words, dtype=torch.int64, device=dev)
        w = base[None, :, None] + plane[:, None, None] + col[None, None, :]          # [2L, n, words]
        return W.fill_words_torch(self.seed, w, g.dtype).reshape(g.L, 2, n, g.chunk)

    def _poolv(self):
        g = self.g
        return self.pool[: g.pool_bytes].view(g.L, 2, g.N, g.chunk)                  # layer-major pool

    def _after_transfers(self):
        """The model's stream waits (on the GPU, not on the host) for the transfers enqueued so far: a block
        may be rewritten only after its eviction has read it, and read only after its load has filled it."""
        import torch
        cur = torch.cuda.current_stream()
        cur.wait_stream(self.s_evict)
        cur.wait_stream(self.s_load)

    def _fill_blocks(self, r, j0, blks):
        if not self.real or not blks:
            return
        import torch
        self._after_transfers()
        idx = torch.tensor(blks, dtype=torch.int64, device=self.pool.device)
        self._poolv().index_copy_(2, idx, self._pattern(r.rid, j0, len(blks)))

    def _fill(self, r, j, blk):
        self._fill_blocks(r, j, [blk])

    def check_request(self, r):
        """True when every device block of r holds the pattern of its logical index."""
        if not self.real or not r.table:
            return True
        import torch
        self._after_transfers()
        idx = torch.tensor(r.table, dtype=torch.int64, device=self.pool.device)
        return bool(torch.equal(self._poolv().index_select(2, idx), self._pattern(r.rid, 0, len(r.table))))

    # ---- helpers ----
    def _ctx(self, r):
        return r.prompt_len + r.generated

    def _blocks_needed(self, r, extra_tokens=0):
        return -(-(self._ctx(r) + extra_tokens) // self.g.B)

    def _grow(self, r):
        """Give r the blocks its context needs; False if the pool is out of blocks."""
        need = self._blocks_needed(r)
        j0, fresh = len(r.table), []
        while len(r.table) < need:
            if not self.free:
                self._fill_blocks(r, j0, fresh)
                return False
            fresh.append(self.free.pop())
            r.table.append(fresh[-1])
        self._fill_blocks(r, j0, fresh)
        return True

    def _buffer(self, r):
        """Unread tokens of r at the current time under the reader model."""
        if not r.t_gen:
            return 0.0
        rc, m = ks.kv_metric_stream(r.t_gen, r.arrival, r.rate)
        read = int(np.searchsorted(m["t_read"], self.t, side="right"))
        return float(len(r.t_gen) - read)

    def _produced(self):
        """Event after everything the "model" (torch, current stream) has written into the pool so far:
        swap-outs must wait for it, exactly as they wait for the decode kernels in a real server."""
        if not self.real:
            return None
        import torch
        ev = torch.cuda.Event()
        ev.record()
        self._events = getattr(self, "_events", [])[-64:] + [ev]     # keep them alive until they have fired
        return ev.cuda_event

    def _xfer_time(self, blocks):
        return self.cfg.io_fixed + blocks * self.g.S / (self.cfg.link_gbps * 1e9) if blocks else 0.0

    def _ok(self, rc, what):
        if rc != kv.KV_OK:
            raise kv.KVSwapError(rc, what)

    def _tables(self, rs):
        off = np.zeros(len(rs) + 1, np.int32)
        off[1:] = np.cumsum([len(r.table) for r in rs])
        ids = np.array([b for r in rs for b in r.table], np.int32)
        return off, ids

    # ---- actions ----
    def _write_through(self, running, dt):
        rs = [r for r in running if r.table]
        if not rs or not self.cfg.write_through:
            return
        # the handle's write queue: post what this iteration produced (priority = unread buffer, the likelier
        # victim first), then drain a chunk sized to the next iteration
        off, ids = self._tables(rs)
        lens = [self._ctx(r) for r in rs]
        prio = [self._buffer(r) for r in rs]
        self._ok(self.kp.wq_post([r.rid for r in rs], off, ids, lens, prio), "kv_wq_post")
        rc, wrote, pending, used = self.kp.wq_drain(interval_us=dt * 1e6, wait_event=self._produced())
        self._ok(rc, "kv_wq_drain")
        self.moved_blocks["write_through"] += int(wrote)

    def _preempt(self, r):
        off, ids = self._tables([r])
        if self.cfg.write_through:
            rc, moved = self.kp.swap_out_delta([r.rid], off, ids, [self._ctx(r)], flags=kv.KV_DELTA_INCLUDE_TAIL,
                                               wait_event=self._produced())
            self._ok(rc, "kv_swap_out_delta")
            n = int(moved.sum())
        else:
            self._ok(self.kp.swap_out([r.rid], off, ids, [self._ctx(r)], wait_event=self._produced()), "kv_swap_out")
            n = len(ids)
        if self.cfg.sync_io:
            self._ok(self.kp.sync(), "kv_sync")
        self.kp.wq_remove(r.rid)                    # its table is about to be given up (KV_ENOENT if it was not queued)
        self.moved_blocks["evict"] += n
        self.free.extend(reversed(r.table))        # the allocator takes the blocks back
        r.table = []
        r.state = "preempted"
        r.preemptions += 1
        self.log.append((self.t, "preempt", r.rid))
        return self._xfer_time(n)

    def _resume(self, r, how):
        nb = self._blocks_needed(r)
        if len(self.free) < nb:
            return None
        r.table = [self.free.pop() for _ in range(nb)]
        if how == ks.KVS_BY_RECOMPUTE:
            self._fill_blocks(r, 0, r.table)        # the prefill produces the same KV again
            if not self.cfg.write_through:          # a cold host copy is dropped; a write-through image stays valid
                self._ok(self.kp.release(r.rid), "kv_req_release")
            cost = self._ctx(r) * self.cfg.prefill_per_token
            r.recomputes += 1
        else:
            off, ids = self._tables([r])
            # the blocks were the model's (or another request's) a moment ago: after its writes, and, inside the
            # library, after any eviction that still reads them
            self._ok(self.kp.swap_in([r.rid], off, ids, kv.KV_KEEP_STAGING if self.cfg.write_through else 0,
                                     wait_event=self._produced()), "kv_swap_in")
            if self.cfg.sync_io:
                self._ok(self.kp.sync(), "kv_sync")
            self.moved_blocks["load"] += nb
            cost = self._xfer_time(nb)
        r.state = "running"
        r.ready_at = self.t + cost
        self.log.append((self.t, "resume", r.rid))
        return cost

    def _start(self, r):
        """Prefill a new request (prefill-first: decoding waits for it)."""
        r.generated = 0
        if len(self.free) < self._blocks_needed(r):
            return False
        self._grow(r)
        if self.cfg.write_through:
            cap = -(-(r.prompt_len + r.out_len) // self.g.B)
            self._ok(self.kp.reserve(r.rid, cap), "kv_req_reserve")
        self.t += r.prompt_len * self.cfg.prefill_per_token
        r.state = "running"
        r.ready_at = self.t
        self.log.append((self.t, "start", r.rid))
        return True

    def _finish(self, r):
        r.state = "done"
        self.ok_content = getattr(self, "ok_content", True) and self.check_request(r)
        self.free.extend(reversed(r.table))
        r.table = []
        self.kp.wq_remove(r.rid)
        self.kp.release(r.rid)                      # KV_ENOENT when it never had a host copy
        self.log.append((self.t, "done", r.rid))

    # ---- scheduling rounds ----
    def _schedule_tokenflow(self, live):
        cfg, g = self.cfg, self.g
        n_run = sum(1 for r in live if r.state == "running")
        gen_rate = 1.0 / cfg.step_time(max(n_run, 1))
        headroom = int(np.ceil(cfg.interval * gen_rate))
        reqs = []
        for r in live:
            st = {"new": ks.KVS_NEW, "running": ks.KVS_RUNNING, "preempted": ks.KVS_PREEMPTED}[r.state]
            rcq, q = self.kp.query(r.rid)
            staged_full = q["wm"] if rcq == kv.KV_OK else 0
            nb = self._blocks_needed(r, headroom if st != ks.KVS_NEW else 0)
            dirty = max(0, self._blocks_needed(r) - staged_full) if st == ks.KVS_RUNNING else 0
            reqs.append(dict(state=st, arrival=r.arrival, rate=r.rate, buffer=self._buffer(r), blocks=nb,
                             dirty_blocks=dirty, tokens=self._ctx(r)))
        io = self.kp.io_stats()
        rate = cfg.link_gbps
        sc = ks.make_config(mem_blocks=cfg.gpu_blocks, ws_blocks=cfg.gpu_blocks + cfg.arena_blocks,
                            max_running=cfg.max_running, interval=cfg.interval, gen_rate=gen_rate,
                            capacity=cfg.max_running / cfg.step_time(cfg.max_running), gamma=cfg.gamma,
                            safety=cfg.safety, w_adjust=cfg.w_adjust, t_critical=cfg.t_critical,
                            tau_schedule=cfg.tau_schedule, weight_tau=0.1 * 1024, weight_alpha=1.0 / (0.1 * 1024),
                            evict_gbps=rate, load_gbps=rate, io_fixed=cfg.io_fixed,
                            evict_queue=io["inflight_bytes"][0] / (rate * 1e9), load_queue=io["inflight_bytes"][1] / (rate * 1e9),
                            block_bytes=float(g.S), prefill_per_token=cfg.prefill_per_token)
        rc, mode, out = ks.kv_sched_step(sc, reqs)
        if rc != ks.KVS_OK:
            raise RuntimeError("kv_sched_step failed")
        self.sched_calls += 1
        # evictions first (they free the blocks the others need), then resumes, then new requests
        for r, o in zip(live, out):
            if o["decision"] == ks.KVS_PREEMPT:
                self._preempt(r)
        for r, o in zip(live, out):
            if o["decision"] == ks.KVS_RUN and r.state == "preempted":
                self._resume(r, o["how"])
        for r, o in zip(live, out):
            if o["decision"] == ks.KVS_RUN and r.state == "new":
                self._start(r)
        return mode

    def _schedule_fcfs(self, live):
        n_run = sum(1 for r in live if r.state == "running")
        for r in live:
            if r.state == "new" and n_run < self.cfg.max_running:
                # a conventional server admits a request only if its whole output will fit
                need = -(-(r.prompt_len + r.out_len) // self.g.B)
                reserved = sum(-(-(x.prompt_len + x.out_len) // self.g.B) - len(x.table) for x in live if x.state == "running")
                if len(self.free) - reserved >= need and self._start(r):
                    n_run += 1

    # ---- main loop ----
    def run(self, max_time=3600.0, progress=None):
        """progress: optional callable(sim) invoked about once per simulated scheduling interval."""
        cfg = self.cfg
        next_sched = 0.0
        pending = list(self.reqs)
        live = []
        self.ok_content = True
        while (pending or live) and self.t < max_time:
            while pending and pending[0].arrival <= self.t:
                r = pending.pop(0)
                r.state = "new"
                live.append(r)
            if not live:
                self.t = pending[0].arrival
                next_sched = min(next_sched, self.t)
                continue
            if self.t >= next_sched:
                if cfg.policy == "tokenflow":
                    self._schedule_tokenflow(live)
                    next_sched = self.t + cfg.interval
                    if progress:
                        progress(self)
                else:
                    self._schedule_fcfs(live)       # a conventional server looks at its queue every iteration
                    next_sched = self.t
                    if progress and int(self.t / cfg.interval) != getattr(self, "_tick", -1):
                        self._tick = int(self.t / cfg.interval)
                        progress(self)
            running = [r for r in live if r.state == "running" and r.ready_at <= self.t]
            if not running:
                # nothing can decode: jump to the next thing that can change that
                nxt = [next_sched] + [r.ready_at for r in live if r.state == "running"] + ([pending[0].arrival] if pending else [])
                self.t = max(self.t + 1e-6, min(nxt))
                continue
            dt = cfg.step_time(len(running))
            self.t += dt
            for r in running:
                r.generated += 1
                if not self._grow(r):               # out of blocks: the token is lost to this iteration
                    r.generated -= 1
                    continue
                r.t_gen.append(self.t)
            self._write_through(running, dt)
            for r in running:
                if r.generated >= r.out_len:
                    self._finish(r)
            live = [r for r in live if r.state != "done"]
        self.kp.sync()
        return self.summary()

    def summary(self):
        cfg = self.cfg
        done = [r for r in self.reqs if r.state == "done"]
        T = max(self.t, 1e-9)
        ttft, reb, wsum, esum, tokens = [], [], [], [], 0
        for r in done:
            rc, m = ks.kv_metric_stream(r.t_gen, r.arrival, r.rate)
            ttft.append(m["ttft"])
            reb.append(m["rebuffer"])
            tau = 0.1 * r.out_len
            wsum.append(ks.kv_metric_weight_sum(m["buffer"], tau, 1.0 / tau)[1])
            esum.append(ks.kv_metric_effective_sum(m["buffer"])[1])
            tokens += len(r.t_gen)
        qos = ks.kv_metric_qos(wsum, ttft, reb, cfg.qos_lambda, cfg.qos_mu, T)[1] if done else 0.0
        return dict(policy=cfg.policy, finished=len(done), of=len(self.reqs), makespan_s=round(T, 3),
                    throughput_tok_s=round(tokens / T, 2), effective_throughput_tok_s=round(sum(esum) / T, 2),
                    qos=round(qos, 3), ttft_mean_s=round(float(np.mean(ttft)), 3) if ttft else None,
                    ttft_p99_s=round(float(np.percentile(ttft, 99)), 3) if ttft else None,
                    rebuffer_total_s=round(float(np.sum(reb)), 3), preemptions=sum(r.preemptions for r in self.reqs),
                    recomputes=sum(r.recomputes for r in self.reqs), blocks_moved=dict(self.moved_blocks),
                    sched_calls=self.sched_calls, kv_content_ok=bool(self.ok_content))

    def close(self):
        self.kp.close()


def burst_requests(seed, n, prompt_mean, out_mean, rates=(15.0, 20.0), at=0.0):
    """A burst of n requests at time `at`, lengths normally distributed (sigma = 20 % of the mean),
    reading rates drawn from `rates`: the shape of the paper's controlled burst setups (Section 7.3)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        p = int(np.clip(rng.normal(prompt_mean, 0.2 * prompt_mean), 16, 4 * prompt_mean))
        o = int(np.clip(rng.normal(out_mean, 0.2 * out_mean), 16, 4 * out_mean))
        out.append(SimRequest(rid=i + 1, arrival=at + 1e-3 * i, prompt_len=p, out_len=o, rate=float(rng.choice(rates))))
    return out
