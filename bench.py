#!/usr/bin/env python3
"""Benchmark of the paged KV-cache swap on one MI355X.

Headline workload: the largest single-GPU configuration, configs[3]: Llama-3-70B-shaped KV (bf16, 80 layers,
8 KV heads, head_dim 128, block_size 16: 5 MiB per block), a pool sized to 200 GB of HBM (38 146 blocks),
128 requests of 1k-16k tokens on block tables drawn from a pool in which a random half of the blocks was freed.
The 128 requests hold ~350 GiB of KV, more than the free half of the pool and far more than the pinned arena,
so they are preempted and resumed in WAVES: as many requests, in order, as fit a 40 GiB host arena (10 waves).

One step = one pass of the whole hot path over one wave:
  1. kv_swap_out  of the wave's requests (plan, gather, device->host)             -> kv_sync
  2. kv_swap_in   into fresh blocks of the fragmented free list, staging kept
                  (host->device, scatter)                                         -> kv_sync
  3. every request generates one more block of tokens; kv_swap_out_delta writes
     through only what is new (its former tail block and the new block)           -> kv_sync
  4. on-device leg: the same blocks are gathered into an HBM arena and scattered
     back to their original ids (both ends in HBM)                                -> kv_sync
  5. the requests are released, so every wave starts from the same pool state.
Step s works on wave s mod 10, warm-up steps included, so that 10 timed steps cover all 128 requests once
(the default; with --steps 20 every wave is timed twice).
`value` = host-link payload bytes of the timed steps (legs 1-3) / their wall time.  Per-leg figures, per-wave
rates, the HBM roofline of the on-device kernels, the fraction of the measured host-link ceiling, isolated
per-request preempt/resume latency over all 128 requests and the CPU oracle's rate (one core, and all cores)
are reported in the same JSON line; `configs` in that line carries the same figures for the other four
configurations, measured in this run after the headline (bench_configs.py).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# HBM bytes per block moved by one on-device launch of the headline workload, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs of this script, each scaled on a plain copy of known size (summary, commands and scale factors:
# profiles/kv_move_kernel_llama70b_waves.md, whose table holds these same numbers; tests/test_host_logic.py
# compares the two).  KiB per block of 5 120 KiB: (read, written).
MEASURED_KIB_PER_BLOCK = {"gather": (5120.1, 5119.8), "scatter_block_by_block": (5120.0, 5119.8),
                          "scatter_plane_by_plane": (5120.1, 5119.8)}
TRAFFIC_SOURCE = "profiles/kv_move_kernel_llama70b_waves.md"


def pct(xs, q):
    return float(np.percentile(np.asarray(xs, dtype=np.float64), q))


def headline(kv, W, BC, torch, dev, args, arena, streams):
    """configs[3] in waves.  Returns the top-level fields of the JSON line."""
    ok = lambda rc, what: BC.ok(kv, rc, what)  # noqa: E731
    wl = W.config(4, num_blocks=args.blocks or None, variant=args.variant)
    g = wl.geom
    lens = W.request_lengths(wl.seed, wl.n_requests, wl.length_dist)
    nb = W.blocks_for(lens, g.B)
    # the pool after a random half of its blocks was freed: F is the shuffled free list every wave allocates from
    _, _, F = W.fragmented_tables(wl.seed, g.N, [], 0.5)
    nreq = wl.n_requests
    arena_slots = min(arena.numel() // g.S, (40 << 30) // g.S)
    # a wave needs its own blocks, as many fresh ones and one more per request, all from the free list
    waves = BC.waves_of(nb, arena_slots, room_per_request=1, limit_blocks=(len(F) - 64) // 2)
    nwaves = len(waves)
    steps = args.steps if args.steps > 0 else nwaves
    warmup = args.warmup if args.warmup >= 0 else 1

    BC.note("headline: allocating and filling the %.0f GiB pool" % (g.pool_bytes / 2**30))
    pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device=dev)
    if not args.no_fill:
        W.fill_buffer_torch(wl.seed, pool, g.dtype)
    max_total = max(int(nb[r].sum()) for r in waves)
    dev_arena = torch.empty(max(max_total * g.S, 8 << 30), dtype=torch.uint8, device=dev)
    bounce = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    staging = arena[:arena_slots * g.S]
    flags = {"auto": kv.KV_PATH_AUTO, "zerocopy": kv.KV_PATH_ZEROCOPY, "dma": kv.KV_PATH_DMA}[args.path]
    evict, load = streams.evict, streams.load
    kp = kv.KVPool(g, pool, staging, bounce=bounce if args.path == "dma" else None, flags=flags,
                   evict_stream=evict, load_stream=load)
    kd = kv.KVPool(g, pool, dev_arena, flags=kv.KV_STAGING_DEVICE, evict_stream=evict, load_stream=load)
    ok(kd.tune(kv.KV_TUNE_KERNEL_EVENTS, 1), "kv_pool_tune")      # ms_kernel of the on-device launches: the kernel alone
    torch.cuda.synchronize()

    # ---- ceilings, measured in this run ----
    one = 1 << 30
    link_d2h = one / kv.kv_bench_link(staging.data_ptr(), dev_arena.data_ptr(), one, 0, 4, evict.cuda_stream) / 1e6
    link_h2d = one / kv.kv_bench_link(staging.data_ptr(), dev_arena.data_ptr(), one, 1, 4, evict.cuda_stream) / 1e6
    # best of three: which copy engines the runtime picks for the two directions varies from try to try
    ms = [kv.kv_bench_link_bidir(staging.data_ptr(), dev_arena.data_ptr(), staging.data_ptr() + one,
                                 dev_arena.data_ptr() + one, one, 3) for _ in range(3)]
    link_bidir = 2 * one / min(ms) / 1e6 if min(ms) > 0 else None
    # 16 GiB of plain copy first: the memory clocks take some hundred milliseconds of load to come up
    lo, hi = dev_arena.data_ptr(), dev_arena.data_ptr() + 4 * one
    kv.kv_bench_copy(hi, lo, 4 * one, 0, 40, evict.cuda_stream)
    copy_gbs = 2 * 4 * one / kv.kv_bench_copy(hi, lo, 4 * one, 0, 5, evict.cuda_stream) / 1e6
    # the 16 KiB-piece shape, kept under its own kernel name as the known-size reference of the counter runs
    kv.kv_bench_copy(hi, lo, 4 * one, 1 << 18, 2, evict.cuda_stream)
    # what chunk-sized scattered accesses allow: the same copy with one side visited in scrambled 32 KiB runs
    run = max(4096, g.chunk)
    gather_ceiling = 2 * 4 * one / kv.kv_bench_copy_scrambled(hi, lo, 4 * one, run, 0, 5, evict.cuda_stream) / 1e6
    scatter_ceiling = 2 * 4 * one / kv.kv_bench_copy_scrambled(hi, lo, 4 * one, run, 1, 5, evict.cuda_stream) / 1e6

    # ---- the waves ----
    # Every wave allocates from the same free list: its own blocks from the first M entries (M = the largest wave), the
    # fresh blocks it is resumed into from the next M, the blocks it grows into from what follows.  So the first M always
    # hold their original content when a wave starts, whatever the waves before it left in the rest.
    tabs = []
    M = max_total
    assert 2 * M + max(len(r) for r in waves) <= len(F)
    for rows in waves:
        n = len(rows)
        off = np.zeros(n + 1, np.int32)
        off[1:] = np.cumsum(nb[rows])
        total = int(off[-1])
        ids, new, extra = F[:total].copy(), F[M:M + total].copy(), F[2 * M:2 * M + n].copy()
        off2 = off + np.arange(n + 1, dtype=np.int32)
        ids2 = np.concatenate([np.append(new[off[i]:off[i + 1]], extra[i]) for i in range(n)]).astype(np.int32)
        tabs.append(dict(rows=rows, n=n, rid=(rows + 1).astype(np.uint64), off=off, ids=ids, new=new, off2=off2, ids2=ids2,
                         lens=lens[rows], lens2=((nb[rows] + 1) * g.B).astype(np.int32), total=total))

    per_wave = [dict(out=[], inn=[], blocks=t["total"], requests=t["n"]) for t in tabs]
    acc = {k: [] for k in ("out", "in", "delta", "dev", "gather_k", "scatter_k", "out_k", "in_k", "plan_us")}
    moved_bytes = {"link": 0, "gather": 0, "scatter": 0, "out": 0, "delta": 0}
    scatter_orders = []
    delta_blocks = []

    def step(s, record):
        w = s % nwaves
        t = tabs[w]
        rid, off, ids, new = t["rid"], t["off"], t["ids"], t["new"]
        c = [time.perf_counter()]
        for i in range(t["n"]):
            ok(kp.reserve(rid[i], int(off[i + 1] - off[i]) + 1), "kv_req_reserve")
        ok(kp.swap_out(rid, off, ids, t["lens"]), "kv_swap_out")
        so = kp.stats() if record else None
        ok(kp.sync(), "kv_sync")
        c.append(time.perf_counter())
        ok(kp.swap_in(rid, off, new, kv.KV_KEEP_STAGING), "kv_swap_in")
        si = kp.stats() if record else None
        ok(kp.sync(), "kv_sync")
        c.append(time.perf_counter())
        rc, moved = kp.swap_out_delta(rid, t["off2"], t["ids2"], t["lens2"])
        ok(rc, "kv_swap_out_delta")
        ok(kp.sync(), "kv_sync")
        c.append(time.perf_counter())
        ok(kd.swap_out(rid, off, new, t["lens"]), "kv_swap_out(device arena)")
        go = kd.stats() if record else None
        ok(kd.swap_in(rid, off, ids), "kv_swap_in(device arena)")
        gi = kd.stats() if record else None
        ok(kd.sync(), "kv_sync")
        c.append(time.perf_counter())
        for i in range(t["n"]):
            ok(kp.release(rid[i]), "kv_req_release")
        if record:
            P = t["total"] * g.S
            acc["out"].append(c[1] - c[0])
            acc["in"].append(c[2] - c[1])
            acc["delta"].append(c[3] - c[2])
            acc["dev"].append(c[4] - c[3])
            acc["out_k"].append(so["ms_kernel"] if so["path"] == kv.KV_PATH_ZEROCOPY else so["ms_total"])
            acc["in_k"].append(si["ms_kernel"] if si["path"] == kv.KV_PATH_ZEROCOPY else si["ms_total"])
            acc["gather_k"].append(go["ms_kernel"])
            acc["scatter_k"].append(gi["ms_kernel"])
            acc["plan_us"].append(so["plan_us"])
            scatter_orders.append(gi["scatter_order"])
            delta_blocks.append(int(moved.sum()))
            moved_bytes["link"] += 2 * P + int(moved.sum()) * g.S
            moved_bytes["out"] += P
            moved_bytes["delta"] += int(moved.sum()) * g.S
            moved_bytes["gather"] += 2 * P
            moved_bytes["scatter"] += 2 * P
            per_wave[w]["out"].append(c[1] - c[0])
            per_wave[w]["inn"].append(c[2] - c[1])

    BC.note("headline: %d warm-up and %d timed steps over %d waves" % (warmup, steps, nwaves))
    for s in range(warmup):
        step(s, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(warmup, warmup + steps):
        step(s, True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    path_used = {kv.KV_PATH_DMA: "dma", kv.KV_PATH_ZEROCOPY: "zerocopy"}
    sstat = kp.stats()

    # ---- check that nothing was skipped: the pool is back where it started ----
    # (after a wave, block new[j] holds what block ids[j] was filled with; ids and untouched blocks hold their own fill)
    rng = np.random.default_rng(1)
    ls, ks, bs = g.strides
    last = tabs[(warmup + steps - 1) % nwaves]
    js = rng.choice(last["total"], size=12, replace=False).tolist()
    pairs = [(int(last["new"][j]), int(last["ids"][j])) for j in js] + [(int(last["ids"][j]), int(last["ids"][j])) for j in js[:4]]
    taken = np.zeros(g.N, bool)
    taken[F] = True
    pairs += [(int(p), int(p)) for p in rng.choice(np.flatnonzero(~taken), size=4)]      # blocks of foreign requests
    bad = 0
    for holder, origin in (pairs if not args.no_fill else []):
        for l in (0, g.L // 2, g.L - 1):
            for c in (0, 1):
                want = W.fill_bytes_torch(wl.seed, l * ls + c * ks + origin * bs, g.chunk, g.dtype, dev)
                o = l * ls + c * ks + holder * bs
                bad += int((pool[o:o + g.chunk] != want).any())
    if bad:
        print("bench.py: pool content check FAILED on %d chunks" % bad, file=sys.stderr)
        sys.exit(3)

    # ---- the on-device kernels back to back on wave 0, each job order of the scatter forced in turn ----
    BC.note("headline: on-device kernels back to back")
    t = tabs[0]
    steady = {}
    ok(kd.swap_out(t["rid"], t["off"], t["ids"], t["lens"]), "kv_swap_out(device arena)")   # wave 0's state after its swap-in
    ok(kd.swap_in(t["rid"], t["off"], t["new"]), "kv_swap_in(device arena)")
    for name, order in (("block_by_block", 1), ("plane_by_plane", 2)):
        ok(kd.tune(kv.KV_TUNE_SCATTER_ORDER, order), "kv_pool_tune")
        gk, sk = [], []
        for rep in range(9):
            ok(kd.swap_out(t["rid"], t["off"], t["new"], t["lens"]), "kv_swap_out(device arena)")
            go = kd.stats()
            ok(kd.swap_in(t["rid"], t["off"], t["ids"]), "kv_swap_in(device arena)")
            gi = kd.stats()
            ok(kd.sync(), "kv_sync")
            if rep:
                gk.append(go["ms_kernel"])
                sk.append(gi["ms_kernel"])
        steady["gather"] = round(2 * t["total"] * g.S / float(np.mean(gk)) / 1e6, 1)
        steady["scatter_" + name] = round(2 * t["total"] * g.S / float(np.mean(sk)) / 1e6, 1)
    ok(kd.tune(kv.KV_TUNE_SCATTER_ORDER, 0), "kv_pool_tune")

    # ---- isolated per-request preempt / resume latency (call -> kv_sync) over all requests, outside the timed steps ----
    BC.note("headline: isolated latency of %d requests" % nreq)
    pre, res = [], []
    cursor = 0
    for i in range(nreq if not args.quick else min(nreq, 16)):
        k = int(nb[i])
        if cursor + k > len(F):
            cursor = 0
        blk = F[cursor:cursor + k]
        cursor += k
        o1 = np.array([0, k], dtype=np.int32)
        r1 = np.array([i + 1], dtype=np.uint64)
        a = time.perf_counter()
        ok(kp.swap_out(r1, o1, blk, lens[i:i + 1]), "kv_swap_out")
        ok(kp.sync(), "kv_sync")
        b = time.perf_counter()
        ok(kp.swap_in(r1, o1, blk), "kv_swap_in")
        ok(kp.sync(), "kv_sync")
        pre.append((b - a) * 1e3)
        res.append((time.perf_counter() - b) * 1e3)

    # ---- per-request completion inside a wave (KV_REQ_EVENTS), outside the timed steps ----
    kev = kv.KVPool(g, pool, staging, flags=flags | kv.KV_REQ_EVENTS, evict_stream=evict, load_stream=load)
    ok(kev.swap_out(t["rid"], t["off"], t["ids"], t["lens"]), "kv_swap_out(events)")
    _, t_out = kev.timeline()
    ev_out_total = kev.stats()["ms_total"]
    ok(kev.swap_in(t["rid"], t["off"], t["ids"]), "kv_swap_in(events)")
    _, t_in = kev.timeline()
    ev_in_total = kev.stats()["ms_total"]
    ok(kev.sync(), "kv_sync")
    kev.close()

    # ---- the copy-engine path on wave 0, for comparison (outside the timed steps) ----
    kdma = kv.KVPool(g, pool, staging, bounce=bounce, flags=kv.KV_PATH_DMA, evict_stream=evict, load_stream=load)
    dma = {}
    P0 = t["total"] * g.S
    for rep in range(2):
        a = time.perf_counter()
        ok(kdma.swap_out(t["rid"], t["off"], t["ids"], t["lens"]), "kv_swap_out(dma)")
        ok(kdma.sync(), "kv_sync")
        b = time.perf_counter()
        ok(kdma.swap_in(t["rid"], t["off"], t["ids"]), "kv_swap_in(dma)")
        ok(kdma.sync(), "kv_sync")
        c = time.perf_counter()
        dma = {"d2h_gbps": round(P0 / (b - a) / 1e9, 2), "h2d_gbps": round(P0 / (c - b) / 1e9, 2)}
    kdma.close()

    s_out, s_in, s_delta, s_dev = (float(np.sum(acc[k])) for k in ("out", "in", "delta", "dev"))
    d2h = moved_bytes["out"] / s_out / 1e9
    h2d = moved_bytes["out"] / s_in / 1e9
    value = moved_bytes["link"] / elapsed / 1e9
    gather_ms, scatter_ms = float(np.mean(acc["gather_k"])), float(np.mean(acc["scatter_k"]))
    gather_gbs = moved_bytes["gather"] / (float(np.sum(acc["gather_k"])) * 1e-3) / 1e9
    scatter_gbs = moved_bytes["scatter"] / (float(np.sum(acc["scatter_k"])) * 1e-3) / 1e9
    blocks_per_launch = moved_bytes["scatter"] / (2 * g.S) / steps
    # the handle times both job orders of a large on-device scatter on its first two calls and keeps the faster one
    # for the pool it was given: 0 block by block, 1 plane by plane
    plane_major = 2 * sum(o == 1 for o in scatter_orders) > len(scatter_orders)

    def traffic(which):
        kib = MEASURED_KIB_PER_BLOCK.get(which)
        if kib is None or args.blocks:
            return None
        return int(round((kib[0] + kib[1]) * 1024 * blocks_per_launch))

    covered = sorted(set(int(r) for s in range(warmup, warmup + steps) for r in tabs[s % nwaves]["rows"]))
    timed_requests = sum(tabs[s % nwaves]["n"] for s in range(warmup, warmup + steps))
    out_k = float(np.sum(acc["out_k"]))
    r2, r3, r4 = (lambda x: round(x, 2)), (lambda x: round(x, 3)), (lambda x: round(x, 4))
    out = {
        "metric": "swap GB/s (D2H, H2D, on-device) + p50 preempt/resume latency per request",
        "value": r2(value), "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": r2(elapsed * 1e3 / steps),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic" if not args.no_fill else "synthetic tables, pool content as allocated (--no-fill)",
        "config": {"workload": "configs[3]: Llama-3-70B-shaped KV bf16 L80 H8 D128 B16 (5 MiB blocks), %d-block pool (%.0f GB), %d "
                               "requests 1k-16k tokens (%d blocks, %.1f GiB per direction) on tables from a 50%% randomly freed pool, "
                               "preempted and resumed in %d waves through a %.0f GiB pinned arena; one step = one wave"
                               % (g.N, g.pool_bytes / 1e9, nreq, int(nb.sum()), int(nb.sum()) * g.S / 2**30, nwaves,
                                  arena_slots * g.S / 2**30),
                   "seed": "0x%X" % wl.seed, "path": path_used.get(sstat["path"], str(sstat["path"])),
                   "waves": nwaves, "waves_timed": len(set(s % nwaves for s in range(warmup, warmup + steps))),
                   "requests_timed": len(covered),
                   "value_def": "link payload (swap-out + swap-in + delta) of the timed steps / their wall time"},
        "legs": {
            "d2h_gbps": r2(d2h), "h2d_gbps": r2(h2d),
            "d2h_frac_of_measured_link": r3(d2h / link_d2h), "h2d_frac_of_measured_link": r3(h2d / link_h2d),
            "delta_blocks_mean": round(float(np.mean(delta_blocks)), 1), "delta_ms_mean": r3(s_delta * 1e3 / steps),
            "delta_gbps": r2(moved_bytes["delta"] / s_delta / 1e9),
            "ondevice_gather_traffic_gbps": round(gather_gbs, 1), "ondevice_scatter_traffic_gbps": round(scatter_gbs, 1),
            "ondevice_back_to_back_traffic_gbps": steady,
            "plan_us_wave": round(float(np.mean(acc["plan_us"])), 1),
            "wave_preempt_ms_per_request": r3(s_out * 1e3 / timed_requests),
            "wave_resume_ms_per_request": r3(s_in * 1e3 / timed_requests),
            "dma_path_wave0_gbps": [dma["d2h_gbps"], dma["h2d_gbps"]],
            "waves_req_gib_d2h_h2d": [[pw["requests"], r2(pw["blocks"] * g.S / 2**30),
                                       r2(pw["blocks"] * g.S / float(np.mean(pw["out"])) / 1e9) if pw["out"] else None,
                                       r2(pw["blocks"] * g.S / float(np.mean(pw["inn"])) / 1e9) if pw["inn"] else None]
                                      for pw in per_wave],
        },
        "latency": {"p50_preempt_ms": r3(pct(pre, 50)), "p90_preempt_ms": r3(pct(pre, 90)),
                    "p50_resume_ms": r3(pct(res, 50)), "p90_resume_ms": r3(pct(res, 90)),
                    "def": "isolated single-request call -> kv_sync, %d requests (mean %.2f GiB)"
                           % (len(pre), float(np.mean(nb[:len(pre)])) * g.S / 2**30),
                    "in_wave0_events": {"p50_preempt_ms": r2(pct(t_out, 50)), "p50_resume_ms": r2(pct(t_in, 50)),
                                        "last_preempt_ms": r2(float(t_out[-1])), "last_resume_ms": r2(float(t_in[-1]))}},
        "link": {"measured_peak_d2h_gbps": r2(link_d2h), "measured_peak_h2d_gbps": r2(link_h2d),
                 "measured_peak_bidirectional_gbps": None if link_bidir is None else r2(link_bidir),
                 "how": "one 1 GiB pinned hipMemcpyAsync per direction, in this run"},
        "roofline_link": {"bound": "host-link", "kernel": "kv_move_kernel<0,4,1,true,false> (a wave's swap-out)",
                          "achieved": r2(moved_bytes["out"] / out_k / 1e6), "peak": 64.0, "unit": "GB/s",
                          "frac": r4(moved_bytes["out"] / out_k / 1e6 / 64.0), "launch_ms": r2(out_k / steps),
                          "bytes_per_launch": int(moved_bytes["out"] / steps), "measured_peak": r2(link_d2h),
                          "frac_of_measured_peak": r4(moved_bytes["out"] / out_k / 1e6 / link_d2h)},
        "roofline_gather": {"bound": "hbm", "kernel": "kv_move_kernel<0,1,0,true,false> (gather, both ends in HBM)",
                            "achieved": round(gather_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": r4(gather_gbs / HBM_PEAK_GBS), "traffic": traffic("gather"),
                            "launch_ms": r3(gather_ms), "bytes_per_launch": int(moved_bytes["gather"] / steps),
                            "measured_gathered_copy_ceiling_gbps": round(gather_ceiling, 1)},
        "roofline": {"bound": "hbm",
                     "kernel": ("kv_move_kernel<1,1,0,true,true> (scatter plane by plane, both ends in HBM)" if plane_major
                                else "kv_move_kernel<1,1,0,true,false> (scatter block by block, both ends in HBM)"),
                     "achieved": round(scatter_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": r4(scatter_gbs / HBM_PEAK_GBS),
                     "traffic": traffic("scatter_plane_by_plane" if plane_major else "scatter_block_by_block"),
                     "traffic_source": TRAFFIC_SOURCE,
                     "launch_ms": r3(scatter_ms), "bytes_per_launch": int(moved_bytes["scatter"] / steps),
                     "blocks_per_launch": round(blocks_per_launch, 1), "algorithmic_bytes_per_block": 2 * g.S,
                     "scatter_orders": "".join(str(o) for o in scatter_orders),
                     "measured_copy_ceiling_gbps": round(copy_gbs, 1),
                     "measured_scattered_copy_ceiling_gbps": round(scatter_ceiling, 1),
                     "frac_of_scattered_copy_ceiling": r4(scatter_gbs / scatter_ceiling)},
    }
    kp.close()
    kd.close()
    del pool, dev_arena, bounce
    BC.release(torch)
    return out, (wl, g, lens, nb)


def compact(name, r):
    """The figures of one configuration that the JSON line carries (the functions in bench_configs.py return more;
    --verbose keeps all of it).  Rates in GB/s, times in ms unless the key says otherwise; pairs are [swap-out, swap-in]."""
    if name == "configs[0]":
        return {"p50_preempt_ms": r["p50_preempt_ms"], "p50_resume_ms": r["p50_resume_ms"], "host_call_us_p50": r["host_call_us_p50"],
                "note": "3 requests per call, 544 KiB: the fixed cost of a call"}
    if name == "configs[1]":
        od = r["ondevice"]
        return {"d2h_gbps": r["d2h_gbps"], "h2d_gbps": r["h2d_gbps"],
                "frac_of_measured_link": [r["d2h_frac_of_measured_link"], r["h2d_frac_of_measured_link"]],
                "delta_blocks": r["delta_blocks"], "delta_ms": r["delta_ms"],
                "ondevice_frac_of_hbm_peak": {k: v["frac_of_hbm_peak"] for k, v in od.items()},
                "ondevice_launch_ms": {k: v["launch_ms"] for k, v in od.items()},
                "p50_preempt_ms": r["p50_preempt_ms"], "p50_resume_ms": r["p50_resume_ms"],
                "p90_preempt_ms": r["p90_preempt_ms"], "p90_resume_ms": r["p90_resume_ms"]}
    if name == "configs[2]":
        ds = r["delta_step"]
        return {"priming_gbps": r["priming_delta"]["gbps"], "step_blocks_mean": ds["blocks_mean"],
                "step_call_to_sync_us": [ds["call_to_sync_us_p50"], ds["call_to_sync_us_p99"]], "step_host_call_us_p50": ds["host_call_us_p50"],
                "preempt_after_write_through_ms_per_request": r["preempt_32_after_write_through"]["ms_per_request"],
                "preempt_cold_ms_per_request": r["preempt_32_cold"]["ms_per_request"],
                "resume_ms_per_request": r["resume_32"]["ms_per_request"],
                "step_next_to_compute": {k: ([v["call_to_sync_us_p50"], v["call_to_sync_us_p99"], v["co_runner_traffic_gbps"]]
                                             if isinstance(v, dict) else v)
                                         for k, v in r["delta_step_next_to_compute"].items()},
                "d2h_gbps": r["d2h_gbps"], "h2d_gbps": r["h2d_gbps"]}
    if name == "configs[4]":
        c = r["contended"]
        leg = lambda x: x["contended_gbps"] + [x["stream_kernel_traffic_gbps"]]  # noqa: E731
        return {"requests": r["requests"], "waves": r["waves"], "d2h_gbps": r["d2h_gbps"], "h2d_gbps": r["h2d_gbps"],
                "frac_of_measured_link": [r["d2h_frac_of_measured_link"], r["h2d_frac_of_measured_link"]],
                "ms_per_request": [r["p50_preempt_ms"], r["p50_resume_ms"]],
                "contended_gbps": [c["d2h_gbps"], c["h2d_gbps"]],
                "co_runner_traffic_gbps": [c["stream_kernel_traffic_gbps_alone"], c["stream_kernel_traffic_gbps_while_swapping"]],
                "wave0_contended_by_link_workgroups": {k: leg(v) for k, v in r["zero_copy_workgroup_budget_first_wave"].items()},
                "wave0_contended_dma_path": leg(r["dma_path_first_wave"]),
                "def": "contended: next to a read-modify-write kernel streaming through 16 GiB; triples are [out, in, co-runner]"}
    if name == "load_evict_overlap":
        return {"both_directions_ceiling_gbps": r["measured_link_gbps"]["both_at_once"],
                "zerocopy_ms": [r["zerocopy"]["serial_ms"], r["zerocopy"]["overlapped_ms"]],
                "zerocopy_overlapped_gbps": r["zerocopy"]["overlapped_aggregate_gbps"],
                "zerocopy_160_workgroups_overlapped_gbps": r["zerocopy_160_workgroups"]["overlapped_aggregate_gbps"],
                "dma_ms": [r["dma"]["serial_ms"], r["dma"]["overlapped_ms"]],
                "dma_overlapped_gbps": r["dma"]["overlapped_aggregate_gbps"],
                "load_into_blocks_being_evicted_ms": {k: v["ms"] for k, v in r["load_into_blocks_being_evicted"].items()},
                "def": "8B shape, 8.9 GiB evicted while 8.9 GiB are loaded (Section 5.3); pairs are [serial, overlapped]"}
    if name == "general_kernel_builds":
        return {k: {"gather_frac": v["gather"]["frac"], "scatter_frac": v["scatter"]["frac"],
                    "launch_ms": [v["gather"]["launch_ms"], v["scatter"]["launch_ms"]], "bytes_per_launch": v["bytes_per_launch"],
                    "scrambled_copy_ceiling_gbps": [v["scrambled_copy_ceiling_gbps"]["source_scrambled"],
                                                    v["scrambled_copy_ceiling_gbps"]["destination_scrambled"]]}
                for k, v in r["kernels"].items()}
    return r


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (waves); 0: one pass over all waves")
    ap.add_argument("--warmup", type=int, default=-1, help="untimed steps; -1: one")
    ap.add_argument("--path", choices=["auto", "zerocopy", "dma"], default="auto")
    ap.add_argument("--cpu-sample", type=int, default=3, help="requests the CPU oracle is timed on (0: skip)")
    ap.add_argument("--blocks", type=int, default=0, help="override the headline pool size (debugging on small boxes)")
    ap.add_argument("--variant", type=int, default=0, help="0: the configuration's own seed; 1, 2: further seeds")
    ap.add_argument("--only", default="headline,1,2,3,5,6,8",
                    help="comma-separated parts to run: headline, 1, 2, 3, 5, 6 (load-evict overlap), 8 (general kernel builds)")
    ap.add_argument("--no-fill", action="store_true",
                    help="leave the headline pool's content as allocated and skip the content check (counter-collection runs, "
                         "where the thousands of fill launches would take minutes; the swap moves bytes whatever they are)")
    ap.add_argument("--verbose", action="store_true", help="keep every field the per-configuration functions return")
    ap.add_argument("--quick", action="store_true", help="fewer isolated-latency requests and fewer waves of configs[4]")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a one-GPU library (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not os.path.exists(os.path.join(ROOT, "paper_2510_02758_amd", "libkvswap.so")):
        import __graft_entry__          # load what is built; build only a tree in which nothing is
        __graft_entry__.build()
    from paper_2510_02758_amd import kvswap as kv
    from paper_2510_02758_amd import workloads as W
    import bench_configs as BC

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    parts = [p.strip() for p in args.only.split(",") if p.strip()]
    streams = BC.Streams(torch)      # before anything else: see the class

    # ---- one pinned arena for every configuration: PyTorch only allocates ----
    arena_bytes = (48 << 30) if not args.blocks else (12 << 30)
    BC.note("pinning a %.0f GiB host arena" % (arena_bytes / 2**30))
    arena = torch.empty(arena_bytes, dtype=torch.uint8, pin_memory=True)
    arena.view(torch.int64)[::512] = 0          # touch every page before timing

    out, info = headline(kv, W, BC, torch, dev, args, arena, streams)
    configs = {}
    runs = {"1": ("configs[0]", BC.config1), "2": ("configs[1]", BC.config2), "3": ("configs[2]", BC.config3),
            "5": ("configs[4]", BC.config5), "6": ("load_evict_overlap", BC.config6), "8": ("general_kernel_builds", BC.config8)}
    for key in ("1", "2", "3", "5", "6", "8"):
        if key not in parts:
            continue
        name, fn = runs[key]
        BC.note("part %s (%s)" % (key, name))
        if key == "5":
            r = fn(kv, W, torch, dev, args, arena, streams, max_waves=3 if (args.quick or args.blocks) else None)
        else:
            r = fn(kv, W, torch, dev, args, arena, streams)
        configs[name] = r if args.verbose else compact(name, r)
    out["configs"] = configs
    del arena
    BC.release(torch)
    if args.cpu_sample > 0:
        wl, g, lens, nb = info
        BC.note("CPU oracle on %d requests" % args.cpu_sample)
        n = min(args.cpu_sample, len(nb))
        # requests of about the mean size: the sample stays near 8 GiB each way whatever the seed
        order = np.argsort(np.abs(nb - np.mean(nb)))[:n]
        out["cpu_baseline"] = BC.oracle_rates(W, g, lens[order], nb[order], n, wl.seed, passes=2)
    BC.note("done")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
