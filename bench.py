#!/usr/bin/env python3
"""Benchmark of the paged KV-cache swap on one MI355X.

Workload: the Llama-3-8B-shaped burst (bf16, 32 layers, 8 KV heads, head_dim 128,
block_size 16, 40 000-block pool = 78 GiB; 64 requests of 512-4096 tokens on
random block tables), synthetic and seeded.

One step = one pass of the whole hot path over that burst:
  1. kv_swap_out  of all 64 requests (plan, gather, device->host)      -> kv_sync
  2. kv_swap_in   into fresh random blocks, staging kept (host->device, scatter) -> kv_sync
  3. every request generates one more block of tokens; kv_swap_out_delta writes
     through only what is new (its former tail block and the new block)  -> kv_sync
  4. on-device leg: the same blocks are gathered into an HBM arena and scattered
     back to their original ids (both ends in HBM)                       -> kv_sync
  5. the requests are released, so the next step starts from the same state.
`value` = host-link payload bytes of the step (legs 1-3) / wall time of the whole
step.  Per-leg figures, the HBM roofline of the on-device kernels, the fraction of
the measured host-link ceiling, isolated per-request preempt/resume latency and
the CPU oracle's rate are reported in the same JSON line.
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

# HBM bytes per on-device launch of the default workload, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs of this script (summary and scale factors: profiles/kv_move_kernel_llama8b_burst64.md):
# (18 602 483 + 18 601 139) KiB for the scatter, against 2 x 18 601 984 KiB algorithmic.
MEASURED_TRAFFIC = {("configs[1]", 9083, "scatter"): (18602495 + 18601208) * 1024,
                    ("configs[1]", 9083, "scatter_plane_by_plane"): (18603478 + 18601147) * 1024,
                    ("configs[1]", 9083, "gather"): (18606378 + 18601147) * 1024}


def pct(xs, q):
    return float(np.percentile(np.asarray(xs, dtype=np.float64), q))


def cpu_baseline(W, wl, lens, off, ids, n_sample):
    """The oracle, as it stands, on the first n_sample requests of the burst: swap-out then
    swap-in against a compact host mirror holding only the blocks involved."""
    from oracle import kv_oracle as ko
    g0 = wl.geom
    rows = list(range(n_sample))
    soff, sids = W.csr_take(off, ids, rows)
    total = int(soff[-1])
    g = W.Geometry(g0.L, g0.H, g0.D, g0.B, g0.dtype, 2 * total)
    unit = W.fill_buffer_np(wl.seed, 1 << 24, g.dtype)
    pool = np.resize(unit, g.pool_bytes)
    staging = np.zeros(total * g.S, dtype=np.uint8)
    ora = ko.Oracle(g.L, g.H, g.D, g.B, g.e, g.N, pool, g.strides, staging)
    rid = np.arange(1, n_sample + 1, dtype=np.uint64)
    src = np.arange(total, dtype=np.int32)          # compact ids, same order as the real tables
    dst = np.arange(total, 2 * total, dtype=np.int32)
    t_out = t_in = 0.0
    passes = 2                                      # there and back again: about 10 s of CPU work
    for k in range(passes):
        a, b = (src, dst) if k % 2 == 0 else (dst, src)
        t0 = time.perf_counter()
        assert ora.swap_out(rid, soff, a, lens[:n_sample]) == ko.OK
        t1 = time.perf_counter()
        assert ora.swap_in(rid, soff, b) == ko.OK
        t2 = time.perf_counter()
        t_out += t1 - t0
        t_in += t2 - t1
    nbytes = passes * total * g.S
    return {
        "value": round(2 * nbytes / (t_out + t_in) / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": "first %d of the 64 requests (%d blocks, %.2f GiB each way), %d passes of swap-out then swap-in on a "
                  "compact host mirror; %.1f s of CPU time" % (n_sample, total, total * g.S / 2**30, passes, t_out + t_in),
        "swap_out_gbps": round(nbytes / t_out / 1e9, 3), "swap_in_gbps": round(nbytes / t_in / 1e9, 3),
        "ms_per_request": round((t_out + t_in) * 1e3 / (passes * n_sample), 2),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--path", choices=["auto", "zerocopy", "dma"], default="auto")
    ap.add_argument("--cpu-sample", type=int, default=40, help="requests the CPU oracle is timed on (0: skip)")
    ap.add_argument("--blocks", type=int, default=0, help="override the pool size (debugging on small boxes)")
    ap.add_argument("--variant", type=int, default=0, help="0: the configuration's own seed; 1, 2: further seeds")
    ap.add_argument("--pool-last", action="store_true", help="allocate the pool after the other device buffers")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a one-GPU library (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not os.path.exists(os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2510_02758_amd", "libkvswap.so")):
        import __graft_entry__          # load what is built; build only a tree in which nothing is
        __graft_entry__.build()
    from paper_2510_02758_amd import kvswap as kv
    from paper_2510_02758_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    wl = W.config(2, num_blocks=args.blocks or None, variant=args.variant)
    g = wl.geom
    lens = W.request_lengths(wl.seed, wl.n_requests, wl.length_dist)
    nb = W.blocks_for(lens, g.B)
    off, ids, free = W.block_tables(wl.seed, g.N, nb)
    n = wl.n_requests
    total = int(off[-1])
    rid = np.arange(1, n + 1, dtype=np.uint64)
    new = free[:total].copy()                     # fresh blocks for the swap-in
    extra = free[total:total + n].copy()          # one more block per request for the write-through leg
    # tables after the requests grew by one block
    off2 = off + np.arange(n + 1, dtype=np.int32)
    ids2 = np.concatenate([np.append(new[off[i]:off[i + 1]], extra[i]) for i in range(n)]).astype(np.int32)
    lens2 = ((nb + 1) * g.B).astype(np.int32)

    # ---- memory: PyTorch only allocates ----
    # Where in device memory the driver puts the pool decides how fast scattered writes into it go (the
    # on-device kernels); --pool-last allocates it after the other device buffers, as a server does after its weights.
    if args.pool_last:
        dev_arena = torch.empty(total * g.S, dtype=torch.uint8, device=dev)
        bounce = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device=dev)
    W.fill_buffer_torch(wl.seed, pool, g.dtype)
    if not args.pool_last:
        dev_arena = torch.empty(total * g.S, dtype=torch.uint8, device=dev)
        bounce = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    staging = torch.empty((total + n) * g.S, dtype=torch.uint8, pin_memory=True)
    staging.view(torch.int64)[::512] = 0          # touch every page before timing
    flags = {"auto": kv.KV_PATH_AUTO, "zerocopy": kv.KV_PATH_ZEROCOPY, "dma": kv.KV_PATH_DMA}[args.path]
    kdma = kv.KVPool(g, pool, staging, bounce=bounce, flags=kv.KV_PATH_DMA)   # the other path, reported beside
    evict, load = torch.cuda.Stream(), torch.cuda.Stream()
    kp = kv.KVPool(g, pool, staging, bounce=bounce if args.path == "dma" else None, flags=flags,
                   evict_stream=evict, load_stream=load)
    kd = kv.KVPool(g, pool, dev_arena, flags=kv.KV_STAGING_DEVICE, evict_stream=evict, load_stream=load)
    torch.cuda.synchronize()

    # ---- ceilings, measured in this run ----
    one = 1 << 30
    scratch = dev_arena[:4 * one] if dev_arena.numel() >= 8 * one else None
    link_d2h = one / kv.kv_bench_link(staging.data_ptr(), dev_arena.data_ptr(), one, 0, 4, evict.cuda_stream) / 1e6
    link_h2d = one / kv.kv_bench_link(staging.data_ptr(), dev_arena.data_ptr(), one, 1, 4, evict.cuda_stream) / 1e6
    link_bidir = None
    if staging.numel() >= 2 * one and dev_arena.numel() >= 2 * one:
        # best of three: which copy engines the runtime picks for the two directions varies from try to try
        ms = [kv.kv_bench_link_bidir(staging.data_ptr(), dev_arena.data_ptr(), staging.data_ptr() + one,
                                     dev_arena.data_ptr() + one, one, 3) for _ in range(3)]
        link_bidir = 2 * one / min(ms) / 1e6 if min(ms) > 0 else None
    copy_gbs = None
    if scratch is not None:
        # 16 GiB of plain copy first: the memory clocks take some hundred milliseconds of load to come up
        kv.kv_bench_copy(dev_arena[4 * one:].data_ptr(), scratch.data_ptr(), 4 * one, 0, 40, evict.cuda_stream)
        ms = kv.kv_bench_copy(dev_arena[4 * one:].data_ptr(), scratch.data_ptr(), 4 * one, 0, 5, evict.cuda_stream)
        copy_gbs = 2 * 4 * one / ms / 1e6
        # the 16 KiB-piece shape, kept under its own kernel name as the known-size reference of the counter runs
        kv.kv_bench_copy(dev_arena[4 * one:].data_ptr(), scratch.data_ptr(), 4 * one, 1 << 18, 2, evict.cuda_stream)

    def ok(rc, what):
        if rc != kv.KV_OK:
            raise kv.KVSwapError(rc, what)

    acc = {k: [] for k in ("out", "in", "delta", "dev", "gather_k", "scatter_k", "out_k", "in_k", "plan_us")}
    scatter_orders = []      # job order the library chose for the on-device scatter of each timed step
    delta_blocks = [0]

    def step(record):
        t = [time.perf_counter()]
        for i in range(n):
            ok(kp.reserve(rid[i], int(nb[i]) + 1), "kv_req_reserve")
        ok(kp.swap_out(rid, off, ids, lens), "kv_swap_out")
        so = kp.stats() if record else None
        ok(kp.sync(), "kv_sync")
        t.append(time.perf_counter())
        ok(kp.swap_in(rid, off, new, kv.KV_KEEP_STAGING), "kv_swap_in")
        si = kp.stats() if record else None
        ok(kp.sync(), "kv_sync")
        t.append(time.perf_counter())
        rc, moved = kp.swap_out_delta(rid, off2, ids2, lens2)
        ok(rc, "kv_swap_out_delta")
        ok(kp.sync(), "kv_sync")
        t.append(time.perf_counter())
        delta_blocks[0] = int(moved.sum())
        ok(kd.swap_out(rid, off, new, lens), "kv_swap_out(device arena)")
        go = kd.stats() if record else None
        ok(kd.swap_in(rid, off, ids), "kv_swap_in(device arena)")
        gi = kd.stats() if record else None
        ok(kd.sync(), "kv_sync")
        t.append(time.perf_counter())
        for i in range(n):
            ok(kp.release(rid[i]), "kv_req_release")
        if record:
            acc["out"].append(t[1] - t[0])
            acc["in"].append(t[2] - t[1])
            acc["delta"].append(t[3] - t[2])
            acc["dev"].append(t[4] - t[3])
            acc["out_k"].append(so["ms_kernel"] if so["path"] == kv.KV_PATH_ZEROCOPY else so["ms_total"])
            acc["in_k"].append(si["ms_kernel"] if si["path"] == kv.KV_PATH_ZEROCOPY else si["ms_total"])
            acc["gather_k"].append(go["ms_kernel"])
            acc["scatter_k"].append(gi["ms_kernel"])
            scatter_orders.append(gi["scatter_order"])
            acc["plan_us"].append(so["plan_us"])

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    path_used = {kv.KV_PATH_DMA: "dma", kv.KV_PATH_ZEROCOPY: "zerocopy"}

    # ---- the on-device kernels back to back (inside a step they run once, right after ~0.7 s of
    # link-bound work, and their first launch is ~8 % slower than the following ones) ----
    steady = []
    for rep in range(4):
        ok(kd.swap_out(rid, off, new, lens), "kv_swap_out(device arena)")
        go = kd.stats()
        ok(kd.swap_in(rid, off, ids), "kv_swap_in(device arena)")
        gi = kd.stats()
        ok(kd.sync(), "kv_sync")
        if rep:
            steady.append((go["ms_kernel"], gi["ms_kernel"]))

    # ---- check that nothing was skipped: the pool is back where it started ----
    # (block new[j] holds what block ids[j] was filled with; untouched blocks hold their own fill)
    rng = np.random.default_rng(1)
    ls, ks, bs = g.strides
    bad = 0
    js = rng.choice(total, size=12, replace=False).tolist()
    pairs = [(int(new[j]), int(ids[j])) for j in js] + [(int(ids[j]), int(ids[j])) for j in js[:4]]
    pairs += [(int(p), int(p)) for p in rng.choice(free[total + n:], size=4)]
    for holder, origin in pairs:
        for l in (0, g.L // 2, g.L - 1):
            for c in (0, 1):
                want = W.fill_bytes_torch(wl.seed, l * ls + c * ks + origin * bs, g.chunk, g.dtype, dev)
                o = l * ls + c * ks + holder * bs
                bad += int((pool[o:o + g.chunk] != want).any())
    if bad:
        print("bench.py: pool content check FAILED on %d chunks" % bad, file=sys.stderr)
        sys.exit(3)

    # ---- isolated per-request preempt / resume latency (call -> kv_sync), outside the timed steps ----
    pre, res = [], []
    for i in range(n):
        o1 = np.array([0, nb[i]], dtype=np.int32)
        a = time.perf_counter()
        ok(kp.swap_out(rid[i:i + 1], o1, ids[off[i]:off[i + 1]], lens[i:i + 1]), "kv_swap_out")
        ok(kp.sync(), "kv_sync")
        b = time.perf_counter()
        ok(kp.swap_in(rid[i:i + 1], o1, ids[off[i]:off[i + 1]]), "kv_swap_in")
        ok(kp.sync(), "kv_sync")
        c = time.perf_counter()
        pre.append((b - a) * 1e3)
        res.append((c - b) * 1e3)
    sstat = kp.stats()

    # ---- per-request completion inside the burst (KV_REQ_EVENTS), outside the timed steps ----
    kev = kv.KVPool(g, pool, staging, flags=flags | kv.KV_REQ_EVENTS, evict_stream=evict, load_stream=load)
    ok(kev.swap_out(rid, off, ids, lens), "kv_swap_out(events)")
    _, t_out = kev.timeline()
    ev_out_total = kev.stats()["ms_total"]
    ok(kev.swap_in(rid, off, ids), "kv_swap_in(events)")
    _, t_in = kev.timeline()
    ev_in_total = kev.stats()["ms_total"]
    ok(kev.sync(), "kv_sync")
    kev.close()

    # ---- the copy-engine path on the same burst, for comparison (outside the timed steps) ----
    dma = {}
    for rep in range(2):
        a = time.perf_counter()
        ok(kdma.swap_out(rid, off, ids, lens), "kv_swap_out(dma)")
        ok(kdma.sync(), "kv_sync")
        b = time.perf_counter()
        ok(kdma.swap_in(rid, off, ids), "kv_swap_in(dma)")
        ok(kdma.sync(), "kv_sync")
        c = time.perf_counter()
        dma = {"d2h_gbps": round(total * g.S / (b - a) / 1e9, 2), "h2d_gbps": round(total * g.S / (c - b) / 1e9, 2)}

    P = total * g.S                              # payload of the burst, bytes
    Pd = delta_blocks[0] * g.S
    m = {k: float(np.mean(v)) for k, v in acc.items()}
    d2h = P / m["out"] / 1e9
    h2d = P / m["in"] / 1e9
    link_payload = 2 * P + Pd
    value = link_payload * args.steps / elapsed / 1e9
    gather_ms, scatter_ms = m["gather_k"], m["scatter_k"]
    # the handle times both job orders of a large on-device scatter on its first two calls (the warm-up steps)
    # and keeps the faster one for the pool it was given: 0 block by block, 1 plane by plane
    plane_major = 2 * sum(o == 1 for o in scatter_orders) > len(scatter_orders)
    scatter_gbs = 2 * P / scatter_ms / 1e6
    gather_gbs = 2 * P / gather_ms / 1e6

    out = {
        "metric": "swap GB/s (D2H, H2D, on-device) + p50 preempt/resume latency per request",
        "value": round(value, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed * 1e3 / args.steps, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-3-8B-shaped KV bf16 L32 H8 D128 B16, %d-block pool, burst of %d "
                               "requests 512-4096 tokens (%d blocks, %.2f GiB per direction), random block tables"
                               % (g.N, n, total, P / 2**30),
                   "seed": "0x%X" % wl.seed,
                   "path": path_used.get(sstat["path"], str(sstat["path"])),
                   "value_def": "host-link payload (swap-out + swap-in + write-through delta) per step / step wall "
                                "time, step = swap-out, swap-in, delta, on-device gather+scatter, release"},
        "legs": {
            "d2h_gbps": round(d2h, 2), "h2d_gbps": round(h2d, 2),
            "d2h_frac_of_measured_link": round(d2h / link_d2h, 3), "h2d_frac_of_measured_link": round(h2d / link_h2d, 3),
            "delta_blocks": delta_blocks[0], "delta_ms": round(m["delta"] * 1e3, 3),
            "delta_gbps": round(Pd / m["delta"] / 1e9, 2),
            "ondevice_payload_gbps": round(2 * P / m["dev"] / 1e9, 1),
            "ondevice_gather_traffic_gbps": round(gather_gbs, 1), "ondevice_scatter_traffic_gbps": round(scatter_gbs, 1),
            "ondevice_back_to_back_traffic_gbps": {
                "gather": round(2 * P / float(np.mean([x[0] for x in steady])) / 1e6, 1),
                "scatter": round(2 * P / float(np.mean([x[1] for x in steady])) / 1e6, 1)},
            "plan_us_burst": round(m["plan_us"], 1),
            "burst_preempt_ms_per_request": round(m["out"] * 1e3 / n, 3),
            "burst_resume_ms_per_request": round(m["in"] * 1e3 / n, 3),
            "other_path_dma": dma,
        },
        "latency": {"p50_preempt_ms": round(pct(pre, 50), 3), "p90_preempt_ms": round(pct(pre, 90), 3),
                    "p50_resume_ms": round(pct(res, 50), 3), "p90_resume_ms": round(pct(res, 90), 3),
                    "def": "isolated single-request call -> kv_sync, over the 64 requests (mean %.0f MiB each)"
                           % (P / n / 2**20),
                    "in_burst": {"p50_preempt_ms": round(pct(t_out, 50), 2), "p50_resume_ms": round(pct(t_in, 50), 2),
                                 "last_preempt_ms": round(float(t_out[-1]), 2), "last_resume_ms": round(float(t_in[-1]), 2),
                                 "burst_ms_with_events": [round(ev_out_total, 2), round(ev_in_total, 2)],
                                 "def": "stream time from the start of the 64-request call to each request's own "
                                        "completion event (KV_REQ_EVENTS, one launch per request)"}},
        "link": {"bound": "host-link", "measured_peak_d2h_gbps": round(link_d2h, 2),
                 "measured_peak_h2d_gbps": round(link_h2d, 2),
                 "measured_peak_bidirectional_gbps": None if link_bidir is None else round(link_bidir, 2),
                 "kernel_out_ms": round(m["out_k"], 2), "kernel_in_ms": round(m["in_k"], 2),
                 "how": "one 1 GiB contiguous pinned hipMemcpyAsync per direction, in this run"},
        "roofline_link": {"bound": "host-link", "kernel": "kv_move_kernel<0,4,1,true,false> (burst swap-out; the longest launch "
                          "of a step, bound by the host link and not by HBM)",
                          "achieved": round(P / m["out_k"] / 1e6, 2), "peak": 64.0, "unit": "GB/s",
                          "frac": round(P / m["out_k"] / 1e6 / 64.0, 4), "launch_ms": round(m["out_k"], 2),
                          "bytes_per_launch": P, "measured_peak": round(link_d2h, 2),
                          "frac_of_measured_peak": round(P / m["out_k"] / 1e6 / link_d2h, 4),
                          "peak_def": "PCIe Gen5 x16, 64 GB/s raw per direction; measured_peak = one contiguous "
                                      "hipMemcpyAsync in this run"},
        "roofline": {"bound": "hbm",
                     "kernel": ("kv_move_kernel<1,1,0,true,true> (scatter plane by plane, both ends in HBM)" if plane_major
                                else "kv_move_kernel<1,1,0,true,false> (scatter block by block, both ends in HBM)"),
                     "scatter_order_per_step": scatter_orders,
                     "achieved": round(scatter_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(scatter_gbs / HBM_PEAK_GBS, 4),
                     "traffic": (MEASURED_TRAFFIC.get(("configs[1]", total, "scatter_plane_by_plane" if plane_major else "scatter"))
                                 if not args.blocks else None),
                     "launch_ms": round(scatter_ms, 3), "bytes_per_launch": 2 * P,
                     "measured_copy_ceiling_gbps": None if copy_gbs is None else round(copy_gbs, 1)},
        "roofline_gather": {"bound": "hbm", "kernel": "kv_move_kernel<0,1,0,true,false> (gather, both ends in HBM)",
                            "achieved": round(gather_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": round(gather_gbs / HBM_PEAK_GBS, 4),
                            "traffic": MEASURED_TRAFFIC.get(("configs[1]", total, "gather")) if not args.blocks else None,
                            "launch_ms": round(gather_ms, 3),
                            "bytes_per_launch": 2 * P},
    }
    kp.close()
    kd.close()
    kdma.close()
    del pool, dev_arena
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(W, wl, lens, off, ids, min(args.cpu_sample, n))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
