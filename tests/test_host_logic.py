"""CPU tests of the GPU library's host side: the shared object loads, exports what
include/kvswap.h declares, and — under KV_PLAN_ONLY, where it never touches HIP —
its request table, extent allocator, validation and descriptor lists satisfy the
same pins as the oracle and agree with the oracle on random operation sequences.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import test_oracle_pins as T
from adapters import PlanOnlyAdapter
from hostpool import HostPool
from oracle import kv_oracle as ko
from paper_2510_02758_amd import kvswap as kv
from paper_2510_02758_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    from paper_2510_02758_amd import kvsched as ks
    lib = ctypes.CDLL(kv.LIB_PATH)
    for header, exports in (("kvswap.h", kv.EXPORTS), ("kvsched.h", ks.EXPORTS)):
        hdr = open(os.path.join(ROOT, "include", header)).read()
        hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
        declared = set(re.findall(r"\b(kv_[a-z_0-9]+)\s*\(", hdr))
        assert declared, header
        for name in sorted(declared):
            assert hasattr(lib, name), "libkvswap.so does not export %s" % name
        assert set(exports) == declared, header
    assert {"kv_pool_create", "kv_swap_out", "kv_swap_out_delta", "kv_swap_in", "kv_sync"} <= set(kv.EXPORTS)
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["kvsched.h", "kvswap.h"]


def test_status_codes_match_header():
    hdr = open(os.path.join(ROOT, "include", "kvswap.h")).read()
    for name, val in re.findall(r"\b(KV_E[A-Z]+) = (-\d+)", hdr):
        assert getattr(kv, name) == int(val)
    # the oracle types the same numbers out on its own
    assert (ko.EINVAL, ko.ERANGE, ko.EDUP, ko.ENOENT, ko.EEXIST, ko.ENOSPC, ko.ESTATE) == \
        (kv.KV_EINVAL, kv.KV_ERANGE, kv.KV_EDUP, kv.KV_ENOENT, kv.KV_EEXIST, kv.KV_ENOSPC, kv.KV_ESTATE)
    assert kv.kv_strerror(kv.KV_EDUP) == "duplicate destination block"


def test_create_rejects_bad_configs():
    g = W.Geometry(2, 4, 64, 16, "f16", 64)

    def make(**kw):
        cfg = kv.kv_pool_config()
        cfg.num_layers, cfg.num_kv_heads, cfg.head_dim, cfg.block_size = g.L, g.H, g.D, g.B
        cfg.dtype, cfg.num_blocks = 0, g.N
        cfg.layer_stride, cfg.kv_stride, cfg.block_stride = g.strides
        cfg.staging_bytes = 10 * g.S
        cfg.flags = kv.KV_PLAN_ONLY
        for k, v in kw.items():
            setattr(cfg, k, v)
        rc, h = kv.kv_pool_create(cfg)
        if rc == kv.KV_OK:
            kv.kv_pool_destroy(h)
        return rc

    assert make() == kv.KV_OK
    assert make(num_layers=0) == kv.KV_EINVAL
    assert make(dtype=7) == kv.KV_EINVAL
    assert make(head_dim=3, block_size=1) == kv.KV_EINVAL  # chunk not a multiple of 16 bytes
    assert make(block_stride=g.chunk + 8) == kv.KV_EINVAL
    assert make(kv_stride=0) == kv.KV_EINVAL
    assert make(flags=kv.KV_PLAN_ONLY | kv.KV_PATH_DMA | kv.KV_PATH_ZEROCOPY) == kv.KV_EINVAL
    assert make(flags=kv.KV_PLAN_ONLY | kv.KV_PATH_DMA) == kv.KV_EINVAL  # DMA path without a bounce buffer
    assert make(scale_layer_stride=2 * 64 * 16, scale_kv_stride=64 * 16, scale_block_stride=16) == kv.KV_OK
    assert make(scale_layer_stride=2 * 64 * 16, scale_kv_stride=64 * 16, scale_block_stride=18) == kv.KV_EINVAL
    # a real (non plan-only) pool needs memory
    assert make(flags=0) == kv.KV_EINVAL


# ---- the oracle's pins, run against planner + descriptor lists -----------------
@pytest.mark.parametrize("layout", T.LAYOUTS)
@pytest.mark.parametrize("gname", list(T.GEOMS))
def test_pins_closed_form(gname, layout):
    T.pin_closed_form(gname, layout, lib=PlanOnlyAdapter)


@pytest.mark.parametrize("gname", list(T.GEOMS))
def test_pins_round_trip(gname):
    T.pin_round_trip(gname, "padded", lib=PlanOnlyAdapter)


@pytest.mark.parametrize("gname", list(T.GEOMS))
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_pins_delta(gname, seed):
    T.pin_delta_equals_full(gname, seed, lib=PlanOnlyAdapter)


def test_pins_rest():
    T.pin_brute_force(2, 2, lib=PlanOnlyAdapter, D=8)
    T.pin_memcpy_case("tiny", lib=PlanOnlyAdapter)
    T.pin_errors(lib=PlanOnlyAdapter)
    T.pin_move_blocks(lib=PlanOnlyAdapter)
    T.pin_first_fit(lib=PlanOnlyAdapter)
    T.pin_cycles(lib=PlanOnlyAdapter)


# ---- random operation sequences: library bookkeeping == oracle bookkeeping ------
@pytest.mark.parametrize("seed", range(6))
def test_random_sequences_agree_with_oracle(seed):
    g = W.Geometry(2, 2, 8, 4, "bf16", 48, scales=(seed % 2 == 1))
    a = HostPool(g, 77 + seed, slots=26)
    b = HostPool(g, 77 + seed, slots=26)
    ora, lib = a.oracle(), PlanOnlyAdapter(b)
    rng = np.random.default_rng(seed)
    ids = list(range(1, 9))
    length = {r: 0 for r in ids}
    table = {r: [] for r in ids}
    free = list(rng.permutation(g.N))
    resident = {r: True for r in ids}
    codes = {}
    for step in range(400):
        op = rng.choice(["grow", "out", "delta", "delta_tail", "in", "in_keep", "reserve", "release", "bad"])
        k = int(rng.integers(1, 4))
        rs = [int(x) for x in rng.choice(ids, size=k, replace=False)]
        if op == "grow":
            for r in rs:
                if resident[r]:
                    length[r] += int(rng.integers(1, 3 * g.B))
                    while len(table[r]) * g.B < length[r] and free:
                        table[r].append(int(free.pop()))
                    length[r] = min(length[r], len(table[r]) * g.B)
            continue
        off = np.zeros(len(rs) + 1, np.int32)
        off[1:] = np.cumsum([len(table[r]) for r in rs])
        flat = [x for r in rs for x in table[r]]
        lens = [length[r] for r in rs]
        if op == "out":
            ra, rb = ora.swap_out(rs, off, flat, lens), lib.swap_out(rs, off, flat, lens)
        elif op in ("delta", "delta_tail"):
            bud = int(rng.integers(0, 5))
            fl = ko.DELTA_INCLUDE_TAIL if op == "delta_tail" else 0
            (ra, ma), (rb, mb) = ora.swap_out_delta(rs, off, flat, lens, bud, fl), \
                lib.swap_out_delta(rs, off, flat, lens, bud, fl)
            assert np.array_equal(ma, mb)
        elif op in ("in", "in_keep"):
            staged = [ora.query(r)[1]["staged"] if ora.query(r)[0] == 0 else 1 for r in rs]
            need = sum(staged)
            if need > len(free):
                continue
            dest = [int(free.pop()) for _ in range(need)]
            off = np.zeros(len(rs) + 1, np.int32)
            off[1:] = np.cumsum(staged)
            fl = ko.KEEP_STAGING if op == "in_keep" else 0
            ra, rb = ora.swap_in(rs, off, dest, fl), lib.swap_in(rs, off, dest, fl)
            if ra == 0:
                at = 0
                for r, n in zip(rs, staged):
                    free = table[r] + free
                    table[r] = dest[at:at + n]
                    at += n
                    if not fl:
                        pass
            else:
                free = dest + free
        elif op == "reserve":
            n = int(rng.integers(0, 6))
            ra, rb = ora.reserve(rs[0], n), lib.reserve(rs[0], n)
        elif op == "release":
            ra, rb = ora.release(rs[0]), lib.release(rs[0])
        else:  # a call with one bad block id somewhere
            if not flat:
                continue
            flat = list(flat)
            flat[int(rng.integers(len(flat)))] = g.N + 3
            ra, rb = ora.swap_out(rs, off, flat, lens), lib.swap_out(rs, off, flat, lens)
        assert ra == rb, (step, op, ra, rb)
        codes[ra] = codes.get(ra, 0) + 1
        for r in ids:
            assert ora.query(r) == lib.query(r), (step, op, r)
        assert np.array_equal(a.staging, b.staging), (step, op)
        assert np.array_equal(a.pool, b.pool), (step, op)
        if g.scales:
            assert np.array_equal(a.scale, b.scale)
    assert codes.get(0, 0) > 50 and len(codes) >= 4, codes  # successes and several error kinds were hit


def test_plan_is_in_call_order():
    g = W.Geometry(1, 1, 8, 2, "f16", 32)
    kp = kv.KVPool(g, flags=kv.KV_PLAN_ONLY, staging_bytes=16 * g.S)
    assert kp.swap_out([7, 3], [0, 2, 5], [9, 4, 1, 0, 30], [4, 5]) == kv.KV_OK
    phys, slot = kp.last_plan()
    assert phys.tolist() == [9, 4, 1, 0, 30] and slot.tolist() == [0, 1, 2, 3, 4]
    st = kp.stats()
    assert st["blocks"] == 5 and st["bytes"] == 5 * g.S and st["op"] == 1
    rc, moved = kp.swap_out_delta([5], [0, 3], [11, 12, 13], [5], flags=kv.KV_DELTA_INCLUDE_TAIL)
    assert rc == kv.KV_OK and moved.tolist() == [3]
    phys, slot = kp.last_plan()
    assert phys.tolist() == [11, 12, 13] and slot.tolist() == [5, 6, 7]
    assert kp.swap_in([3], [0, 3], [20, 21, 22]) == kv.KV_OK
    phys, slot = kp.last_plan()
    assert phys.tolist() == [20, 21, 22] and slot.tolist() == [2, 3, 4]
    kp.close()


def test_budget_formula_without_measurements():
    """Under KV_PLAN_ONLY nothing is ever measured: the budget uses the documented defaults
    (32 GB/s, 50 us fixed cost)."""
    g = W.Geometry(32, 8, 128, 16, "bf16", 64)
    kp = kv.KVPool(g, flags=kv.KV_PLAN_ONLY, staging_bytes=16 * g.S)
    io = kp.io_stats()
    assert io["inflight_calls"] == [0, 0] and io["ewma_gbps"] == [0.0, 0.0]
    for d in (0, 1):
        assert kp.budget_blocks(d, 0.0) == 0 and kp.budget_blocks(d, 50.0) == 0
        assert kp.budget_blocks(d, 1050.0) == int(1000.0 * 32.0 * 1e3 / g.S)      # 1 ms of link time
    assert kp.budget_blocks(2, 100.0) == kv.KV_EINVAL
    kp.close()


def test_timed_delta_orders_by_priority_and_applies_the_budget():
    """Section 5.2: larger buffers first, sized to the interval.  Plan-only: rate 32 GB/s, fixed
    50 us, so the budget is known in closed form; the oracle, given the same order and budget,
    must stage the same bytes."""
    g = W.Geometry(1, 1, 8, 2, "f16", 64)                   # S = 64 bytes
    a = HostPool(g, 5, slots=20)
    b = HostPool(g, 5, slots=20)
    ora, lib = a.oracle(), PlanOnlyAdapter(b)
    rid = [10, 11, 12]
    off = [0, 4, 8, 13]
    blk = list(range(20, 33))
    tok = [8, 8, 9]                                          # 4, 4 and 4 full blocks (+ a tail for the third)
    prio = [1.0, 3.0, 2.0]
    interval = 50.011                                        # (50.011 - 50) us * 32 GB/s / 64 B = 5.5 -> 5 blocks
    rc, moved, used = lib.kp.swap_out_delta_timed(rid, off, blk, tok, prio, interval)
    assert rc == kv.KV_OK and used == 5
    assert moved.tolist() == [0, 4, 1]                       # request 11 first, then 12, nothing left for 10
    phys, slot = lib.kp.last_plan()
    assert phys.tolist() == [24, 25, 26, 27, 28]
    lib._apply_out()
    order = [1, 2, 0]
    o2, b2 = W.csr_take(np.array(off, np.int32), np.array(blk, np.int32), order)
    rc, m2 = ora.swap_out_delta([rid[i] for i in order], o2, b2, [tok[i] for i in order], budget=5)
    assert rc == ko.OK and m2.tolist() == [4, 1, 0]
    assert np.array_equal(a.staging, b.staging)
    for r in rid:
        assert ora.query(r) == lib.query(r)
    # an interval shorter than the fixed cost: nothing moves, nothing changes
    rc, moved, used = lib.kp.swap_out_delta_timed(rid, off, blk, tok, prio, 10.0)
    assert rc == kv.KV_OK and used == 0 and not moved.any()
    for r in rid:
        assert ora.query(r) == lib.query(r)
    # no priorities: call order; a long interval moves everything that is full
    rc, moved, used = lib.kp.swap_out_delta_timed(rid, off, blk, tok, None, 1e6)
    assert rc == kv.KV_OK and moved.tolist() == [4, 0, 3] and used > 1000
    # errors pass through unchanged
    rc, _, _ = lib.kp.swap_out_delta_timed(rid, off, [999] * 13, tok, prio, 100.0)
    assert rc == kv.KV_ERANGE
    rc, _, _ = lib.kp.swap_out_delta_timed(rid, off, blk, tok, prio, -1.0)
    assert rc == kv.KV_EINVAL


# ------------------------------------------------------------------ write queue (Section 5.2)
def test_write_queue_drains_by_priority_under_a_budget():
    """kv_wq_post + kv_wq_drain is one kv_swap_out_delta over the queued requests in priority order:
    the oracle, handed that order and that budget, must reach the same bytes and the same request state."""
    g = W.Geometry(1, 1, 8, 2, "f16", 64)
    a, b = HostPool(g, 6, slots=24), HostPool(g, 6, slots=24)
    ora, lib = a.oracle(), PlanOnlyAdapter(b)
    kp = lib.kp
    rid, off, blk, tok = [10, 11, 12], [0, 4, 8, 13], list(range(20, 33)), [8, 8, 9]
    for o in (ora, lib):                                    # extents are reserved up front, as for any write-through
        assert o.reserve(12, 8) == 0 and o.reserve(10, 8) == 0
    assert kp.wq_post(rid, off, blk, tok, [1.0, 3.0, 2.0]) == kv.KV_OK
    assert kp.wq_pending() == (kv.KV_OK, 12, 3)
    rc, wrote, pend, used = kp.wq_drain(block_budget=5)
    assert (rc, wrote, pend, used) == (kv.KV_OK, 5, 7, 5)
    phys, slot = kp.last_plan()
    assert phys.tolist() == [24, 25, 26, 27, 28]            # request 11 whole, then one block of 12
    lib._apply_out()
    order = [1, 2, 0]
    o2, b2 = W.csr_take(np.array(off, np.int32), np.array(blk, np.int32), order)
    rc, m2 = ora.swap_out_delta([rid[i] for i in order], o2, b2, [tok[i] for i in order], budget=5)
    assert rc == ko.OK and m2.tolist() == [4, 1, 0]
    assert np.array_equal(a.staging, b.staging) and all(ora.query(r) == lib.query(r) for r in rid)
    # request 10 grows by two blocks and becomes the most urgent; the others keep their entries
    assert kp.wq_post([10], [0, 6], [20, 21, 22, 23, 40, 41], [12], [9.0]) == kv.KV_OK
    rc, wrote, pend, used = kp.wq_drain()                   # no budget: everything that is full
    assert (rc, wrote, pend) == (kv.KV_OK, 9, 0)
    lib._apply_out()
    rc, m3 = ora.swap_out_delta([10, 11, 12], [0, 6, 10, 15], [20, 21, 22, 23, 40, 41] + blk[4:], [12, 8, 9])
    assert rc == ko.OK and m3.tolist() == [6, 0, 3]
    assert np.array_equal(a.staging, b.staging) and all(ora.query(r) == lib.query(r) for r in rid)
    # an interval: plan-only rate 32 GB/s, fixed 50 us, 64-byte slots -> (50.005 - 50) us * 32e3 B/us / 64 = 2 blocks
    assert kp.wq_post([12], [0, 7], blk[8:] + [50, 51], [14], [0.5]) == kv.KV_OK          # 7 full blocks, 4 written
    rc, wrote, pend, used = kp.wq_drain(interval_us=50.005)
    assert (rc, wrote, pend, used) == (kv.KV_OK, 2, 1, 2)
    rc, wrote, pend, used = kp.wq_drain(interval_us=10.0)   # shorter than the fixed cost: nothing fits, nothing moves
    assert (rc, wrote, pend, used) == (kv.KV_OK, 0, 1, 0)
    kp.close()


def test_write_queue_entries_follow_the_requests():
    g = W.Geometry(1, 1, 8, 2, "f16", 64)
    kp = kv.KVPool(g, flags=kv.KV_PLAN_ONLY, staging_bytes=40 * g.S)
    assert kp.wq_post([1, 2, 3], [0, 2, 4, 6], [0, 1, 2, 3, 4, 5], [4, 4, 4]) == kv.KV_OK
    assert kp.wq_pending() == (kv.KV_OK, 6, 3)
    # a full swap-out, a release and a swap-in each take their requests out of the queue
    assert kp.swap_out([1], [0, 2], [0, 1], [4]) == kv.KV_OK
    assert kp.wq_pending() == (kv.KV_OK, 4, 2) and kp.wq_remove(1) == kv.KV_ENOENT
    rc, wrote, pend, _ = kp.wq_drain(block_budget=1)
    assert (rc, wrote, pend) == (kv.KV_OK, 1, 3)
    assert kp.release(2) == kv.KV_OK and kp.wq_pending() == (kv.KV_OK, 2, 1)
    assert kp.swap_in([1], [0, 2], [10, 11]) == kv.KV_OK
    assert kp.wq_remove(3) == kv.KV_OK and kp.wq_remove(3) == kv.KV_ENOENT
    assert kp.wq_drain() == (kv.KV_OK, 0, 0, 0)
    # rejected posts record nothing
    assert kp.wq_post([5, 5], [0, 1, 2], [0, 1], [2, 2]) == kv.KV_EINVAL                   # named twice
    assert kp.wq_post([5], [0, 1], [0], [4]) == kv.KV_EINVAL                               # 4 tokens need 2 blocks
    assert kp.wq_post([5], [0, 1], [64], [2]) == kv.KV_ERANGE
    assert kp.wq_post([5], [0, 1], [0], [2], [float("nan")]) == kv.KV_EINVAL
    assert kp.swap_out([6], [0, 1], [7], [2]) == kv.KV_OK
    assert kp.wq_post([6], [0, 1], [7], [2]) == kv.KV_EEXIST                               # swapped out
    assert kp.wq_pending() == (kv.KV_OK, 0, 0)
    # a drain that cannot be planned changes nothing: the arena has 40 slots
    assert kp.wq_post([8], [0, 60], list(range(60)), [120]) == kv.KV_OK
    rc, _, _, _ = kp.wq_drain()
    assert rc == kv.KV_ENOSPC and kp.wq_pending() == (kv.KV_OK, 60, 1) and kp.query(8)[0] == kv.KV_ENOENT
    assert kp.wq_drain(interval_us=-1.0)[0] == kv.KV_EINVAL and kp.wq_drain(block_budget=-1)[0] == kv.KV_EINVAL
    kp.close()


def test_a_queue_entry_that_a_direct_delta_has_overtaken_is_skipped():
    """A request posted with 4 tokens, then written through directly up to 8 tokens: its entry has nothing left to
    write.  The drain must serve the other requests, not fail with KV_ESTATE."""
    g = W.Geometry(1, 1, 8, 2, "f16", 64)
    kp = kv.KVPool(g, flags=kv.KV_PLAN_ONLY, staging_bytes=40 * g.S)
    assert kp.wq_post([1, 2], [0, 2, 4], [0, 1, 2, 3], [4, 4]) == kv.KV_OK
    rc, moved = kp.swap_out_delta([1], [0, 4], [0, 1, 8, 9], [8])
    assert rc == kv.KV_OK and list(moved) == [4]
    rc, wrote, pend, _ = kp.wq_drain()
    assert (rc, wrote, pend) == (kv.KV_OK, 2, 0)
    assert kp.query(1)[1]["wm"] == 4 and kp.query(2)[1]["wm"] == 2     # watermarks: untouched, written
    kp.close()


@pytest.mark.parametrize("seed", range(4))
def test_write_queue_random_against_oracle(seed):
    """Random growth, posts, budgets and preempt / resume cycles: after every drain the staged bytes and the
    per-request state equal the oracle's, which receives the same requests in the same priority order."""
    rng = np.random.default_rng(900 + seed)
    g = W.Geometry(2, 1, 8, 2, "f16", 96)
    a, b = HostPool(g, 40 + seed, slots=80), HostPool(g, 40 + seed, slots=80)
    ora, lib = a.oracle(), PlanOnlyAdapter(b)
    kp = lib.kp
    free = list(rng.permutation(g.N))
    table, length, prio, queued = {}, {}, {}, {}
    for r in range(1, 7):
        table[r], length[r] = [], 0
        for o in (ora, lib):
            assert o.reserve(r, 13) == 0                     # 6 x 13 of the 80 slots
    for step in range(120):
        grow = [r for r in table if rng.random() < 0.6]
        for r in grow:                                       # decode: a few more tokens, new blocks as needed
            length[r] = min(length[r] + int(rng.integers(1, 4)), 13 * g.B)
            while len(table[r]) * g.B < length[r] and free:
                table[r].append(int(free.pop()))
            length[r] = min(length[r], len(table[r]) * g.B)
            prio[r] = float(rng.integers(0, 4))
        if grow:
            off = np.concatenate([[0], np.cumsum([len(table[r]) for r in grow])]).astype(np.int32)
            blk = [x for r in grow for x in table[r]]
            assert kp.wq_post(grow, off, blk, [length[r] for r in grow], [prio[r] for r in grow]) == kv.KV_OK
            for r in grow:
                queued[r] = (list(table[r]), length[r], prio[r], step * 100 + grow.index(r))
        if rng.random() < 0.7:
            budget = int(rng.integers(0, 6))
            rc, wrote, pend, used = kp.wq_drain(block_budget=budget)
            assert rc == kv.KV_OK
            lib._apply_out()
            order = sorted(queued, key=lambda r: (-queued[r][2], queued[r][3]))
            if order:
                off = np.concatenate([[0], np.cumsum([len(queued[r][0]) for r in order])]).astype(np.int32)
                rc, moved = ora.swap_out_delta(order, off, [x for r in order for x in queued[r][0]],
                                               [queued[r][1] for r in order], budget=budget)
                assert rc == ko.OK and int(moved.sum()) == wrote
            assert np.array_equal(a.staging, b.staging)
            for r in table:
                assert ora.query(r) == lib.query(r)
            want = sum(max(0, queued[r][1] // g.B - (ora.query(r)[1]["wm"] if ora.query(r)[0] == 0 else 0)) for r in queued)
            assert pend == want
        if rng.random() < 0.15 and queued:                   # preempt one (tail flush) and bring it back elsewhere
            r = int(rng.choice(list(queued)))
            off = [0, len(table[r])]
            for o in (ora, lib):
                rc, _ = o.swap_out_delta([r], off, table[r], [length[r]], flags=kv.KV_DELTA_INCLUDE_TAIL)
                assert rc == 0
            new = [int(free.pop(0)) for _ in table[r]]
            free.extend(table[r])
            for o in (ora, lib):
                assert o.swap_in([r], off, new, kv.KV_KEEP_STAGING) == 0
            table[r] = new
            queued.pop(r)                                    # the library dropped its entry at the swap-in
    kp.close()


def test_duplicate_checks_on_a_pool_of_millions_of_blocks():
    """Token-level pools: short lists are checked by sorting, not with a bitmap over the whole pool.  Same answers."""
    g = W.Geometry(1, 1, 8, 1, "f16", 3_000_000)
    kp = kv.KVPool(g, flags=kv.KV_PLAN_ONLY, staging_bytes=4096 * g.S)
    rng = np.random.default_rng(3)
    blocks = rng.choice(g.N, size=600, replace=False).astype(np.int32)
    assert kp.swap_out([1], [0, 300], blocks[:300], [300]) == kv.KV_OK
    dup = blocks[300:600].copy()
    dup[17] = dup[250]
    assert kp.swap_in([1], [0, 300], dup) == kv.KV_EDUP
    assert kp.query(1)[1]["swapped"] == 1                       # nothing changed
    assert kp.swap_in([1], [0, 300], blocks[300:600]) == kv.KV_OK
    # moves: a repeated destination, a destination that is also a source, and a clean one
    src, dst = blocks[:100], blocks[100:200]
    bad = dst.copy(); bad[3] = bad[99]
    assert kp.move_blocks(src, bad) == kv.KV_EDUP
    bad = dst.copy(); bad[50] = src[7]
    assert kp.move_blocks(src, bad) == kv.KV_EDUP
    assert kp.move_blocks(src, dst) == kv.KV_OK
    phys, slot = kp.last_plan()
    assert phys.tolist() == src.tolist() and slot.tolist() == dst.tolist()
    # a long list on the same pool takes the bitmap again: same answers
    big = rng.choice(g.N, size=20000, replace=False).astype(np.int32)
    assert kp.move_blocks(big[:10000], big[10000:]) == kv.KV_OK
    bad = big[10000:].copy(); bad[5] = big[77]
    assert kp.move_blocks(big[:10000], bad) == kv.KV_EDUP
    kp.close()


def test_binding_fails_loudly_without_the_library(tmp_path):
    """No fallback path: a copy of the package without libkvswap.so must refuse to import."""
    import shutil
    import subprocess
    import sys
    pkg = tmp_path / "paper_2510_02758_amd"
    shutil.copytree(os.path.join(ROOT, "paper_2510_02758_amd"), pkg,
                    ignore=shutil.ignore_patterns("*.so", "__pycache__", "csrc"))
    code = ("import sys; sys.path.insert(0, %r)\n"
            "try:\n    import paper_2510_02758_amd.kvswap\n"
            "except ImportError as e:\n    print('refused:', e); sys.exit(7)\n"
            "sys.exit(0)\n" % str(tmp_path))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300, cwd=str(tmp_path))
    assert r.returncode == 7 and "libkvswap.so is not built" in r.stdout, r.stdout + r.stderr
    # the scheduler binding lives in the same library and refuses too
    code = code.replace("paper_2510_02758_amd.kvswap", "paper_2510_02758_amd.kvsched")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300, cwd=str(tmp_path))
    assert r.returncode == 7, r.stdout + r.stderr


def test_oracle_and_product_do_not_know_each_other():
    """The package (binding, workloads, simulator, native sources) never imports or includes the oracle, and the
    oracle never imports or includes the package: only tests, the smoke entry and the benchmark scripts at the repository root bring them together."""
    pkg = os.path.join(ROOT, "paper_2510_02758_amd")
    for d, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".inc", ".hpp", ".cpp", ".h")):
                text = open(os.path.join(d, f), errors="ignore").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b|#include\s+\"[^\"]*oracle", text, flags=re.M), \
                    "%s uses the oracle" % f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert not re.search(r"^\s*(from|import)\s+paper_2510_02758_amd", text, flags=re.M), f
            assert '#include "../paper' not in text and "csrc/" not in text.replace("paper_2510_02758_amd/csrc/scheduler.cpp", ""), f
    for f in os.listdir(os.path.join(ROOT, "include")):
        assert "oracle" not in open(os.path.join(ROOT, "include", f)).read()


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU benchmark: any other --gpus ends with a message and a non-zero status before
    anything touches a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0 and "one-GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_oracle_leg_runs_on_the_cpu():
    """The cpu_baseline leg of bench.py is the oracle and nothing else: it runs here, on a tiny sample, on one core and
    then once more with the sample's blocks cut over all cores."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_configs_module", os.path.join(ROOT, "bench_configs.py"))
    bc = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bc)
    g = W.Geometry(4, 8, 128, 16, "bf16", 64)
    lens = np.array([300, 520], np.int32)
    out = bc.oracle_rates(W, g, lens, W.blocks_for(lens, g.B), 2, 7, passes=2)
    assert out["kind"] == "oracle" and out["cores"] == 1 and out["unit"] == "GB/s" and out["value"] > 0
    assert "2 requests of the workload" in out["sample"]
    assert out["all_cores"] == min(out["host_cores"], 19 + 33) and out["all_cores_value"] > 0


def test_bench_waves_cover_every_request_once():
    """The wave split of the headline: in order, every request exactly once, each wave within the arena and the free list."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_configs_module", os.path.join(ROOT, "bench_configs.py"))
    bc = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bc)
    wl = W.config(4)
    nb = W.blocks_for(W.request_lengths(wl.seed, wl.n_requests, wl.length_dist), wl.geom.B)
    slots = (40 << 30) // wl.geom.S
    waves = bc.waves_of(nb, slots, room_per_request=1, limit_blocks=9000)
    assert np.array_equal(np.concatenate(waves), np.arange(128)) and len(waves) == 10
    for rows in waves:
        assert int((nb[rows] + 1).sum()) <= slots
    with pytest.raises(ValueError):
        bc.waves_of(nb, 100)


def test_bench_traffic_constants_are_the_profile_summarys():
    """bench.py reports `traffic` from per-block counter figures it carries as constants: they must be the numbers of the
    committed rocprofv3 summary, not a copy that has drifted."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    text = open(os.path.join(ROOT, bench.TRAFFIC_SOURCE)).read()
    rows = {"gather": "gather, HBM to HBM", "scatter_block_by_block": "scatter block by block, HBM to HBM",
            "scatter_plane_by_plane": "scatter plane by plane, HBM to HBM"}
    for key, label in rows.items():
        line = [ln for ln in text.splitlines() if label in ln and ln.startswith("| `kv_move_kernel")]
        assert len(line) == 1, key
        cells = [c.strip() for c in line[0].split("|")]
        assert (float(cells[3]), float(cells[4])) == tuple(bench.MEASURED_KIB_PER_BLOCK[key]), key
        assert abs((float(cells[3]) + float(cells[4])) / (2 * 5120) - 1) < 0.01      # nothing is moved twice
