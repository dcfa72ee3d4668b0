"""Pins of the CPU oracle against facts fixed outside of it.

The swap is a permutation copy, so its result has a plain definition
(Section 5 of the paper: preempt offloads a request's KV cache, resume reloads
it; Section 5.1: only KV newer than the previous offload is written).  The
pins below never re-run the oracle's loop; they check its output against
  1. the closed-form staging offset of every byte over an address-coded pool,
  2. round-trip identity,
  3. the untouched complement (pool and arena),
  4. delta write-through == one full swap-out,
  5. an element-level dictionary model under brute force on tiny pools,
  6. the block-major identity-table case, which is a single memcpy,
  7. the error table, each error leaving state and memory unchanged,
  8. a hand-worked first-fit placement example (tests/golden).
test_oracle_mutants.py plants mistakes in the oracle source and checks that
these pins notice each of them.
"""
import itertools
import os

import numpy as np
import pytest

from hostpool import CANARY, HostPool, sizes
from oracle import kv_oracle as ko
from paper_2510_02758_amd import workloads as W

GEOMS = {
    "tiny": W.Geometry(2, 4, 64, 16, "f16", 64),
    "odd": W.Geometry(3, 1, 24, 5, "bf16", 37),
    "fp8s": W.Geometry(2, 3, 16, 4, "fp8_e4m3", 29, scales=True),
}
LAYOUTS = ["layer", "block", "padded"]


def make_requests(seed, geom, n, lo, hi):
    lens = W.request_lengths(seed, n, ("uniform", lo, hi))
    off, ids, free = W.block_tables(seed, geom.N, W.blocks_for(lens, geom.B))
    return np.arange(100, 100 + n, dtype=np.uint64), lens, off, ids, free


# ---------------------------------------------------------------- pin 1
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("gname", list(GEOMS))
def pin_closed_form(gname, layout, lib=None):
    g = GEOMS[gname]
    hp = HostPool(g, 0xC0DE + len(gname), layout)
    pool0 = hp.pool.copy()
    ora = hp.oracle(lib)
    rid, lens, off, ids, _ = make_requests(7, g, 4, 1, 6 * g.B)
    assert ora.swap_out(rid, off, ids, lens) == ko.OK
    # fresh arena + first fit: request i starts right after request i-1
    bases = off[:-1].astype(np.int64)
    sv = hp.slots_view()
    for i in range(len(rid)):
        row = ids[off[i]:off[i + 1]]
        rc, q = ora.query(rid[i])
        assert rc == ko.OK and q["offset"] == bases[i] * sizes(g).S and q["staged"] == len(row)
        assert q["wm"] == lens[i] // g.B and q["swapped"] == 1 and q["cap"] == len(row)
        got = sv[bases[i]: bases[i] + len(row)]
        assert np.array_equal(got, hp.block_image(row, pool0))
    # pool is only read
    assert np.array_equal(hp.pool, pool0)
    # element-level form of the same statement, element (r, j, l, c, t, h, d)
    rng = np.random.default_rng(1)
    ls, ks, bs = hp.strides
    for _ in range(200):
        i = int(rng.integers(len(rid)))
        row = ids[off[i]:off[i + 1]]
        j, l, c = int(rng.integers(len(row))), int(rng.integers(g.L)), int(rng.integers(2))
        t, h, d = int(rng.integers(g.B)), int(rng.integers(g.H)), int(rng.integers(g.D))
        inner = ((t * g.H + h) * g.D + d) * g.e
        st = (bases[i] + j) * sizes(g).S + (l * 2 + c) * sizes(g).chunk + inner
        src = l * ls + c * ks + int(row[j]) * bs + inner
        assert np.array_equal(hp.staging[st:st + g.e], pool0[src:src + g.e])
        if g.scales:
            sls, sks, sbs = hp.scale_strides
            st = (bases[i] + j) * sizes(g).S + sizes(g).block_bytes + (l * 2 + c) * g.H * 4 + h * 4
            src = l * sls + c * sks + int(row[j]) * sbs + h * 4
            assert np.array_equal(hp.staging[st:st + 4], hp.scale[src:src + 4])


test_closed_form = pin_closed_form


# ---------------------------------------------------------------- pins 2 + 3
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("gname", list(GEOMS))
def pin_round_trip(gname, layout, lib=None):
    g = GEOMS[gname]
    hp = HostPool(g, 0xBEEF, layout, slots=20)
    pool0 = hp.pool.copy()
    scale0 = None if hp.scale is None else hp.scale.copy()
    ora = hp.oracle(lib)
    rid, lens, off, ids, free = make_requests(11, g, 3, 1, 5 * g.B)
    total = off[-1]
    assert ora.swap_out(rid, off, ids, lens) == ko.OK
    # arena: everything outside the extents is still canary
    used = total * sizes(g).S
    assert (hp.staging[used:] == CANARY).all()
    # swap in to the SAME blocks: whole pool unchanged
    hp.pool[:] ^= 0  # no-op, keeps the array writable check honest
    assert ora.swap_in(rid, off, ids, ko.KEEP_STAGING) == ko.OK
    assert np.array_equal(hp.pool, pool0)
    if scale0 is not None:
        assert np.array_equal(hp.scale, scale0)
    # clobber the old blocks (the allocator reuses them), then swap in elsewhere
    new = free[:total].copy()
    trash = hp.data_index(ids)
    hp.pool[trash.reshape(-1)] = 0x11
    pool1 = hp.pool.copy()
    assert ora.swap_in(rid, off, new) == ko.OK
    assert np.array_equal(hp.block_image(new), hp.block_image(ids, pool0, scale0))
    # complement: every byte that is not in a destination chunk is as before
    mask = np.ones(len(hp.pool), bool)
    mask[hp.data_index(new).reshape(-1)] = False
    assert np.array_equal(hp.pool[mask], pool1[mask])
    if scale0 is not None:
        smask = np.ones(len(hp.scale), bool)
        smask[hp.scale_index(new).reshape(-1)] = False
        assert np.array_equal(hp.scale[smask], scale0[smask])
    # released
    for r in rid:
        assert ora.query(r)[0] == ko.ENOENT


test_round_trip = pin_round_trip


# ---------------------------------------------------------------- pin 4
@pytest.mark.parametrize("gname", list(GEOMS))
@pytest.mark.parametrize("seed", [1, 2, 3])
def pin_delta_equals_full(gname, seed, lib=None):
    g = GEOMS[gname]
    rng = np.random.default_rng(seed)
    n = 3
    final = rng.integers(2 * g.B, 7 * g.B, size=n).astype(np.int32)
    nb = W.blocks_for(final, g.B)
    off, ids, _ = W.block_tables(seed, g.N, nb)
    rid = np.array([5, 9, 7], dtype=np.uint64)

    full = HostPool(g, 0xD17A, slots=30)
    of = full.oracle(lib)
    assert of.swap_out(rid, off, ids, final) == ko.OK

    inc = HostPool(g, 0xD17A, slots=30)
    oi = inc.oracle(lib)
    for i in range(n):  # same placement as the full swap-out: reserve in call order
        assert oi.reserve(rid[i], int(nb[i])) == ko.OK
    cur = np.minimum(final, rng.integers(0, g.B, size=n)).astype(np.int32)
    moved_total = np.zeros(n, np.int64)
    while (cur < final).any():
        cur = np.minimum(final, cur + rng.integers(0, 2 * g.B, size=n)).astype(np.int32)
        budget = int(rng.integers(0, 4))  # 0 = unlimited
        # tables grow with the request: pass only the blocks allocated so far
        rows = W.blocks_for(cur, g.B)
        o2 = np.zeros(n + 1, np.int32)
        o2[1:] = np.cumsum(rows)
        i2 = np.concatenate([ids[off[i]:off[i] + rows[i]] for i in range(n)])
        before = [oi.query(r)[1]["wm"] for r in rid]
        rc, moved = oi.swap_out_delta(rid, o2, i2, cur, budget=budget)
        assert rc == ko.OK
        left = budget
        for i in range(n):  # the budget rule, restated: serve in order, never split a block
            want = cur[i] // g.B - before[i]
            exp = want if budget == 0 else min(want, left)
            if budget:
                left -= exp
            assert moved[i] == exp
            assert oi.query(rid[i])[1]["wm"] == before[i] + exp
        moved_total += moved
        # Section 5.3: blocks already written through may be reclaimed at once.  Overwrite them
        # on the device side; no later delta may read them again.
        for i in range(n):
            done = ids[off[i]:off[i] + oi.query(rid[i])[1]["wm"]]
            if len(done):
                inc.pool[inc.data_index(done).reshape(-1)] = 0x5A
                if inc.scale is not None:
                    inc.scale[inc.scale_index(done).reshape(-1)] = 0x5A
    # drain what the budgets left behind, then flush the tails
    rc, moved = oi.swap_out_delta(rid, off, ids, final)
    assert rc == ko.OK
    moved_total += moved
    assert np.array_equal(moved_total, final // g.B)  # each full block written exactly once
    rc, moved = oi.swap_out_delta(rid, off, ids, final, flags=ko.DELTA_INCLUDE_TAIL)
    assert rc == ko.OK
    assert np.array_equal(moved, (final % g.B != 0).astype(np.int32))
    assert np.array_equal(inc.staging, full.staging)
    for r in rid:
        qa, qb = of.query(r)[1], oi.query(r)[1]
        assert (qa["offset"], qa["staged"], qa["wm"]) == (qb["offset"], qb["staged"], qb["wm"])
    # a second tail flush moves the tail again (the watermark counts full blocks only)
    rc, moved2 = oi.swap_out_delta(rid, off, ids, final, flags=ko.DELTA_INCLUDE_TAIL)
    assert rc == ko.OK and np.array_equal(moved2, moved)
    # and a plain delta has nothing left to do
    rc, moved3 = oi.swap_out_delta(rid, off, ids, final)
    assert rc == ko.OK and not moved3.any()
    for i in range(n):  # ... and does not forget the flushed tail
        assert oi.query(rid[i])[1]["staged"] == nb[i]


test_delta_equals_full = pin_delta_equals_full


# ---------------------------------------------------------------- pin 5
class DictModel:
    """Element-by-element model: pool[(l, c, phys, t)] and staged[(req, j, l, c, t)]."""

    def __init__(self, L, B, N, values):
        self.L, self.B, self.N = L, B, N
        self.pool = dict(values)
        self.staged = {}
        self.nblk = {}

    def swap_out(self, req, table):
        for j, p in enumerate(table):
            for l in range(self.L):
                for c in range(2):
                    for t in range(self.B):
                        self.staged[(req, j, l, c, t)] = self.pool[(l, c, p, t)]
        self.nblk[req] = len(table)

    def swap_in(self, req, table):
        assert len(table) == self.nblk[req]
        for j, p in enumerate(table):
            for l in range(self.L):
                for c in range(2):
                    for t in range(self.B):
                        self.pool[(l, c, p, t)] = self.staged[(req, j, l, c, t)]


def _pool_to_dict(hp):
    g = hp.geom
    ls, ks, bs = hp.strides
    d = {}
    for l in range(g.L):
        for c in range(2):
            for p in range(g.N):
                for t in range(g.B):
                    tok = g.H * g.D * g.e
                    o = l * ls + c * ks + p * bs + t * tok
                    d[(l, c, p, t)] = bytes(hp.pool[o:o + tok])
    return d


@pytest.mark.parametrize("L,B", [(1, 1), (2, 1), (1, 2), (2, 2)])
def pin_brute_force(L, B, lib=None, D=1):
    N = 5
    g = W.Geometry(L, 1, D, B, "f16", N)  # H = D = 1: one element per token
    cases = 0
    # every way to give two requests disjoint ordered tables of sizes (2,1) and (1,2) out of
    # 5 blocks, every subset of them swapped out, every placement of the swap-in destinations
    for sizes in [(2, 1), (1, 2), (3, 0)]:
        for perm in itertools.permutations(range(N), sum(sizes)):
            tables = [list(perm[:sizes[0]]), list(perm[sizes[0]:])]
            for subset in [(0,), (1,), (0, 1), (1, 0)]:
                hp = HostPool(g, 0xB207E + cases % 7, slots=4)
                model = DictModel(L, B, N, _pool_to_dict(hp))
                ora = hp.oracle(lib)
                rows = [tables[i] for i in subset]
                off = np.zeros(len(rows) + 1, np.int32)
                off[1:] = np.cumsum([len(r) for r in rows])
                flat = [b for r in rows for b in r]
                # tail blocks are half full when B == 2: lengths end mid-block
                lens = [max(0, len(r) * B - (B - 1)) for r in rows]
                rid = np.array([10 + i for i in subset], np.uint64)
                assert ora.swap_out(rid, off, flat, lens) == ko.OK
                for i, r in zip(subset, rows):
                    model.swap_out(10 + i, r)
                # destinations: a rotation of all blocks, so they overlap the sources
                k = cases % N
                dest_pool = [(b + k) % N for b in range(N)]
                dest = dest_pool[:len(flat)]
                drows, at = [], 0
                for r in rows:
                    drows.append(dest[at:at + len(r)])
                    at += len(r)
                assert ora.swap_in(rid, off, dest) == ko.OK
                for i, r in zip(subset, drows):
                    model.swap_in(10 + i, r)
                assert _pool_to_dict(hp) == model.pool
                cases += 1
    assert cases > 500


test_brute_force = pin_brute_force


def test_brute_force_all_destinations():
    """All destination permutations for one request of 3 blocks out of 4 (L=2, B=2)."""
    g = W.Geometry(2, 1, 1, 2, "bf16", 4)
    for src in itertools.permutations(range(4), 3):
        for dst in itertools.permutations(range(4), 3):
            hp = HostPool(g, 0x1234, slots=3)
            model = DictModel(2, 2, 4, _pool_to_dict(hp))
            ora = hp.oracle()
            assert ora.swap_out([1], [0, 3], list(src), [5]) == ko.OK
            model.swap_out(1, list(src))
            assert ora.swap_in([1], [0, 3], list(dst)) == ko.OK
            model.swap_in(1, list(dst))
            assert _pool_to_dict(hp) == model.pool


# ---------------------------------------------------------------- pin 6
@pytest.mark.parametrize("gname", list(GEOMS))
def pin_memcpy_case(gname, lib=None):
    g = GEOMS[gname]
    if g.scales:
        g = W.Geometry(g.L, g.H, g.D, g.B, g.dtype, g.N)  # data only: then a slot is exactly a block
    hp = HostPool(g, 0x3E3C, "block")
    ora = hp.oracle(lib)
    nb = 9
    assert ora.swap_out([77], [0, nb], np.arange(nb), [nb * g.B]) == ko.OK
    n = nb * sizes(g).block_bytes
    assert hp.staging[:n].tobytes() == hp.pool[:n].tobytes()  # one memcpy
    assert (hp.staging[n:] == CANARY).all()
    # and the way back: move the image somewhere else with one slice assignment
    expect = hp.pool.copy()
    expect[20 * sizes(g).block_bytes: 20 * sizes(g).block_bytes + n] = hp.pool[:n]
    assert ora.swap_in([77], [0, nb], np.arange(20, 20 + nb)) == ko.OK
    assert np.array_equal(hp.pool, expect)


test_memcpy_case = pin_memcpy_case


# ---------------------------------------------------------------- pin 7
def _snapshot(hp, ora, rids):
    return (hp.pool.copy(), hp.staging.copy(), [ora.query(r) for r in rids])


def _same(hp, ora, rids, snap):
    return (np.array_equal(hp.pool, snap[0]) and np.array_equal(hp.staging, snap[1])
            and [ora.query(r) for r in rids] == snap[2])


def pin_errors(lib=None):
    g = GEOMS["tiny"]
    B = g.B
    hp = HostPool(g, 0xE44, slots=10)
    ora = hp.oracle(lib)
    known = [1, 2, 3, 4, 5, 6]
    assert ora.swap_out([1], [0, 2], [3, 4], [2 * B]) == ko.OK
    assert ora.reserve(2, 3) == ko.OK
    snap = _snapshot(hp, ora, known)

    def unchanged():
        return _same(hp, ora, known, snap)

    # bad block id (too large, negative) — also when it sits in a later request of the call
    assert ora.swap_out([3], [0, 1], [g.N], [B]) == ko.ERANGE and unchanged()
    assert ora.swap_out([3], [0, 1], [-1], [B]) == ko.ERANGE and unchanged()
    assert ora.swap_out([3, 4], [0, 1, 2], [5, g.N], [B, B]) == ko.ERANGE and unchanged()
    # row length must be ceil(len / B)
    assert ora.swap_out([3], [0, 2], [5, 6], [B]) == ko.EINVAL and unchanged()
    assert ora.swap_out([3], [0, 1], [5], [B + 1]) == ko.EINVAL and unchanged()
    assert ora.swap_out([3], [0, 1], [5], [-1]) == ko.EINVAL and unchanged()
    # the same request twice in a call
    assert ora.swap_out([3, 3], [0, 1, 2], [5, 6], [B, B]) == ko.EINVAL and unchanged()
    # decreasing CSR
    assert ora.swap_out([3, 4], [0, 2, 1], [5, 6], [B, B]) == ko.EINVAL and unchanged()
    # double swap-out, delta after swap-out
    assert ora.swap_out([1], [0, 2], [3, 4], [2 * B]) == ko.EEXIST and unchanged()
    assert ora.swap_out_delta([1], [0, 2], [3, 4], [2 * B])[0] == ko.EEXIST and unchanged()
    # the second request of a call fails: the first must not have happened
    assert ora.swap_out([3, 1], [0, 1, 3], [5, 3, 4], [B, 2 * B]) == ko.EEXIST and unchanged()
    # arena full: 10 slots, 2 + 3 taken
    assert ora.swap_out([3], [0, 6], [1, 2, 3, 4, 5, 6], [6 * B]) == ko.ENOSPC and unchanged()
    assert ora.swap_out([3, 4], [0, 3, 6], [1, 2, 3, 4, 5, 6], [3 * B, 3 * B]) == ko.ENOSPC and unchanged()
    assert ora.reserve(3, 6) == ko.ENOSPC and unchanged()
    # cannot grow in place: request 2 (slots 2..4) grows to 4 — free; then 3 blocks it
    assert ora.reserve(2, 3) == ko.EEXIST and unchanged()
    # swap-in: unknown request, wrong row length, duplicate destination, bad id
    assert ora.swap_in([9], [0, 1], [7]) == ko.ENOENT and unchanged()
    assert ora.swap_in([1], [0, 1], [7]) == ko.EINVAL and unchanged()
    assert ora.swap_in([1], [0, 2], [7, 7]) == ko.EDUP and unchanged()
    assert ora.swap_in([1], [0, 2], [7, g.N]) == ko.ERANGE and unchanged()
    assert ora.swap_in([1, 9], [0, 2, 3], [7, 8, 9]) == ko.ENOENT and unchanged()
    # release / query of an unknown id
    assert ora.release(9) == ko.ENOENT and unchanged()
    assert ora.query(9)[0] == ko.ENOENT
    # delta: shrinking below the watermark
    assert ora.swap_out_delta([2], [0, 3], [10, 11, 12], [2 * B + 1])[0] == ko.OK
    assert ora.query(2)[1]["wm"] == 2
    snap = _snapshot(hp, ora, known)
    assert ora.swap_out_delta([2], [0, 3], [10, 11, 12], [2 * B - 1])[0] == ko.ESTATE and unchanged()
    assert ora.swap_out_delta([2], [0, 1], [10], [2 * B])[0] == ko.EINVAL and unchanged()
    assert ora.swap_out_delta([2], [0, 3], [10, 11, 12], [3 * B], budget=-1)[0] == ko.EINVAL and unchanged()
    # growth in place: request 2 owns slots 2..4; slot 5 is free, so 4 blocks fit ...
    assert ora.swap_out_delta([2], [0, 4], [10, 11, 12, 13], [4 * B])[0] == ko.OK
    assert ora.query(2)[1] == dict(offset=2 * sizes(g).S, cap=4, staged=4, wm=4, swapped=0)
    # ... but once request 3 sits right behind it, it cannot grow further
    assert ora.reserve(3, 1) == ko.OK and ora.query(3)[1]["offset"] == 6 * sizes(g).S
    snap = _snapshot(hp, ora, known)
    assert ora.swap_out_delta([2], [0, 5], [10, 11, 12, 13, 14], [5 * B])[0] == ko.ENOSPC and unchanged()
    # move_blocks
    assert ora.move_blocks([1, 2], [3, 3]) == ko.EDUP and unchanged()
    assert ora.move_blocks([1, 2], [2, 5]) == ko.EDUP and unchanged()
    assert ora.move_blocks([1, g.N], [2, 5]) == ko.ERANGE and unchanged()
    # empty calls are fine and do nothing
    assert ora.swap_out([], [0], [], []) == ko.OK and unchanged()
    assert ora.swap_in([], [0], []) == ko.OK and unchanged()
    assert ora.move_blocks([], []) == ko.OK and unchanged()
    # a request of zero tokens: known afterwards, owns nothing, swaps in nothing
    assert ora.swap_out([6], [0, 0], [], [0]) == ko.OK
    assert ora.query(6)[1] == dict(offset=0, cap=0, staged=0, wm=0, swapped=1)
    assert np.array_equal(hp.staging, snap[1])
    assert ora.swap_in([6], [0, 0], []) == ko.OK and ora.query(6)[0] == ko.ENOENT


test_errors = pin_errors


def pin_move_blocks(lib=None):
    g = GEOMS["fp8s"]
    hp = HostPool(g, 0x404E, "padded")
    pool0, scale0 = hp.pool.copy(), hp.scale.copy()
    ora = hp.oracle(lib)
    src, dst = [3, 9, 3, 0], [5, 1, 7, 28]  # a source may repeat
    assert ora.move_blocks(src, dst) == ko.OK
    assert np.array_equal(hp.block_image(dst), hp.block_image(src, pool0, scale0))
    mask = np.ones(len(hp.pool), bool)
    mask[hp.data_index(dst).reshape(-1)] = False
    assert np.array_equal(hp.pool[mask], pool0[mask])
    smask = np.ones(len(hp.scale), bool)
    smask[hp.scale_index(dst).reshape(-1)] = False
    assert np.array_equal(hp.scale[smask], scale0[smask])
    assert (hp.staging == CANARY).all()


test_move_blocks = pin_move_blocks


# ---------------------------------------------------------------- pin 8
def _run_script(path, lib=None):
    """Replay a hand-worked trace: each line is an operation and the result it must give."""
    g = W.Geometry(1, 1, 8, 1, "f16", 64)
    hp = HostPool(g, 1, slots=12)
    ora = hp.oracle(lib)
    nxt = 0
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        op, *a = line.split()
        if op == "reserve":      # reserve <req> <blocks> -> <base | error>
            rc = ora.reserve(int(a[0]), int(a[1]))
        elif op == "release":    # release <req> -> ok
            rc = ora.release(int(a[0]))
        elif op == "out":        # out <req> <blocks> -> <base | error>   (full swap-out)
            nb = int(a[1])
            ids = [(nxt + k) % g.N for k in range(nb)]
            nxt += nb
            rc = ora.swap_out([int(a[0])], [0, nb], ids, [nb])
        elif op == "in":         # in <req> <blocks> -> ok   (swap-in, extent released)
            nb = int(a[1])
            rc = ora.swap_in([int(a[0])], [0, nb], list(range(nb)))
        else:
            raise ValueError(line)
        want = a[-1]
        if want.startswith("E"):
            assert rc == getattr(ko, want), line
        elif want == "ok":
            assert rc == ko.OK, line
        else:
            assert rc == ko.OK, line
            assert ora.query(int(a[0]))[1]["offset"] == int(want) * sizes(g).S, line


def pin_first_fit(lib=None):
    _run_script(os.path.join(os.path.dirname(__file__), "golden", "first_fit_trace.txt"), lib)


test_first_fit = pin_first_fit


# ------------------------------------------------- repeated preempt/resume cycles
def pin_cycles(lib=None):
    """Section 5.1: a request may be preempted and resumed many times, growing in between."""
    g = GEOMS["odd"]
    hp = HostPool(g, 0xC1C1E, slots=24)
    ora = hp.oracle(lib)
    rng = np.random.default_rng(5)
    free = list(rng.permutation(g.N))
    table, length = [], 0
    truth = []  # expected image of each logical block, tracked through index gathers only
    for cycle in range(6):
        grow = int(rng.integers(1, 3 * g.B))
        length += grow
        while len(table) * g.B < length:
            b = int(free.pop())
            table.append(b)
            truth.append(hp.block_image([b])[0].copy())
        # "decode" overwrites the tail block: new tokens appear in it
        tail = table[-1]
        hp.pool[hp.data_index([tail])[0]] ^= np.uint8(cycle + 1)
        truth[-1] = hp.block_image([tail])[0].copy()
        nb = len(table)
        if cycle % 2 == 0:
            assert ora.swap_out([42], [0, nb], table, [length]) == ko.OK
        else:
            rc, moved = ora.swap_out_delta([42], [0, nb], table, [length], flags=ko.DELTA_INCLUDE_TAIL)
            assert rc == ko.OK
        q = ora.query(42)[1]
        assert q["staged"] == nb and q["wm"] == length // g.B
        # the allocator takes the blocks back and something else overwrites them
        hp.pool[hp.data_index(table).reshape(-1)] = 0xEE
        free = table + free
        table = [int(free.pop()) for _ in range(nb)]
        assert ora.swap_in([42], [0, nb], table, ko.KEEP_STAGING) == ko.OK
        assert np.array_equal(hp.block_image(table), np.stack(truth))
        # stale write-through copy of the tail: the next delta must rewrite it (wm excludes it)
        assert ora.query(42)[1]["swapped"] == 0


test_cycles = pin_cycles

PINS = [
    (pin_closed_form, ("tiny", "layer")), (pin_closed_form, ("fp8s", "padded")), (pin_closed_form, ("odd", "block")),
    (pin_round_trip, ("fp8s", "padded")), (pin_round_trip, ("tiny", "layer")),
    (pin_delta_equals_full, ("odd", 1)), (pin_delta_equals_full, ("fp8s", 2)),
    (pin_brute_force, (2, 2)), (pin_memcpy_case, ("tiny",)), (pin_errors, ()), (pin_move_blocks, ()),
    (pin_first_fit, ()), (pin_cycles, ()),
]


def test_the_pins_sizes_and_the_generators_shapes_agree():
    """The pins work out chunk, block and slot sizes themselves (hostpool.sizes); the input generator carries the same
    definitions for the library's benefit.  A slip in either shows here."""
    for g in (W.Geometry(2, 4, 64, 16, "f16", 10), W.Geometry(32, 8, 128, 16, "bf16", 10),
              W.Geometry(32, 32, 128, 32, "fp8_e4m3", 10, scales=True), W.Geometry(80, 1, 128, 1, "bf16", 10)):
        z = sizes(g)
        assert (z.chunk, z.block_bytes, z.scale_chunk, z.block_scale_bytes, z.S) == \
               (g.chunk, g.block_bytes, g.scale_chunk, g.block_scale_bytes, g.S)
    assert sizes(W.Geometry(32, 8, 128, 16, "bf16", 10)).S == 2 << 20          # "2 MiB per block across layers, K+V"
    assert sizes(W.Geometry(80, 8, 128, 16, "bf16", 10)).S == 5 << 20
    assert sizes(W.Geometry(32, 32, 128, 32, "fp8_e4m3", 10, scales=True)).S == (8 << 20) + (8 << 10)
