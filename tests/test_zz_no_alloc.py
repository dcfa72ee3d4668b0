"""kv_move_blocks_noalloc, the entry point for callers that cannot allocate, against kv_move_blocks.

Two pools with the same content; the same moves go through kv_move_blocks on one and through
kv_move_blocks_noalloc on the other, two calls in a row without a wait in between, the second smaller than the
first (the library's fixed descriptor array then still holds the tail of the first call's list).  The pools must
be equal byte for byte, and equal to what the CPU oracle's move produces.  Runs alone and after the other tests.
"""
import numpy as np
import pytest

from oracle import kv_oracle as ko
from paper_2510_02758_amd import kvswap as kv
from paper_2510_02758_amd import workloads as W

pytestmark = pytest.mark.gpu


def _moves(rng, N, n):
    """n distinct destinations, none of them a source; sources may repeat."""
    perm = rng.permutation(N)
    dst = perm[:n].astype(np.int32)
    src = rng.choice(perm[n:], size=n, replace=True).astype(np.int32)
    return src, dst


@pytest.mark.parametrize("shape", ["bf16_32k_chunks", "fp8_scales", "f16_small_chunks"])
def test_noalloc_move_equals_move_blocks(gpu, shape):
    import torch
    if shape == "bf16_32k_chunks":
        g = W.Geometry(4, 8, 128, 16, "bf16", 1500)
    elif shape == "fp8_scales":
        g = W.Geometry(3, 4, 64, 16, "fp8_e4m3", 900, scales=True)
    else:
        g = W.Geometry(2, 2, 8, 2, "f16", 2000)              # 64-byte chunks: several per job
    seed = 0x5EED0A00
    host_pool = W.fill_buffer_np(seed, g.pool_bytes, g.dtype)
    host_scale = W.fill_buffer_np(seed ^ 0x5CA1E, g.scale_bytes, "raw") if g.scales else None
    rng = np.random.default_rng(11)
    first = _moves(rng, g.N, 700 if g.N >= 1500 else 400)
    second = _moves(rng, g.N, 37)                            # smaller: the array still holds the tail of the first list

    # the oracle, one call after the other
    ora_pool = host_pool.copy()
    ora_scale = host_scale.copy() if g.scales else None
    ora = ko.Oracle(g.L, g.H, g.D, g.B, g.e, g.N, ora_pool, g.strides, np.zeros(g.S, np.uint8), scale=ora_scale,
                    scale_strides=g.scale_strides if g.scales else None)
    for src, dst in (first, second):
        assert ora.move_blocks(src, dst) == ko.OK

    pools, scales, handles = [], [], []
    for _ in range(2):
        pools.append(torch.from_numpy(host_pool.copy()).to(gpu))
        scales.append(torch.from_numpy(host_scale.copy()).to(gpu) if g.scales else None)
        arena = torch.zeros(2 * g.S, dtype=torch.uint8).pin_memory()
        handles.append(kv.KVPool(g, pools[-1], arena, scale=scales[-1]))
    ref, na = handles
    for src, dst in (first, second):                         # two calls in a row, no wait in between
        assert ref.move_blocks(src, dst) == kv.KV_OK
        assert na.move_blocks_noalloc(src, dst) == kv.KV_OK
    st = na.stats()
    assert st["op"] == 4 and st["blocks"] == len(second[0]) and st["launches"] == 1
    assert ref.sync() == kv.KV_OK and na.sync() == kv.KV_OK
    assert torch.equal(pools[0], pools[1]), "kv_move_blocks_noalloc and kv_move_blocks disagree"
    assert np.array_equal(pools[1].cpu().numpy(), ora_pool), "pool differs from the oracle"
    if g.scales:
        assert torch.equal(scales[0], scales[1])
        assert np.array_equal(scales[1].cpu().numpy(), ora_scale), "scales differ from the oracle"

    # refusals: nothing is enqueued, nothing changes
    before = pools[1].clone()
    too_many = np.zeros(kv.KV_NOALLOC_MAX_BLOCKS + 1, np.int32)
    assert na.move_blocks_noalloc(too_many, too_many) == kv.KV_E2BIG
    assert "fixed descriptor array" in kv.kv_strerror(kv.KV_E2BIG)
    assert na.move_blocks_noalloc([1, 2], [3, 3]) == kv.KV_EDUP          # one destination twice
    assert na.move_blocks_noalloc([1, 2], [2, 5]) == kv.KV_EDUP          # a destination that is a source
    assert na.move_blocks_noalloc([1], [g.N]) == kv.KV_ERANGE
    assert na.move_blocks_noalloc([1, 1], [4, 5]) == kv.KV_OK            # a source twice is legal
    assert ref.move_blocks([1, 1], [4, 5]) == kv.KV_OK
    assert na.sync() == kv.KV_OK and ref.sync() == kv.KV_OK
    assert torch.equal(pools[0], pools[1])
    changed = (before != pools[1]).any().item()
    assert changed                                                        # blocks 4 and 5 now hold block 1
    for h in handles:
        h.close()


def test_noalloc_move_is_ordered_against_swap_in(gpu):
    """A swap-in issued right after an allocation-free move, into the blocks the move reads, must see them moved
    first; a move issued right after a swap-in, out of the blocks the swap-in writes, must see them written."""
    import torch
    g = W.Geometry(4, 8, 128, 16, "bf16", 1200)
    seed = 0x5EED0A01
    host_pool = W.fill_buffer_np(seed, g.pool_bytes, g.dtype)
    rng = np.random.default_rng(5)
    perm = rng.permutation(g.N).astype(np.int32)
    a, b, c = perm[:300], perm[300:600], perm[600:900]
    lens = np.array([300 * g.B], np.int32)
    off = np.array([0, 300], np.int32)
    rid = np.array([7], np.uint64)

    ora_pool = host_pool.copy()
    ora_stage = np.zeros(300 * g.S, np.uint8)
    ora = ko.Oracle(g.L, g.H, g.D, g.B, g.e, g.N, ora_pool, g.strides, ora_stage)
    pool = torch.from_numpy(host_pool.copy()).to(gpu)
    arena = torch.zeros(300 * g.S, dtype=torch.uint8).pin_memory()
    kp = kv.KVPool(g, pool, arena)

    assert ora.swap_out(rid, off, a, lens) == ko.OK and kp.swap_out(rid, off, a, lens) == kv.KV_OK
    # move a -> b on the evict stream, then load the request into a: the load must not overtake the move's reads
    assert ora.move_blocks(a, b) == ko.OK and kp.move_blocks_noalloc(a, b) == kv.KV_OK
    assert ora.swap_in(rid, off, a[::-1].copy(), ko.KEEP_STAGING) == ko.OK
    assert kp.swap_in(rid, off, a[::-1].copy(), kv.KV_KEEP_STAGING) == kv.KV_OK
    # and a move out of what that load writes
    assert ora.move_blocks(a, c) == ko.OK and kp.move_blocks_noalloc(a, c) == kv.KV_OK
    assert kp.sync() == kv.KV_OK
    assert np.array_equal(pool.cpu().numpy(), ora_pool)
    assert np.array_equal(arena.numpy(), ora_stage)
    kp.close()
