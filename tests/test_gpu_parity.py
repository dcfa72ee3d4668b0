"""GPU parity: the HIP library against the CPU oracle, byte for byte, through the C ABI.

Integer/byte work: the bar is bit-exact (np.array_equal on raw bytes), no tolerance.
Every case runs on all three transfer paths: zero-copy kernels into the pinned arena,
bounce buffer + hipMemcpyAsync, and the on-device arena.
"""
import numpy as np
import pytest

import test_oracle_pins as T
from adapters import GpuAdapter
from hostpool import CANARY, HostPool
from oracle import kv_oracle as ko
from paper_2510_02758_amd import kvswap as kv
from paper_2510_02758_amd import workloads as W

pytestmark = pytest.mark.gpu

PATHS = {"zerocopy": kv.KV_PATH_ZEROCOPY, "dma": kv.KV_PATH_DMA, "device": kv.KV_STAGING_DEVICE}


def adapter(path, **kw):
    return lambda hp: GpuAdapter(hp, PATHS[path], **kw)


# ---- the oracle's own pins, with the GPU library underneath ---------------------
@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("layout", T.LAYOUTS)
@pytest.mark.parametrize("gname", list(T.GEOMS))
def test_pins_closed_form(gpu, gname, layout, path):
    T.pin_closed_form(gname, layout, lib=adapter(path))


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("gname", list(T.GEOMS))
def test_pins_round_trip(gpu, gname, path):
    T.pin_round_trip(gname, "padded", lib=adapter(path))


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("gname", list(T.GEOMS))
def test_pins_delta(gpu, gname, path):
    T.pin_delta_equals_full(gname, 2, lib=adapter(path))


@pytest.mark.parametrize("path", list(PATHS))
def test_pins_rest(gpu, path):
    T.pin_memcpy_case("tiny", lib=adapter(path))
    T.pin_errors(lib=adapter(path))
    T.pin_move_blocks(lib=adapter(path))
    T.pin_first_fit(lib=adapter(path))
    T.pin_cycles(lib=adapter(path))


# ---- oracle vs GPU, element by element ------------------------------------------
def run_both(g, seed, layout, path, n_req, lo, hi, n_victims, tune=(), bounce_slots=3, slots=None):
    """Same seeded inputs through the oracle (host arrays) and the library (device);
    returns nothing, asserts equality of arena and pool after each phase."""
    lens = W.request_lengths(seed, n_req, ("uniform", lo, hi))
    off, ids, free = W.block_tables(seed, g.N, W.blocks_for(lens, g.B))
    victims = np.sort(W.pick(seed, n_req, n_victims))
    voff, vids = W.csr_take(off, ids, victims)
    rid = (1000 + victims).astype(np.uint64)
    vlen = lens[victims]
    nslots = (len(vids) + 5) if slots is None else slots

    a = HostPool(g, seed, layout, slots=nslots)
    ora = a.oracle()
    b = HostPool(g, seed, layout, slots=nslots)
    gpu = GpuAdapter(b, PATHS[path], bounce_slots=bounce_slots, tune=tune)

    assert ora.swap_out(rid, voff, vids, vlen) == ko.OK
    assert gpu.swap_out(rid, voff, vids, vlen) == kv.KV_OK
    assert np.array_equal(a.staging, b.staging), "arena differs after swap-out"
    assert np.array_equal(a.pool, b.pool)
    st = gpu.kp.stats()
    assert st["blocks"] == len(vids) and st["bytes"] == len(vids) * g.S

    # the allocator reuses the victims' blocks for something else
    for hp in (a, b):
        hp.pool[hp.data_index(vids).reshape(-1)] = 0x3C
    assert len(free) >= len(vids), "test geometry too small for its requests"
    new = free[: len(vids)]
    assert ora.swap_in(rid, voff, new) == ko.OK
    assert gpu.swap_in(rid, voff, new) == kv.KV_OK
    assert np.array_equal(a.pool, b.pool), "pool differs after swap-in"
    if g.scales:
        assert np.array_equal(a.scale, b.scale), "scales differ after swap-in"
    assert np.array_equal(a.staging, b.staging)
    for r in rid:
        assert gpu.query(r)[0] == kv.KV_ENOENT
    gpu.close()


@pytest.mark.parametrize("variant", [0, 1, 2], ids=["seed", "seed+1", "seed+2"])
@pytest.mark.parametrize("path", list(PATHS))
def test_config1_tiny_fp16(gpu, path, variant):
    """BASELINE config 1: fp16, L=2, H=4, D=64, B=16, 1024 blocks; 8 requests of 16-256 tokens;
    3 swapped out, then swapped into different free blocks.  The configuration's own seed and two further ones."""
    wl = W.config(1, variant=variant)
    run_both(wl.geom, wl.seed, "layer", path, wl.n_requests, 16, 256, wl.n_preempt)


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("layout", ["layer", "padded"])
def test_ragged_pieces_and_grid_stride(gpu, path, layout):
    """chunk = 20 KiB + 48 B: one full 16 KiB piece and a ragged one whose last lane group is
    partly idle; a 3-workgroup cap makes every workgroup loop over many jobs; the DMA path is
    cut into slices of 2 blocks."""
    g = W.Geometry(3, 1, 5132, 2, "bf16", 96)  # chunk = 2*1*5132*2 = 20528 bytes
    assert g.chunk == 20528 and g.chunk % 16 == 0 and g.chunk % 16384 != 0
    tune = ((kv.KV_TUNE_MAX_WGS_DEVICE, 3), (kv.KV_TUNE_MAX_WGS_LINK, 3), (kv.KV_TUNE_DMA_SLICE_BLOCKS, 2))
    run_both(g, 0xA11CE, layout, path, 6, 2, 24, 4, tune=tune)


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("unroll", [1, 2, 4, 8])
def test_every_piece_size(gpu, path, unroll):
    g = W.Geometry(2, 2, 1160, 8, "bf16", 80)  # chunk = 37120 B = 2320 x 16: ragged for every piece size
    assert g.chunk == 37120
    tune = ((kv.KV_TUNE_KERNEL_VARIANT, unroll),)
    run_both(g, 0xBEE + unroll, "layer", path, 5, 4, 40, 3, tune=tune)


@pytest.mark.parametrize("unroll", [0, 1, 2, 8])
def test_whole_line_host_stores(gpu, unroll):
    """KV_TUNE_HOST_STORES 1: the gather into the host arena writes whole 128-byte lines per store instruction with
    non-temporal stores instead of 64 consecutive bytes per lane; ragged pieces, every piece size, small chunks."""
    tune = ((kv.KV_TUNE_HOST_STORES, 1),) + (((kv.KV_TUNE_KERNEL_VARIANT, unroll),) if unroll else ())
    run_both(W.Geometry(2, 2, 1160, 8, "bf16", 80), 0x7057 + unroll, "layer", "zerocopy", 5, 4, 40, 3, tune=tune)
    run_both(W.Geometry(3, 1, 5132, 2, "bf16", 96), 0x7058 + unroll, "padded", "zerocopy", 6, 2, 24, 4,
             tune=tune + ((kv.KV_TUNE_MAX_WGS_LINK, 3),))
    run_both(W.Geometry(7, 2, 64, 4, "bf16", 300), 0x7059 + unroll, "layer", "zerocopy", 9, 4, 100, 6, tune=tune)


@pytest.mark.parametrize("variant", [101, 102, 104])
@pytest.mark.parametrize("layout", ["layer", "padded"])
def test_pipelined_resident_workgroups(gpu, variant, layout):
    """The experimental build with resident, software-pipelined workgroups (both ends in HBM, chunks that are a
    multiple of the piece): a workgroup cap of 7 makes every workgroup walk many pieces, 3 requests of a few blocks
    leave some workgroups with a single piece, and a launch with fewer pieces than workgroups leaves some with none."""
    g = W.Geometry(3, 4, 64, 32, "bf16", 700)   # chunk = 32*4*64*2 = 16 KiB: 4, 2 or 1 pieces
    assert g.chunk == 16384
    tune = ((kv.KV_TUNE_KERNEL_VARIANT, variant), (kv.KV_TUNE_SCATTER_ORDER, 1))
    run_both(g, 0x91BE + variant, layout, "device", 9, 32, 32 * 40, 6, tune=tune + ((kv.KV_TUNE_MAX_WGS_DEVICE, 7),))
    run_both(g, 0x91BF + variant, layout, "device", 3, 32, 32 * 3, 2, tune=tune)
    run_both(g, 0x91C0 + variant, layout, "device", 1, 32, 32, 1, tune=tune + ((kv.KV_TUNE_MAX_WGS_DEVICE, 4096),))


@pytest.mark.parametrize("layout", ["layer", "padded"])
def test_scatter_plane_by_plane(gpu, layout):
    """The other job order of the on-device scatter (planes outside, descriptors sorted by destination block inside),
    forced for every size: ragged 9 KiB chunks, few and many blocks, a workgroup cap that makes workgroups loop."""
    g = W.Geometry(2, 4, 72, 16, "f16", 400)  # chunk = 16*4*72*2 = 9216 B: two full pieces and a ragged one
    assert g.chunk == 9216
    run_both(g, 0x9A7E, layout, "device", 12, 16, 400, 9, tune=((kv.KV_TUNE_SCATTER_ORDER, 2),))
    run_both(g, 0x9A7F, layout, "device", 3, 16, 48, 2, tune=((kv.KV_TUNE_SCATTER_ORDER, 2), (kv.KV_TUNE_MAX_WGS_DEVICE, 5)))


def test_scatter_plane_by_plane_with_scales(gpu):
    """A pool with scales has the same two job orders for its data; its scale jobs follow in a launch of their own."""
    g = W.Geometry(4, 32, 128, 32, "fp8_e4m3", 128, scales=True)   # 128 KiB chunks, 128-byte scale pieces
    run_both(g, 0x5CA7, "layer", "device", 6, 32, 256, 4, tune=((kv.KV_TUNE_SCATTER_ORDER, 2),))
    g2 = W.Geometry(2, 8, 64, 16, "fp8_e4m3", 300, scales=True)    # 8 KiB chunks
    run_both(g2, 0x5CA8, "padded", "device", 9, 16, 300, 5, tune=((kv.KV_TUNE_SCATTER_ORDER, 2), (kv.KV_TUNE_MAX_WGS_DEVICE, 5)))


def test_scatter_order_is_chosen_by_timing(gpu):
    """1024 blocks and more, both ends in HBM: the first such swap-in goes block by block, the second plane by plane,
    the later ones use whichever has the better rate so far (kv_stats.scatter_order says which; with launches as
    short as these the rates are close and the choice may change from one call to the next); every one of them is
    bit-exact."""
    import torch
    g = W.Geometry(1, 4, 64, 16, "bf16", 4096)  # 8 KiB chunks, 16 KiB blocks
    seed, n_req = 0x0D3, 24
    lens = W.request_lengths(seed, n_req, ("uniform", 48 * g.B, 80 * g.B))
    off, ids, free = W.block_tables(seed, g.N, W.blocks_for(lens, g.B))
    assert 1024 <= len(ids) <= len(free)
    rid = np.arange(1, n_req + 1, dtype=np.uint64)
    a = HostPool(g, seed, "layer", slots=len(ids) + 4)
    ora = a.oracle()
    b = HostPool(g, seed, "layer", slots=len(ids) + 4)
    lib = GpuAdapter(b, kv.KV_STAGING_DEVICE)
    orders = []
    cur = ids
    for it in range(6):
        nxt = free[: len(ids)] if it % 2 == 0 else ids
        assert ora.swap_out(rid, off, cur, lens) == ko.OK and lib.swap_out(rid, off, cur, lens) == kv.KV_OK
        assert lib.kp.stats()["scatter_order"] == -1
        assert ora.swap_in(rid, off, nxt) == ko.OK and lib.swap_in(rid, off, nxt) == kv.KV_OK
        assert np.array_equal(a.pool, b.pool) and np.array_equal(a.staging, b.staging), "iteration %d" % it
        orders.append(lib.kp.stats()["scatter_order"])
        cur = nxt
    assert orders[:2] == [0, 1] and all(o in (0, 1) for o in orders[2:]), orders
    # a small swap-in is not of this kind
    assert lib.swap_out(rid[:1], off[:2], cur[: off[1]], lens[:1]) == kv.KV_OK
    assert lib.swap_in(rid[:1], off[:2], cur[: off[1]]) == kv.KV_OK and lib.kp.stats()["scatter_order"] == -1
    lib.close()


@pytest.mark.parametrize("path", list(PATHS))
def test_fp8_with_scales(gpu, path):
    """fp8 values and fp32 scales travel together (BASELINE config 5 shape, scaled down):
    H=32, D=128, B=32 -> chunk 128 KiB, scale chunk 128 B."""
    g = W.Geometry(4, 32, 128, 32, "fp8_e4m3", 128, scales=True)
    run_both(g, 0x5EED0005, "layer", path, 6, 32, 256, 4)
    g2 = W.Geometry(3, 6, 16, 4, "fp8_e4m3", 160, scales=True)  # 24-byte scale pieces, padded strides
    run_both(g2, 0xF8, "padded", path, 7, 1, 40, 5)


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("knob", [1, 2])
def test_scale_side_band_variants(gpu, path, knob):
    """The scale side band word by word (1) and staged through LDS (2) give the same bytes."""
    tune = ((kv.KV_TUNE_SCALE_LDS, knob),)
    run_both(W.Geometry(4, 32, 128, 32, "fp8_e4m3", 128, scales=True), 0x5CA + knob, "layer", path, 6, 32, 256, 4,
             tune=tune)
    run_both(W.Geometry(3, 6, 16, 4, "fp8_e4m3", 160, scales=True), 0x5CB + knob, "padded", path, 7, 1, 40, 5,
             tune=tune)
    run_both(W.Geometry(6, 2, 32, 1, "fp8_e4m3", 400, scales=True), 0x5CC + knob, "block", path, 9, 1, 40, 6,
             tune=tune)


@pytest.mark.parametrize("path", list(PATHS))
def test_small_chunks(gpu, path):
    """Token-level pool (B=1) and a tensor-parallel shard with one KV head: chunks of 256 B / 4 KiB."""
    run_both(W.Geometry(4, 1, 128, 1, "bf16", 512), 0x701, "layer", path, 12, 1, 40, 7)
    run_both(W.Geometry(5, 1, 128, 16, "bf16", 256), 0x702, "layer", path, 10, 16, 300, 6)


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("unroll", [0, 1, 2, 8])
def test_small_chunk_groups(gpu, path, unroll):
    """Chunks below 4 KiB are moved several per workgroup: 48 B (3 lanes per chunk, 85 chunks per
    group, lanes left over), 1 KiB, 2 KiB, and 3088 B (one chunk per group, 63 idle lanes); 2L is
    not a multiple of the group size, so the last group of every block is ragged."""
    tune = ((kv.KV_TUNE_KERNEL_VARIANT, unroll),) if unroll else ()
    run_both(W.Geometry(45, 1, 24, 1, "bf16", 300), 0x5C1 + unroll, "layer", path, 9, 1, 30, 6, tune=tune)
    run_both(W.Geometry(7, 2, 64, 4, "bf16", 300), 0x5C2 + unroll, "padded", path, 9, 4, 100, 6, tune=tune)
    run_both(W.Geometry(5, 1, 128, 8, "bf16", 300), 0x5C3 + unroll, "block", path, 9, 8, 200, 6, tune=tune)
    run_both(W.Geometry(3, 1, 193, 8, "bf16", 300), 0x5C4 + unroll, "layer", path, 9, 8, 200, 6, tune=tune)
    run_both(W.Geometry(3, 4, 16, 4, "fp8_e4m3", 200, scales=True), 0x5C5 + unroll, "padded", path, 7, 4, 90, 5,
             tune=tune)


@pytest.mark.parametrize("path", list(PATHS))
def test_limits_whole_pool_and_full_arena(gpu, path):
    """Edges: one request owning EVERY block of the pool (ids 0 and N-1 included), an arena with
    exactly as many slots as blocks, a one-token request, a zero-token request, an empty call; the
    whole pool comes back permuted through a swap-in issued with no sync after the swap-out."""
    g = W.Geometry(3, 2, 64, 8, "bf16", 257)                  # chunk 2 KiB (small-chunk groups), odd block count
    seed = 0x11A17
    a = HostPool(g, seed, slots=g.N)
    b = HostPool(g, seed, slots=g.N)
    ora = a.oracle()
    gpuad = GpuAdapter(b, PATHS[path], bounce_slots=7)
    kp = gpuad.kp
    rng = np.random.default_rng(9)
    table = rng.permutation(g.N).astype(np.int32)
    dest = rng.permutation(g.N).astype(np.int32)
    lens = [(g.N - 1) * g.B - 5, 1, 0]                        # 256 blocks (ragged tail), 1 block, 0 blocks
    off = [0, g.N - 1, g.N, g.N]
    rid = [1, 2, 3]
    for o, OK in ((ora, ko.OK), (None, kv.KV_OK)):
        if o is None:
            gpuad._push()
            assert kp.swap_out([], [0], [], []) == OK         # empty call
            assert kp.swap_out(rid, off, table, lens) == OK
            assert kp.swap_in(rid, off, dest) == OK           # no sync: ordered inside the library
            gpuad._pull()
        else:
            assert o.swap_out([], [0], [], []) == OK
            assert o.swap_out(rid, off, table, lens) == OK
            assert o.swap_in(rid, off, dest) == OK
    assert np.array_equal(a.staging, b.staging)
    assert np.array_equal(a.pool, b.pool)
    # the arena was exactly full: one more block does not fit, and says so before doing anything
    assert gpuad.swap_out([1], [0, g.N], table, [g.N * g.B]) == kv.KV_OK
    assert ora.swap_out([1], [0, g.N], table, [g.N * g.B]) == ko.OK
    assert gpuad.swap_out([9], [0, 1], [0], [1]) == kv.KV_ENOSPC and ora.swap_out([9], [0, 1], [0], [1]) == ko.ENOSPC
    assert np.array_equal(a.staging, b.staging)
    gpuad.close()


def test_back_to_back_without_sync(gpu):
    """Stream ordering: swap-out then swap-in of the same requests with no kv_sync in between;
    then a second swap-out that reuses the slots the first swap-in is still reading."""
    g = W.Geometry(4, 8, 128, 16, "bf16", 600)
    import torch
    seed = 0x0DE2
    lens = W.request_lengths(seed, 10, ("uniform", 100, 700))
    off, ids, free = W.block_tables(seed, g.N, W.blocks_for(lens, g.B))
    rid = np.arange(1, 11, dtype=np.uint64)
    nslots = int(off[-1]) + 2
    a = HostPool(g, seed, slots=nslots)
    ora = a.oracle()
    pool = torch.from_numpy(a.pool.copy()).cuda()
    staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
    kp = kv.KVPool(g, pool, staging, flags=kv.KV_PATH_ZEROCOPY)
    new = free[: len(ids)]
    # library: three calls in a row, no sync; the third reuses the arena slots of the first, so
    # the evict stream has to wait for the swap-in that still reads them
    assert kp.swap_out(rid, off, ids, lens) == kv.KV_OK
    assert kp.swap_in(rid, off, new) == kv.KV_OK
    rid2 = rid + 100
    assert kp.swap_out(rid2[::-1], *W.csr_take(off, new, np.arange(10)[::-1]), lens[::-1]) == kv.KV_OK
    assert kp.sync() == kv.KV_OK
    # oracle: the same three calls
    assert ora.swap_out(rid, off, ids, lens) == ko.OK
    assert ora.swap_in(rid, off, new) == ko.OK
    o2, i2 = W.csr_take(off, new, np.arange(10)[::-1])
    assert ora.swap_out(rid2[::-1], o2, i2, lens[::-1]) == ko.OK
    assert np.array_equal(pool.cpu().numpy(), a.pool)
    assert np.array_equal(staging.numpy(), a.staging)
    kp.close()


@pytest.mark.parametrize("path", ["zerocopy", "dma"])
@pytest.mark.parametrize("events,seg_max,order", [(0, 0, "reverse"), (kv.KV_REQ_EVENTS, 0, "reverse"),
                                                  (kv.KV_REQ_EVENTS, 16 << 20, "reverse"), (kv.KV_REQ_EVENTS, 16 << 20, "same"),
                                                  (kv.KV_REQ_EVENTS, 2 << 20, "same"), (kv.KV_REQ_EVENTS, 16 << 20, "head_first")])
def test_device_block_hazards_between_streams(gpu, events, seg_max, order, path):
    """The library orders the evict and load streams around DEVICE blocks too: a swap-in may be
    handed blocks that an unfinished swap-out still reads, a swap-out or a move may read blocks an
    unfinished swap-in still writes, all without kv_sync in between.  Expected result: the oracle's,
    which runs the same calls one after the other.  With segments cut inside a request (seg_max) the
    follow-up runs piece by piece behind the call it depends on: in the same block order it trails it
    by one segment, the narrowest window there is; in the opposite order its first piece needs the
    other call's last; "head_first" takes the first 8 blocks in the same order and the rest in the opposite
    one, so the first piece may start at once while the second has to wait for nearly the whole other call:
    a wait taken only once per call would let it run far too early."""
    import torch
    g = W.Geometry(32, 8, 128, 16, "bf16", 1400)             # 2 MiB blocks, 2.7 GiB pool
    seed = 0xB10CC
    a = HostPool(g, seed, slots=1300)
    ora = a.oracle()
    pool = torch.from_numpy(a.pool.copy()).cuda()
    staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
    if path == "dma":             # slices of 24 blocks through each half of the bounce buffer
        bounce = torch.zeros(2 * 24 * g.S, dtype=torch.uint8, device="cuda")
        kp = kv.KVPool(g, pool, staging, bounce=bounce, flags=kv.KV_PATH_DMA | events)
    else:
        kp = kv.KVPool(g, pool, staging, flags=kv.KV_PATH_ZEROCOPY | events)
    if seg_max:
        assert kp.tune(kv.KV_TUNE_SEGMENT_BYTES, seg_max) == kv.KV_OK
        assert kp.tune(kv.KV_TUNE_SEGMENT_MAX_BYTES, seg_max) == kv.KV_OK
    perm = np.random.default_rng(4).permutation(g.N).astype(np.int32)
    X, Y, Z = perm[:300], perm[300:600], perm[600:900]
    offA = np.array([0, 100, 300], np.int32)                  # request A = two requests, 100 + 200 blocks
    lensA = np.array([100 * g.B, 200 * g.B - 3], np.int32)
    lensB = np.array([300 * g.B], np.int32)

    # Each follow-up walks the blocks in the opposite order, so that without ordering the second
    # kernel reaches the far end of the list long before the first one does.
    def walk(v):
        if order == "reverse":
            return v[::-1].copy()
        if order == "head_first":
            return np.concatenate([v[:8], v[8:][::-1]])
        return v
    Xr, Zr = walk(X), walk(Z)

    def script(o, OK):
        # B's KV lives in blocks Y and is swapped out first
        assert o.swap_out([7], [0, 300], Y, lensB) == OK
        # 1. evict A from X, and at once load B into the very same blocks
        assert o.swap_out([1, 2], offA, X, lensA) == OK
        assert o.swap_in([7], [0, 300], Xr, kv.KV_KEEP_STAGING) == OK
        # 2. at once evict a new request that owns the blocks B was just loaded into (fresh slots)
        assert o.swap_out([8], [0, 300], X, lensB) == OK
        # 3. load A somewhere else and at once move it on inside the pool
        assert o.swap_in([1, 2], offA, Z) == OK
        assert o.move_blocks(Zr, Y) == OK

    script(kp, kv.KV_OK)          # the library: six calls back to back, nothing waits on the host
    assert kp.sync() == kv.KV_OK
    script(ora, ko.OK)            # the oracle: the same calls, one after the other
    assert np.array_equal(staging.numpy(), a.staging), "staging differs: a gather read blocks too late or too early"
    assert np.array_equal(pool.cpu().numpy(), a.pool), "pool differs: a scatter or move ran too early"
    kp.close()


@pytest.mark.parametrize("mode", ["zerocopy", "dma", "device_arena"])
@pytest.mark.parametrize("order", ["same", "reverse", "shuffled"])
def test_evict_and_load_in_one_call(gpu, mode, order):
    """kv_evict_and_load: two requests are evicted while a third is loaded into the very blocks they give up, in the
    order they are evicted, in the opposite order, or in any order; phases of 8 blocks.  Then a second call whose
    load needs no block of its eviction, and calls with one side empty.  Expected: what the oracle reaches with
    swap_out followed by swap_in; nothing waits on the host before the end."""
    import torch
    g = W.Geometry(32, 8, 128, 16, "bf16", 1400)             # 2 MiB blocks
    a = HostPool(g, 0xE71C7, slots=1300)
    ora = a.oracle()
    pool = torch.from_numpy(a.pool.copy()).cuda()
    if mode == "device_arena":
        staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8, device="cuda")
        kp = kv.KVPool(g, pool, staging, flags=kv.KV_STAGING_DEVICE)
    elif mode == "dma":
        staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
        bounce = torch.zeros(2 * 24 * g.S, dtype=torch.uint8, device="cuda")
        kp = kv.KVPool(g, pool, staging, bounce=bounce, flags=kv.KV_PATH_DMA)
    else:
        staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
        kp = kv.KVPool(g, pool, staging, flags=kv.KV_PATH_ZEROCOPY)
    assert kp.tune(kv.KV_TUNE_PHASE_BYTES, 8 * g.S) == kv.KV_OK
    rng = np.random.default_rng(12)
    perm = rng.permutation(g.N).astype(np.int32)
    X, Y, Z, V = perm[:300], perm[300:600], perm[600:900], perm[900:1100]
    offA = np.array([0, 100, 300], np.int32)
    lensA = np.array([100 * g.B, 200 * g.B - 5], np.int32)
    lensB = np.array([300 * g.B], np.int32)
    Xw = {"same": X, "reverse": X[::-1].copy(), "shuffled": rng.permutation(X).astype(np.int32)}[order]

    # B lives in Y and is swapped out first; A (two requests) lives in X
    for o, OK in ((kp, kv.KV_OK), (ora, ko.OK)):
        assert o.swap_out([7], [0, 300], Y, lensB) == OK
    # 1. evict A while B is loaded into A's blocks
    assert kp.evict_and_load([1, 2], offA, X, lensA, [7], [0, 300], Xw, kv.KV_KEEP_STAGING) == kv.KV_OK
    assert ora.swap_out([1, 2], offA, X, lensA) == ko.OK and ora.swap_in([7], [0, 300], Xw, ko.KEEP_STAGING) == ko.OK
    # 2. at once: evict a request that owns the blocks B has just been loaded into, while A comes back elsewhere
    assert kp.evict_and_load([8], [0, 300], X, lensB, [1, 2], offA, Z) == kv.KV_OK
    assert ora.swap_out([8], [0, 300], X, lensB) == ko.OK and ora.swap_in([1, 2], offA, Z) == ko.OK
    # 3. one side empty
    assert kp.evict_and_load([9], [0, 200], V, [200 * g.B], [], [0], []) == kv.KV_OK
    assert ora.swap_out([9], [0, 200], V, [200 * g.B]) == ko.OK
    assert kp.evict_and_load([], [0], [], [], [9], [0, 200], V[::-1].copy()) == kv.KV_OK
    assert ora.swap_in([9], [0, 200], V[::-1].copy()) == ko.OK
    # refusals leave everything as it was: a request in both sets, an unknown request to load (the eviction must not happen)
    assert kp.evict_and_load([8], [0, 300], X, lensB, [8], [0, 300], Y) == kv.KV_EINVAL
    assert kp.evict_and_load([1], [0, 100], Z[:100], [100 * g.B], [99], [0, 1], [5]) == kv.KV_ENOENT
    assert kp.query(1)[0] == kv.KV_ENOENT                     # request 1 is resident and unknown to the arena: not evicted
    assert kp.sync() == kv.KV_OK
    host = staging.cpu().numpy() if mode == "device_arena" else staging.numpy()
    assert np.array_equal(host, a.staging), "staging differs from the oracle"
    assert np.array_equal(pool.cpu().numpy(), a.pool), "pool differs from the oracle: a load phase ran before its blocks were read"
    for r in (1, 2, 7, 8, 9):
        (rc_a, qa), (rc_b, qb) = kp.query(r), ora.query(r)
        assert rc_a == rc_b and (rc_a != 0 or qa == qb), r
    kp.close()


def test_segments_cut_inside_a_request(gpu):
    """KV_TUNE_SEGMENT_MAX_BYTES: a long request goes out in pieces of that size (one launch each on the
    zero-copy path); its completion is that of its last piece; the bytes are the oracle's."""
    import torch
    g = W.Geometry(8, 8, 128, 16, "bf16", 400)             # block = 512 KiB
    a = HostPool(g, 0x5E6, slots=260)
    ora = a.oracle()
    pool = torch.from_numpy(a.pool.copy()).cuda()
    staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
    kp = kv.KVPool(g, pool, staging, flags=kv.KV_PATH_ZEROCOPY | kv.KV_REQ_EVENTS)
    assert kp.tune(kv.KV_TUNE_SEGMENT_BYTES, 1 << 20) == kv.KV_OK          # 2 blocks
    assert kp.tune(kv.KV_TUNE_SEGMENT_MAX_BYTES, 4 << 20) == kv.KV_OK      # 8 blocks
    perm = np.random.default_rng(8).permutation(g.N).astype(np.int32)
    off = np.array([0, 1, 101, 104, 204], np.int32)        # 1, 100, 3 and 100 blocks
    lens = np.array([1, 100, 3, 100], np.int32) * g.B
    rid = [11, 12, 13, 14]
    assert kp.swap_out(rid, off, perm[:204], lens) == kv.KV_OK
    assert kp.req_wait(12) == kv.KV_OK and kp.req_poll(11) == 1            # 11 ended in an earlier piece than 12
    # pieces of 8 blocks: [0,8) .. [88,96), then [96,101) ends request 12, [101,104) is request 13,
    # [104,112) .. [192,200), [200,204) ends request 14: 12 + 1 + 1 + 12 + 1
    assert kp.stats()["launches"] == 27
    assert kp.sync() == kv.KV_OK
    ids, done_ms = kp.timeline()
    assert [int(x) for x in ids] == rid and np.all(np.diff(done_ms) >= 0)
    assert ora.swap_out(rid, off, perm[:204], lens) == ko.OK
    assert np.array_equal(staging.numpy(), a.staging)
    assert kp.swap_in(rid, off, perm[204:408 - 8].tolist() + perm[:8].tolist()) == kv.KV_OK
    assert kp.sync() == kv.KV_OK
    assert ora.swap_in(rid, off, np.concatenate([perm[204:400], perm[:8]])) == ko.OK
    assert np.array_equal(pool.cpu().numpy(), a.pool)
    kp.close()


def test_wait_event_orders_after_producer(gpu):
    """The caller's compute stream fills the blocks; kv_swap_out must wait for its event."""
    import torch
    g = W.Geometry(2, 8, 128, 16, "bf16", 2048)
    n = 1024
    pool = torch.zeros(g.pool_bytes, dtype=torch.uint8, device="cuda")
    staging = torch.zeros(n * g.S, dtype=torch.uint8).pin_memory()
    kp = kv.KVPool(g, pool, staging)
    big = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    compute = torch.cuda.Stream()
    ev = torch.cuda.Event()
    compute.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(compute):
        for _ in range(20):
            big.add_(1)  # keeps the stream busy so that a missing wait would be visible
        pool.fill_(7)
        ev.record(compute)
    ids = np.arange(n, dtype=np.int32)
    assert kp.swap_out([1], [0, n], ids, [n * g.B], wait_event=ev.cuda_event) == kv.KV_OK
    assert kp.sync() == kv.KV_OK
    assert int(staging.min()) == 7 and int(staging.max()) == 7
    kp.close()


def test_auto_path_choice(gpu):
    """KV_PATH_AUTO: zero-copy without a bounce buffer; with one, transfers of 8 MiB and more go
    through the copy engines.  Either way the bytes are the oracle's."""
    import torch
    g = W.Geometry(8, 8, 128, 16, "bf16", 400)             # block = 512 KiB
    seed = 0xA070
    a = HostPool(g, seed, slots=200)
    ora = a.oracle()
    pool = torch.from_numpy(a.pool.copy()).cuda()
    staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
    bounce = torch.zeros(2 * 40 * g.S, dtype=torch.uint8, device="cuda")
    kp = kv.KVPool(g, pool, staging, bounce=bounce)         # flags = KV_PATH_AUTO
    rng = np.random.default_rng(3)
    perm = rng.permutation(g.N).astype(np.int32)
    small, big = perm[:8], perm[8:8 + 100]                  # 4 MiB and 50 MiB
    assert kp.swap_out([1], [0, 8], small, [8 * g.B]) == kv.KV_OK
    assert kp.stats()["path"] == kv.KV_PATH_ZEROCOPY
    assert kp.swap_out([2], [0, 100], big, [100 * g.B]) == kv.KV_OK
    st = kp.stats()
    assert st["path"] == kv.KV_PATH_DMA and st["copies"] == 3 and st["launches"] == 3   # slices of 40 blocks
    assert kp.swap_in([2], [0, 100], perm[200:300]) == kv.KV_OK
    assert kp.stats()["path"] == kv.KV_PATH_DMA
    assert kp.swap_in([1], [0, 8], perm[300:308]) == kv.KV_OK
    assert kp.stats()["path"] == kv.KV_PATH_ZEROCOPY
    assert kp.sync() == kv.KV_OK
    assert ora.swap_out([1], [0, 8], small, [8 * g.B]) == ko.OK
    assert ora.swap_out([2], [0, 100], big, [100 * g.B]) == ko.OK
    assert ora.swap_in([2], [0, 100], perm[200:300]) == ko.OK
    assert ora.swap_in([1], [0, 8], perm[300:308]) == ko.OK
    assert np.array_equal(pool.cpu().numpy(), a.pool)
    assert np.array_equal(staging.numpy(), a.staging)
    kp.close()
    kp2 = kv.KVPool(g, pool, staging)                       # no bounce buffer: always zero-copy
    assert kp2.swap_out([2], [0, 100], big, [100 * g.B]) == kv.KV_OK
    assert kp2.stats()["path"] == kv.KV_PATH_ZEROCOPY
    kp2.close()


@pytest.mark.parametrize("base", ["zerocopy", "dma", "device"])
def test_per_request_events(gpu, base):
    """KV_REQ_EVENTS: the burst is cut at request boundaries; bytes stay the oracle's, every request
    can be polled / waited for, and the timeline is monotone in call order."""
    import torch
    flags = PATHS[base] | kv.KV_REQ_EVENTS
    g = W.Geometry(4, 8, 128, 16, "bf16", 900)              # block = 256 KiB
    seed = 0xE7E
    lens = W.request_lengths(seed, 12, ("uniform", 50, 900))
    off, ids, free = W.block_tables(seed, g.N, W.blocks_for(lens, g.B))
    rid = np.arange(1, 13, dtype=np.uint64)
    total = int(off[-1])
    a = HostPool(g, seed, slots=total + 2)
    ora = a.oracle()
    b = HostPool(g, seed, slots=total + 2)
    gpuad = GpuAdapter(b, flags, bounce_slots=16, tune=((kv.KV_TUNE_SEGMENT_BYTES, 2 << 20),))
    kp = gpuad.kp
    assert ora.swap_out(rid, off, ids, lens) == ko.OK
    gpuad._push()
    assert kp.swap_out(rid, off, ids, lens) == kv.KV_OK
    for r in rid[::-1]:
        assert kp.req_wait(r) == kv.KV_OK
        assert kp.req_poll(r) == 1
    tids, tms = kp.timeline()
    st = kp.stats()
    assert tids.tolist() == rid.tolist()
    assert (np.diff(tms) >= 0).all() and tms[0] > 0 and tms[-1] <= st["ms_total"] * 1.001
    # a 2 MiB floor = 8 blocks: requests of 4..57 blocks -> several segments, each one launch (zero-copy)
    nseg = len(np.unique(tms))
    assert nseg >= 6
    if base != "dma":
        assert st["launches"] == nseg
    gpuad._pull()
    assert np.array_equal(a.staging, b.staging) and np.array_equal(a.pool, b.pool)
    new = free[:total]
    assert ora.swap_in(rid, off, new) == ko.OK
    assert gpuad.swap_in(rid, off, new) == kv.KV_OK
    assert np.array_equal(a.pool, b.pool)
    tids, tms = kp.timeline()
    assert tids.tolist() == rid.tolist() and (np.diff(tms) >= 0).all()
    assert kp.req_poll(12345) == 1                           # never seen: nothing in flight
    gpuad.close()


def test_telemetry_and_time_budget(gpu):
    """Section 5.2: a write sized from the measured rate finishes inside the interval it was sized
    for.  The budget must equal the documented formula applied to the reported telemetry."""
    import time
    import torch
    g = W.config(2).geom
    pool = torch.zeros(600 * g.block_bytes, dtype=torch.uint8, device="cuda")
    g = W.Geometry(g.L, g.H, g.D, g.B, g.dtype, 600)
    staging = torch.zeros(520 * g.S, dtype=torch.uint8).pin_memory()
    kp = kv.KVPool(g, pool, staging)
    ids = np.arange(600, dtype=np.int32)
    # measure: a few large and a few small calls in each direction
    for it in range(4):
        assert kp.swap_out([1], [0, 128], ids[:128], [128 * g.B]) == kv.KV_OK
        assert kp.swap_in([1], [0, 128], ids[128:256]) == kv.KV_OK
        assert kp.swap_out([2], [0, 1], ids[300:301], [g.B]) == kv.KV_OK
        assert kp.swap_in([2], [0, 1], ids[301:302]) == kv.KV_OK
    assert kp.sync() == kv.KV_OK
    io = kp.io_stats()
    assert io["inflight_calls"] == [0, 0] and io["inflight_bytes"] == [0, 0]
    assert io["total_calls"] == [8, 8] and io["total_bytes"] == [4 * 129 * g.S] * 2
    for d in (0, 1):
        assert 20.0 < io["ewma_gbps"][d] < 70.0, io        # a PCIe Gen5 x16 link
        assert 5.0 < io["ewma_small_us"][d] < 2000.0, io
    interval = 3000.0                                       # a 3 ms decode step
    want = int((interval - io["ewma_small_us"][0]) * io["ewma_gbps"][0] * 1e3 / g.S)
    budget = kp.budget_blocks(0, interval)
    assert budget == want and 40 < budget < 120
    # a delta with that budget over a long request moves exactly `budget` blocks, within the interval
    assert kp.reserve(7, 500) == kv.KV_OK
    t0 = time.perf_counter()
    rc, moved = kp.swap_out_delta([7], [0, 500], ids[:500], [500 * g.B], budget=budget)
    assert rc == kv.KV_OK and moved.tolist() == [budget]
    assert kp.sync() == kv.KV_OK
    wall_us = (time.perf_counter() - t0) * 1e6
    assert kp.stats()["ms_total"] * 1e3 < 1.25 * interval, kp.stats()
    assert wall_us < 2.0 * interval
    # the same in one call, two requests, the second one more urgent
    assert kp.release(7) == kv.KV_OK
    assert kp.reserve(20, 200) == kv.KV_OK and kp.reserve(21, 200) == kv.KV_OK
    rc, moved, used = kp.swap_out_delta_timed([20, 21], [0, 200, 400], ids[:400], [200 * g.B] * 2, [0.5, 2.0], interval)
    assert rc == kv.KV_OK and 40 < used < 120 and moved.tolist() == [0, used]
    assert kp.sync() == kv.KV_OK
    assert kp.stats()["ms_total"] * 1e3 < 1.25 * interval
    assert kp.release(20) == kv.KV_OK and kp.release(21) == kv.KV_OK
    # queued work shrinks the budget: enqueue 256 blocks, ask again before they finish
    assert kp.swap_out([8], [0, 256], ids[:256], [256 * g.B]) == kv.KV_OK
    io2 = kp.io_stats()
    b2 = kp.budget_blocks(0, interval)
    if io2["inflight_bytes"][0]:
        assert b2 < budget
    assert kp.sync() == kv.KV_OK
    kp.close()


def test_write_queue_on_the_gpu(gpu):
    """kv_wq_post / kv_wq_drain with real transfers: decode steps post their growth, each drain writes a
    budgeted chunk in priority order; the arena must equal the oracle's after the same deltas, and a drain
    sized from an interval must finish inside it."""
    import torch
    g = W.Geometry(4, 8, 128, 16, "bf16", 700)              # 256 KiB blocks
    a = HostPool(g, 0xC0FFEE, slots=640)
    ora = a.oracle()
    pool = torch.from_numpy(a.pool.copy()).cuda()
    staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
    kp = kv.KVPool(g, pool, staging)
    rng = np.random.default_rng(12)
    perm = rng.permutation(g.N).astype(np.int32)
    rid = [1, 2, 3, 4]
    tables = {r: perm[150 * i:150 * (i + 1)] for i, r in enumerate(rid)}
    for r in rid:
        assert kp.reserve(r, 150) == kv.KV_OK and ora.reserve(r, 150) == ko.OK
    length = {r: 0 for r in rid}
    for step in range(12):
        prio = {}
        for r in rid:
            length[r] = min(length[r] + int(rng.integers(1, 12)) * g.B + int(rng.integers(0, g.B)), 150 * g.B)
            prio[r] = float(rng.integers(0, 3))
        nb = {r: -(-length[r] // g.B) for r in rid}
        off = np.concatenate([[0], np.cumsum([nb[r] for r in rid])]).astype(np.int32)
        blk = np.concatenate([tables[r][:nb[r]] for r in rid])
        assert kp.wq_post(rid, off, blk, [length[r] for r in rid], [prio[r] for r in rid]) == kv.KV_OK
        budget = int(rng.integers(1, 30))
        rc, wrote, pend, used = kp.wq_drain(block_budget=budget)
        assert rc == kv.KV_OK and used == budget
        order = sorted(rid, key=lambda r: (-prio[r], rid.index(r)))
        o2 = np.concatenate([[0], np.cumsum([nb[r] for r in order])]).astype(np.int32)
        rc, moved = ora.swap_out_delta(order, o2, np.concatenate([tables[r][:nb[r]] for r in order]),
                                       [length[r] for r in order], budget=budget)
        assert rc == ko.OK and int(moved.sum()) == wrote
    rc, wrote, pend, used = kp.wq_drain()                    # flush what is left
    assert rc == kv.KV_OK and pend == 0
    rc, moved = ora.swap_out_delta(rid, off, blk, [length[r] for r in rid])
    assert rc == ko.OK and int(moved.sum()) == wrote
    assert kp.sync() == kv.KV_OK
    assert np.array_equal(staging.numpy(), a.staging)
    for r in rid:
        assert kp.query(r)[1] == ora.query(r)[1]
    # a drain sized from an interval: warm the telemetry up, then 2 ms worth of a long request
    for r in rid:
        assert kp.release(r) == kv.KV_OK
    assert kp.wq_pending() == (kv.KV_OK, 0, 0)
    for it in range(3):
        assert kp.swap_out([9], [0, 400], perm[:400], [400 * g.B]) == kv.KV_OK
        assert kp.swap_in([9], [0, 400], perm[:400]) == kv.KV_OK
    assert kp.sync() == kv.KV_OK
    assert kp.release(9) == kv.KV_ENOENT                    # the swap-in gave its extent back
    assert kp.reserve(10, 600) == kv.KV_OK
    assert kp.wq_post([10], [0, 600], perm[:600], [600 * g.B]) == kv.KV_OK
    rc, wrote, pend, used = kp.wq_drain(interval_us=2000.0)
    assert rc == kv.KV_OK and wrote == used and 200 < used < 500 and pend == 600 - used   # ~55 GB/s * 2 ms / 256 KiB
    assert kp.sync() == kv.KV_OK
    assert kp.stats()["ms_total"] < 1.25 * 2.0
    kp.close()


def test_one_call_longer_than_the_descriptor_ring(gpu):
    """Token-level blocks (B = 1, 256 bytes each), one request of 150 000 of them through a bounce buffer
    that holds 2048 at a time: the call is cut into 74 slices whose descriptors together exceed the ring
    (65 536 entries), so late slices reuse the ring space of early ones of the same call."""
    import torch
    g = W.Geometry(1, 1, 64, 1, "f16", 200000)
    n = 150000
    a = HostPool(g, 0x4126, slots=n + 8)
    ora = a.oracle()
    pool = torch.from_numpy(a.pool.copy()).cuda()
    staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
    bounce = torch.zeros(2 * 2048 * g.S, dtype=torch.uint8, device="cuda")
    kp = kv.KVPool(g, pool, staging, bounce=bounce, flags=kv.KV_PATH_DMA)
    perm = np.random.default_rng(5).permutation(g.N).astype(np.int32)
    assert kp.swap_out([1], [0, n], perm[:n], [n]) == kv.KV_OK
    st = kp.stats()
    assert st["launches"] == 74 and st["copies"] == 74
    assert kp.swap_in([1], [0, n], perm[g.N - n:][::-1].copy()) == kv.KV_OK
    assert kp.sync() == kv.KV_OK
    assert ora.swap_out([1], [0, n], perm[:n], [n]) == ko.OK
    assert np.array_equal(staging.numpy(), a.staging)
    assert ora.swap_in([1], [0, n], perm[g.N - n:][::-1].copy()) == ko.OK
    assert np.array_equal(pool.cpu().numpy(), a.pool)
    kp.close()


def test_control_thread_polls_while_the_main_thread_enqueues(gpu):
    """Section 6: a control thread follows the transfers through events while the serving thread keeps
    enqueuing.  The handle serialises the two with its own lock; results stay the oracle's."""
    import threading
    import torch
    g = W.Geometry(8, 8, 128, 16, "bf16", 600)             # 512 KiB blocks
    a = HostPool(g, 0x7EAD, slots=320)
    ora = a.oracle()
    pool = torch.from_numpy(a.pool.copy()).cuda()
    staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
    kp = kv.KVPool(g, pool, staging, flags=kv.KV_REQ_EVENTS)
    perm = np.random.default_rng(21).permutation(g.N).astype(np.int32)
    stop, seen, errors = threading.Event(), {"polls": 0, "busy": 0}, []

    def control():
        try:
            while not stop.is_set():
                for r in range(1, 9):
                    rc = kp.req_poll(r)
                    assert rc in (0, 1), rc
                    seen["busy"] += rc == 0
                    seen["polls"] += 1
                io = kp.io_stats()
                assert min(io["inflight_calls"]) >= 0 and min(io["inflight_bytes"]) >= 0
        except Exception as e:                              # noqa: BLE001 - reported by the main thread
            errors.append(e)

    t = threading.Thread(target=control)
    t.start()
    rid = list(range(1, 9))
    off = np.arange(0, 9 * 36, 36, dtype=np.int32)[:9]
    lens = [36 * g.B] * 8
    try:
        for it in range(6):
            src = np.roll(perm, 31 * it)[:288]
            dst = np.roll(perm, 31 * it)[288:576]
            assert kp.swap_out(rid, off, src, lens) == kv.KV_OK
            assert kp.swap_in(rid, off, dst) == kv.KV_OK
            assert ora.swap_out(rid, off, src, lens) == ko.OK and ora.swap_in(rid, off, dst) == ko.OK
            assert kp.req_wait(rid[it % 8]) == kv.KV_OK
    finally:
        stop.set()
        t.join(60)
    assert not t.is_alive() and not errors, errors
    assert kp.sync() == kv.KV_OK
    assert seen["polls"] > 100
    assert np.array_equal(pool.cpu().numpy(), a.pool) and np.array_equal(staging.numpy(), a.staging)
    kp.close()


def test_reserved_extent_waits_for_the_previous_owners_swap_in(gpu):
    """Request A is swapped in without KV_KEEP_STAGING (its slots are free again the moment the call returns)
    while the load stream is held back by a bounded spin kernel; request B then reserves the same slots and is
    swapped out into them.  B's write must wait for A's read: A's new blocks have to receive A's data."""
    import torch
    g = W.Geometry(8, 8, 128, 16, "bf16", 300)              # 512 KiB blocks
    a = HostPool(g, 0xABBA, slots=64)
    ora = a.oracle()
    pool = torch.from_numpy(a.pool.copy()).cuda()
    staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
    evict, load = torch.cuda.Stream(), torch.cuda.Stream()
    kp = kv.KVPool(g, pool, staging, evict_stream=evict, load_stream=load)
    perm = np.random.default_rng(2).permutation(g.N).astype(np.int32)
    A_src, A_dst, B_src = perm[:60], perm[60:120], perm[120:180]
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda._sleep(1_000_000)                              # first launch of the spin kernel: not timed
    t0.record(); torch.cuda._sleep(20_000_000); t1.record(); t1.synchronize()
    spin = int(100.0 / max(t0.elapsed_time(t1), 1e-3) * 20_000_000)   # about 100 ms

    def script(o, hold):
        assert o.swap_out([1], [0, 60], A_src, [60 * g.B]) == 0
        hold()
        assert o.swap_in([1], [0, 60], A_dst, 0) == 0       # extent of request 1 is released here
        assert o.reserve(2, 60) == 0                         # first fit: the same 60 slots
        assert o.swap_out([2], [0, 60], B_src, [60 * g.B]) == 0

    def hold():
        assert kp.sync() == kv.KV_OK
        with torch.cuda.stream(load):
            torch.cuda._sleep(spin)

    script(kp, hold)
    assert kp.query(2)[1]["offset"] == 0                     # B really sits on A's old slots
    assert kp.sync() == kv.KV_OK
    script(ora, lambda: None)
    assert np.array_equal(pool.cpu().numpy(), a.pool), "request 1 was loaded from slots request 2 had already overwritten"
    assert np.array_equal(staging.numpy(), a.staging)
    kp.close()


def test_new_extent_over_slots_of_two_previous_owners(gpu):
    """An extent that covers the old slots of two requests: one whose swap-in (load stream, held back) still reads
    its slots, and one whose eviction (evict stream) is the newer call.  The newer same-stream call must not hide
    the older dependency on the other stream."""
    import torch
    g = W.Geometry(8, 8, 128, 16, "bf16", 400)              # 512 KiB blocks
    a = HostPool(g, 0xD0D0, slots=80)
    ora = a.oracle()
    pool = torch.from_numpy(a.pool.copy()).cuda()
    staging = torch.full((len(a.staging),), CANARY, dtype=torch.uint8).pin_memory()
    evict, load = torch.cuda.Stream(), torch.cuda.Stream()
    kp = kv.KVPool(g, pool, staging, evict_stream=evict, load_stream=load)
    perm = np.random.default_rng(6).permutation(g.N).astype(np.int32)
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda._sleep(1_000_000)                              # first launch of the spin kernel: not timed
    t0.record(); torch.cuda._sleep(20_000_000); t1.record(); t1.synchronize()
    per_ms = 20_000_000 / max(t0.elapsed_time(t1), 1e-3)

    def script(o, hold):
        assert o.reserve(1, 30) == 0                                      # slots [0, 30)
        assert o.reserve(4, 1) == 0                                       # [30, 31): keeps the two runs apart for now
        assert o.swap_out([1], [0, 30], perm[:30], [30 * g.B]) == 0
        hold()
        assert o.swap_in([1], [0, 30], perm[30:60], 0) == 0               # load stream; gives [0, 30) up
        assert o.reserve(3, 40) == 0                                      # does not fit there: [31, 71)
        assert o.swap_out([3], [0, 40], perm[60:100], [40 * g.B]) == 0    # evict stream, the newer call
        assert o.release(3) == 0
        assert o.release(4) == 0
        assert o.reserve(2, 70) == 0                                      # [0, 70): over both
        assert o.swap_out([2], [0, 70], perm[100:170], [70 * g.B]) == 0

    def hold():
        assert kp.sync() == kv.KV_OK
        with torch.cuda.stream(load):
            torch.cuda._sleep(int(120 * per_ms))
        with torch.cuda.stream(evict):
            torch.cuda._sleep(int(20 * per_ms))

    script(kp, hold)
    assert kp.query(2)[1]["offset"] == 0 and kp.query(2)[1]["cap"] == 70
    assert kp.sync() == kv.KV_OK
    script(ora, lambda: None)
    assert np.array_equal(pool.cpu().numpy(), a.pool), "request 1 was loaded from slots that request 2 had overwritten"
    assert np.array_equal(staging.numpy(), a.staging)
    kp.close()


def test_create_checks_memory_kinds(gpu):
    import torch
    g = W.Geometry(2, 4, 64, 16, "f16", 64)
    pool = torch.zeros(g.pool_bytes, dtype=torch.uint8, device="cuda")
    pinned = torch.zeros(8 * g.S, dtype=torch.uint8).pin_memory()
    pageable = torch.zeros(8 * g.S, dtype=torch.uint8)
    with pytest.raises(kv.KVSwapError):
        kv.KVPool(g, pool, pageable)                       # arena must be pinned
    with pytest.raises(kv.KVSwapError):
        kv.KVPool(g, pinned, pinned)                       # pool must be device memory
    with pytest.raises(kv.KVSwapError):
        kv.KVPool(g, pool, pinned, flags=kv.KV_STAGING_DEVICE)  # device arena flag, host pointer
    small = torch.zeros(g.pool_bytes // 2, dtype=torch.uint8, device="cuda")
    big_geom = W.Geometry(2, 4, 64, 16, "f16", 1 << 20)     # strides run far past the allocation
    with pytest.raises(kv.KVSwapError):
        kv.KVPool(big_geom, small, pinned)
    kv.KVPool(g, pool, pinned).close()
