"""GPU parity at the benchmark's full sizes (BASELINE configs 2-5), in the launch
configuration bench.py times.  The pools (78-186 GiB) have no host mirror: they are
address coded, so
  * sampled requests go through the CPU oracle on a compact mirror and are compared
    byte for byte with the library's staging extents and destination blocks;
  * every moved block is checked on the device against the closed form (block new[j]
    must hold the fill of block old[j]);
  * the complement is checked whole: the set of blocks whose content differs from their
    own fill must be exactly the set of destination blocks.
Bar: bit-exact.
"""
import os

import numpy as np
import pytest

import devcheck as DC
from oracle import kv_oracle as ko
from paper_2510_02758_amd import kvswap as kv
from paper_2510_02758_amd import workloads as W

pytestmark = pytest.mark.gpu
CANARY = 0xA5


@pytest.fixture(autouse=True)
def _release_cached_memory():
    """These tests take most of the box's pinnable memory (about 64 GiB) one after another:
    give back what torch's caching allocators hold before and after each."""
    import gc
    import torch

    def drop():
        gc.collect()
        if torch.cuda.is_available():
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
            if hasattr(torch._C, "_host_emptyCache"):
                torch._C._host_emptyCache()
    drop()
    yield
    drop()


def _pinned(torch, nbytes):
    """A canary-filled pinned arena; boxes that cannot pin this much skip the test."""
    try:
        t = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    except (RuntimeError, MemoryError) as e:      # torch.AcceleratorError derives from RuntimeError
        pytest.skip("cannot pin %.1f GiB of host memory on this box: %s" % (nbytes / 2**30, str(e)[:80]))
    t.fill_(CANARY)
    return t


def _oracle_on_sample(g, strides, seed, rows, off, ids, lens, new_ids, scale_seed=None):
    """Run swap-out + swap-in of the sampled requests through the oracle on a compact mirror.
    Returns (expected staging image per request, expected destination block images)."""
    soff, sids = W.csr_take(off, ids, rows)
    total = int(soff[-1])
    gc, pool, scale = DC.compact_mirror(g, strides, seed, sids, total, scale_seed)
    staging = np.full(total * gc.S, CANARY, np.uint8)
    ora = ko.Oracle(gc.L, gc.H, gc.D, gc.B, gc.e, gc.N, pool, gc.strides, staging, scale=scale,
                    scale_strides=gc.scale_strides if g.scales else None)
    rid = np.arange(1, len(rows) + 1, dtype=np.uint64)
    assert ora.swap_out(rid, soff, np.arange(total), lens[rows]) == ko.OK
    stage_img = staging.copy().reshape(total, gc.S)
    assert ora.swap_in(rid, soff, np.arange(total, 2 * total)) == ko.OK
    pv = pool.reshape(gc.L, 2, gc.N, gc.chunk)[:, :, total:, :]          # destination blocks
    dest_img = pv.transpose(2, 0, 1, 3).reshape(total, -1)
    return soff, stage_img, dest_img


def _device_blocks(pool, g, strides, phys):
    """Download blocks `phys` as [n, 2L*chunk] in (l, c) order."""
    import torch
    ls, ks, bs = strides
    idx = torch.as_tensor(np.asarray(phys, dtype=np.int64), device=pool.device)
    parts = []
    for l in range(g.L):
        for c in range(2):
            rows = torch.as_strided(pool, (g.N, g.chunk), (bs, 1), storage_offset=l * ls + c * ks)
            parts.append(rows.index_select(0, idx))
    return torch.stack(parts, dim=1).reshape(len(phys), -1).cpu().numpy()


# every configuration runs on its own seed and on two further seeds of the same recipe (other lengths, tables, fill)
SEEDS = pytest.mark.parametrize("variant", [0, 1, 2], ids=["seed", "seed+1", "seed+2"])


@SEEDS
def test_config2_llama8b_burst64(gpu, variant):
    import torch
    wl = W.config(2, variant=variant)
    g = wl.geom
    lens = W.request_lengths(wl.seed, wl.n_requests, wl.length_dist)
    off, ids, free = W.block_tables(wl.seed, g.N, W.blocks_for(lens, g.B))
    n, total = wl.n_requests, int(off[-1])
    assert 32 * n <= total <= 256 * n
    new = free[:total]
    rid = np.arange(1, n + 1, dtype=np.uint64)
    pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device=gpu)
    W.fill_buffer_torch(wl.seed, pool, g.dtype)
    spare = 3
    staging = _pinned(torch, (total + spare) * g.S)
    kp = kv.KVPool(g, pool, staging)                      # default path, default launch shape

    assert kp.swap_out(rid, off, ids, lens) == kv.KV_OK
    assert kp.sync() == kv.KV_OK
    st = kp.stats()
    assert st["blocks"] == total and st["bytes"] == total * g.S
    sv = staging.numpy()[: (total + spare) * g.S].reshape(total + spare, g.S)
    assert (sv[total:] == CANARY).all(), "slots beyond the extents were written"
    # closed form on the first and last block of every request
    for i in range(n):
        rc, q = kp.query(rid[i])
        assert rc == 0 and q["offset"] == int(off[i]) * g.S and q["staged"] == off[i + 1] - off[i]
        ends = [int(off[i]), int(off[i + 1]) - 1]
        want = DC.host_blocks(g, g.strides, wl.seed, ids[ends])
        assert np.array_equal(sv[ends], want), "request %d" % i
    # sampled requests through the oracle
    rows = [0, 21, 42, 63]
    soff, stage_img, dest_img = _oracle_on_sample(g, g.strides, wl.seed, rows, off, ids, lens, new)
    for k, r in enumerate(rows):
        got = sv[off[r]:off[r + 1]]
        assert np.array_equal(got, stage_img[soff[k]:soff[k + 1]]), "staging of request %d differs from the oracle" % r
    assert DC.count_wrong_blocks(pool, g, g.strides, wl.seed, ids, ids) == 0   # swap-out only reads

    # the allocator hands the victims' blocks to someone else
    dirty = torch.as_tensor(ids.astype(np.int64), device=gpu)
    for l in range(g.L):
        for c in range(2):
            rowsv = torch.as_strided(pool, (g.N, g.chunk), (g.strides[2], 1),
                                     storage_offset=l * g.strides[0] + c * g.strides[1])
            rowsv.index_fill_(0, dirty, 0x3C)
    assert kp.swap_in(rid, off, new) == kv.KV_OK
    assert kp.sync() == kv.KV_OK
    assert DC.count_wrong_blocks(pool, g, g.strides, wl.seed, new, ids) == 0, "a destination block is wrong"
    for k, r in enumerate(rows):
        got = _device_blocks(pool, g, g.strides, new[off[r]:off[r + 1]])
        assert np.array_equal(got, dest_img[soff[k]:soff[k + 1]]), "pool blocks of request %d differ from the oracle" % r
    changed = DC.changed_blocks(pool, g, g.strides, wl.seed)
    assert np.array_equal(changed, np.sort(np.concatenate([ids, new]))), "a block outside the tables was touched"
    assert (sv[total:] == CANARY).all()
    for r in rid:
        assert kp.query(r)[0] == kv.KV_ENOENT
    kp.close()


@SEEDS
def test_config3_write_through_burst(gpu, variant):
    """256 requests, log-normal lengths, 64 decode steps of one token each with a delta per step,
    then 32 requests preempted (tail flush) and resumed into fresh blocks."""
    import torch
    wl = W.config(3, variant=variant)
    g = wl.geom
    n, steps = wl.n_requests, 64
    lens = W.request_lengths(wl.seed, n, wl.length_dist).astype(np.int64)
    assert lens.min() >= 16 and lens.max() + steps <= 8192
    final_nb = W.blocks_for(lens + steps, g.B)
    off, ids, free = W.block_tables(wl.seed, g.N, final_nb)       # each request's blocks, allocation order
    rid = np.arange(1, n + 1, dtype=np.uint64)
    pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device=gpu)
    W.fill_buffer_torch(wl.seed, pool, g.dtype)
    total = int(off[-1])
    staging = _pinned(torch, total * g.S)
    kp = kv.KVPool(g, pool, staging)
    for i in range(n):
        assert kp.reserve(rid[i], int(final_nb[i])) == kv.KV_OK

    sample = list(range(0, n, 16))                                  # 16 requests go through the oracle as well
    soff, sids = W.csr_take(off, ids, sample)
    stotal = int(soff[-1])
    gc, mpool, _ = DC.compact_mirror(g, g.strides, wl.seed, sids, stotal)
    mstaging = np.full(stotal * gc.S, CANARY, np.uint8)
    ora = ko.Oracle(gc.L, gc.H, gc.D, gc.B, gc.e, gc.N, mpool, gc.strides, mstaging)
    srid = rid[sample]
    for k in range(len(sample)):
        assert ora.reserve(srid[k], int(final_nb[sample[k]])) == ko.OK

    def tables(cur):
        nb = W.blocks_for(cur, g.B)
        o = np.zeros(n + 1, np.int32)
        o[1:] = np.cumsum(nb)
        flat = np.concatenate([ids[off[i]:off[i] + nb[i]] for i in range(n)])
        so = np.zeros(len(sample) + 1, np.int32)
        so[1:] = np.cumsum(nb[sample])
        sflat = np.concatenate([np.arange(soff[k], soff[k] + nb[sample[k]]) for k in range(len(sample))])
        return o, flat, so, sflat

    cur = lens.copy()
    wm = np.zeros(n, np.int64)
    moved_blocks = 0
    for s in range(steps + 1):                                      # s = 0 is the priming delta
        if s:
            cur += 1
        o, flat, so, sflat = tables(cur)
        rc, moved = kp.swap_out_delta(rid, o, flat, cur)
        assert rc == kv.KV_OK
        assert np.array_equal(moved, cur // g.B - wm), "step %d: blocks_moved" % s   # closed form
        wm = cur // g.B
        moved_blocks += int(moved.sum())
        rc, omoved = ora.swap_out_delta(srid, so, sflat, cur[sample])
        assert rc == ko.OK and np.array_equal(omoved, moved[sample])
    assert kp.sync() == kv.KV_OK
    assert moved_blocks == int((cur // g.B).sum())
    assert int((cur // g.B - lens // g.B).sum()) == 4 * n            # 64 tokens = exactly 4 blocks each
    sv = staging.numpy().reshape(total, g.S)
    msv = mstaging.reshape(stotal, gc.S)
    for k, r in enumerate(sample):
        assert np.array_equal(sv[off[r]:off[r + 1]], msv[soff[k]:soff[k + 1]]), "request %d" % r
    # every request: the last full block is staged, the tail slot (if any) is still canary
    for i in range(n):
        j = int(wm[i]) - 1
        assert np.array_equal(sv[off[i] + j], DC.host_blocks(g, g.strides, wl.seed, [ids[off[i] + j]])[0])
        if cur[i] % g.B:
            assert (sv[off[i] + wm[i]] == CANARY).all()

    # preempt 32 requests: only the tail is left to write; then resume them elsewhere
    victims = np.sort(W.pick(wl.seed, n, wl.n_preempt))
    o, flat, _, _ = tables(cur)
    vo, vflat = W.csr_take(o, flat, victims)
    rc, moved = kp.swap_out_delta(rid[victims], vo, vflat, cur[victims], flags=kv.KV_DELTA_INCLUDE_TAIL)
    assert rc == kv.KV_OK and np.array_equal(moved, (cur[victims] % g.B != 0).astype(np.int32))
    new = free[: len(vflat)]
    assert kp.swap_in(rid[victims], vo, new) == kv.KV_OK             # no sync in between: the library orders it
    assert kp.sync() == kv.KV_OK
    assert DC.count_wrong_blocks(pool, g, g.strides, wl.seed, new, vflat) == 0
    changed = DC.changed_blocks(pool, g, g.strides, wl.seed)
    assert np.array_equal(changed, np.sort(new))
    for v in victims:
        assert kp.query(rid[v])[0] == kv.KV_ENOENT
    kp.close()


def _sample_rows(seed, wave, nb_rows, max_blocks):
    """Seeded sample of a wave's requests for the oracle: the wave's rows in a seeded random order, taken while the
    sample stays within max_blocks; at least one (the smallest, if none fits)."""
    rng = np.random.default_rng((seed << 8) + wave)
    order = rng.permutation(len(nb_rows))
    picked, used = [], 0
    for r in order:
        if used + int(nb_rows[r]) <= max_blocks:
            picked.append(int(r))
            used += int(nb_rows[r])
    if not picked:
        picked = [int(np.argmin(nb_rows))]
    return sorted(picked)


def _waves(nb, slots, limit_blocks):
    out, done = [], 0
    while done < len(nb):
        k = done
        while k < len(nb) and int(nb[done:k + 1].sum()) <= min(slots, limit_blocks):
            k += 1
        assert k > done
        out.append(np.arange(done, k))
        done = k
    return out


@SEEDS
def test_config4_llama70b_fragmented_waves(gpu, variant):
    """80 layers, 200 GB pool (38 146 blocks of 5 MiB), tables drawn from a half-freed pool (another random half for
    every wave).  The 128 requests total ~350 GiB, more than the free half: they are preempted and resumed in waves
    through a 40 GiB arena, ALL of them (the two further seeds: their first two waves).  The test tracks, on the host,
    whose original fill every block must hold afterwards; every moved block is checked on the device, a seeded sample
    of each wave's requests through the oracle."""
    import torch
    wl = W.config(4, variant=variant)
    g = wl.geom
    assert g.N == 38146 and g.block_bytes == 5 << 20
    lens = W.request_lengths(wl.seed, wl.n_requests, wl.length_dist)
    nb = W.blocks_for(lens, g.B)
    assert wl.n_requests == 128 and int(nb.sum()) * g.S > 300 << 30
    pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device=gpu)
    W.fill_buffer_torch(wl.seed, pool, g.dtype)
    arena_slots = (40 << 30) // g.S
    staging = _pinned(torch, arena_slots * g.S)
    kp = kv.KVPool(g, pool, staging)
    content = np.arange(g.N, dtype=np.int64)          # content[b] = block whose original fill b holds
    waves = _waves(nb, arena_slots, limit_blocks=9000)  # a wave and its destinations both come out of the free half
    assert len(waves) >= 9 and sum(len(w) for w in waves) == 128
    if variant:
        waves = waves[:2]
    done = 0
    for wave, rows in enumerate(waves):
        off, ids, free = W.fragmented_tables(wl.seed + wave, g.N, nb[rows], 0.5)
        rid = (rows + 1).astype(np.uint64)
        new = free[: len(ids)]
        assert len(new) == len(ids)
        print("config 4: wave %d, requests %d..%d, %d blocks" % (wave, rows[0], rows[-1], len(ids)), flush=True)
        assert kp.swap_out(rid, off, ids, lens[rows]) == kv.KV_OK
        assert kp.swap_in(rid, off, new) == kv.KV_OK       # back to back: ordered by the library
        assert kp.sync() == kv.KV_OK
        src_content = content[ids]
        content[new] = src_content
        assert DC.count_wrong_blocks(pool, g, g.strides, wl.seed, new, src_content) == 0, "wave %d" % wave
        sample = _sample_rows(wl.seed, wave, nb[rows], 200)
        soff, stage_img, dest_img = _oracle_on_sample(g, g.strides, wl.seed, sample, off, src_content.astype(np.int32),
                                                      lens[rows], new)
        for k, r in enumerate(sample):
            got = _device_blocks(pool, g, g.strides, new[off[r]:off[r + 1]])
            assert np.array_equal(got, dest_img[soff[k]:soff[k + 1]]), "wave %d request %d" % (wave, rows[r])
            q = staging.numpy()[int(off[r]) * g.S: int(off[r + 1]) * g.S].reshape(-1, g.S)
            assert np.array_equal(q, stage_img[soff[k]:soff[k + 1]]), "wave %d request %d staging" % (wave, rows[r])
        done += len(rows)
    assert done == (128 if not variant else sum(len(w) for w in waves))
    changed = DC.changed_blocks(pool, g, g.strides, wl.seed)
    assert np.array_equal(changed, np.flatnonzero(content != np.arange(g.N))), "a foreign block was touched"
    kp.close()


@SEEDS
def test_config5_fp8_scales_under_contention(gpu, variant):
    """fp8 KV with fp32 scales per (block, layer, K|V, head): 8 MiB + 8 KiB per block.  All 512 requests (~515 GiB,
    more than the GPU holds) go out and come back in waves through a 32 GiB arena (the two further seeds: their first
    two waves); every fourth wave is swapped in while another stream streams through HBM.  Data and scales: every
    moved block checked on the device, a seeded sample of each wave through the oracle, the complement at the end."""
    import torch
    wl = W.config(5, variant=variant)
    g = wl.geom
    assert g.chunk == 128 << 10 and g.scale_chunk == 128 and g.S == (8 << 20) + (8 << 10)
    sseed = wl.seed ^ 0x5CA1E
    lens = W.request_lengths(wl.seed, wl.n_requests, wl.length_dist)
    nb = W.blocks_for(lens, g.B)
    assert wl.n_requests == 512 and int(nb.sum()) * g.S > 288 * 10**9
    pool = torch.empty(g.pool_bytes, dtype=torch.uint8, device=gpu)
    scale = torch.empty(g.scale_bytes, dtype=torch.uint8, device=gpu)
    W.fill_buffer_torch(wl.seed, pool, g.dtype)
    W.fill_buffer_torch(sseed, scale, "raw")
    arena_slots = (32 << 30) // g.S
    staging = _pinned(torch, (arena_slots + 1) * g.S)
    kp = kv.KVPool(g, pool, staging, scale=scale)
    sv = staging.numpy().reshape(arena_slots + 1, g.S)
    noise = torch.empty(8 << 30, dtype=torch.uint8, device=gpu)
    side = torch.cuda.Stream()
    content = np.arange(g.N, dtype=np.int64)
    waves = _waves(nb, arena_slots, limit_blocks=(g.N - 8) // 2)
    assert sum(len(w) for w in waves) == 512
    if variant:
        waves = waves[:2]
    done = 0
    for wave, rows in enumerate(waves):
        off, ids, free = W.block_tables(wl.seed + wave, g.N, nb[rows])
        total = int(off[-1])
        new = free[:total]
        rid = (rows + 1).astype(np.uint64)
        print("config 5: wave %d, requests %d..%d, %d blocks" % (wave, rows[0], rows[-1], total), flush=True)
        assert kp.swap_out(rid, off, ids, lens[rows]) == kv.KV_OK
        assert kp.sync() == kv.KV_OK
        src_content = content[ids]
        assert (sv[arena_slots] == CANARY).all()
        # sampled requests through the oracle (data + scales)
        sample = _sample_rows(wl.seed, wave, nb[rows], 24)
        soff, stage_img, dest_img = _oracle_on_sample(g, g.strides, wl.seed, sample, off, src_content.astype(np.int32),
                                                      lens[rows], new, sseed)
        for q, r in enumerate(sample):
            assert np.array_equal(sv[off[r]:off[r + 1]], stage_img[soff[q]:soff[q + 1]]), "wave %d request %d" % (wave, rows[r])
        # closed form for the scale part of every request's first block
        for i in range(len(rows)):
            want = DC.host_blocks(g, g.scale_strides, sseed, [src_content[off[i]]], dtype="raw", width=g.scale_chunk)[0]
            assert np.array_equal(sv[off[i], g.block_bytes:], want)
        if wave % 4 == 0:      # this wave comes back while a streaming kernel keeps HBM busy on another stream
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for _ in range(40):
                    noise.add_(1)
        assert kp.swap_in(rid, off, new) == kv.KV_OK
        assert kp.sync() == kv.KV_OK
        side.synchronize()
        content[new] = src_content
        assert DC.count_wrong_blocks(pool, g, g.strides, wl.seed, new, src_content) == 0, "wave %d" % wave
        assert DC.count_wrong_blocks(scale, g, g.scale_strides, sseed, new, src_content, dtype="raw",
                                     width=g.scale_chunk) == 0, "wave %d scales" % wave
        done += len(rows)
    assert done == (512 if not variant else sum(len(w) for w in waves))
    moved = np.flatnonzero(content != np.arange(g.N))
    assert np.array_equal(DC.changed_blocks(pool, g, g.strides, wl.seed), moved)
    assert np.array_equal(DC.changed_blocks(scale, g, g.scale_strides, sseed, dtype="raw", width=g.scale_chunk), moved)
    kp.close()


@pytest.mark.gpu
def test_bench_line_has_the_agreed_shape(gpu):
    """bench.py on a small pool of the headline shape (same steps, same launches, two waves): one JSON line with the
    agreed fields."""
    import json
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--blocks", "8000", "--steps", "2", "--warmup", "1",
                        "--cpu-sample", "1", "--only", "headline,1", "--quick"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "configs"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["unit"] == "GB/s" and d["dtype"] == "u8"
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"] and d["config"]["workload"].startswith("configs[3]")
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and 0.3 < rf["frac"] < 1.0
    assert "traffic" in rf and rf["algorithmic_bytes_per_block"] == 2 * (5 << 20)
    assert abs(rf["bytes_per_launch"] - rf["blocks_per_launch"] * rf["algorithmic_bytes_per_block"]) < 2 * (5 << 20)
    assert rf["measured_scattered_copy_ceiling_gbps"] > 1000
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] == 1 and cb["unit"] == "GB/s" and cb["value"] > 0 and cb["sample"]
    assert cb["all_cores"] >= 1 and cb["all_cores_value"] > 0
    assert 30.0 < d["value"] < 64.0 and 30.0 < d["legs"]["d2h_gbps"] < 64.0 and 30.0 < d["legs"]["h2d_gbps"] < 64.0
    assert "configs[0]" in d["configs"]
