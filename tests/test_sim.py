"""The serving-loop simulator: scheduler + swap library + synthetic decode model.

CPU: the swap library runs plan-only (bookkeeping and descriptor lists, no bytes); the tests check
the loop's invariants and the qualitative claim the paper makes for bursts (preemption on buffered
requests cuts time-to-first-token, Section 7.3).  GPU: the same loop moves real KV blocks; at the
end every request's blocks must hold exactly the pattern written at allocation, however often the
request was preempted, written through, resumed into other blocks or recomputed.
"""
import numpy as np
import pytest

from paper_2510_02758_amd import kvswap as kv
from paper_2510_02758_amd import sim as S
from paper_2510_02758_amd import workloads as W

GEOM = W.Geometry(2, 2, 64, 16, "bf16", 1)      # 8 KiB blocks; the pool size comes from the SimConfig


def make(policy, n=24, gpu_blocks=260, seed=3, **kw):
    cfg = S.SimConfig(geom=GEOM, gpu_blocks=gpu_blocks, arena_blocks=2000, max_running=6, interval=0.5,
                      policy=policy, **kw)
    reqs = S.burst_requests(seed, n, prompt_mean=256, out_mean=384, rates=(15.0, 20.0))
    return cfg, reqs


def run(policy, **kw):
    cfg, reqs = make(policy, **kw)
    sim = S.Simulator(cfg, reqs)
    out = sim.run(max_time=2000.0)
    # conservation: every block is free again, nothing is left in the arena
    assert sorted(sim.free) == list(range(cfg.gpu_blocks))
    for r in reqs:
        assert r.state == "done" and len(r.t_gen) == r.out_len and r.t_gen == sorted(r.t_gen)
        assert sim.kp.query(r.rid)[0] == kv.KV_ENOENT
    sim.close()
    return out, reqs


def test_tokenflow_finishes_everything_and_preempts():
    out, reqs = run("tokenflow")
    assert out["finished"] == out["of"] == 24
    assert out["preemptions"] > 0 and out["blocks_moved"]["write_through"] > 0
    # write-through leaves only tails to move at preemption time: far fewer blocks than are loaded back
    assert out["blocks_moved"]["evict"] < out["blocks_moved"]["load"]


def test_burst_tokenflow_against_fcfs():
    """24 requests at once, 6 decode slots, readers at 15-20 tokens/s against ~43 tokens/s of decode
    speed: running requests pile up buffer while the others wait.  Preempting the buffered ones gives
    everyone a first token sooner and keeps more of the generated tokens timely."""
    tf, _ = run("tokenflow")
    ff, _ = run("fcfs")
    assert ff["preemptions"] == 0
    assert tf["ttft_mean_s"] < 0.6 * ff["ttft_mean_s"]
    assert tf["effective_throughput_tok_s"] > ff["effective_throughput_tok_s"]
    assert tf["throughput_tok_s"] > 0.85 * ff["throughput_tok_s"]      # preemption costs little raw throughput


def test_without_write_through_evictions_move_whole_requests():
    wt, _ = run("tokenflow", write_through=True)
    cold, _ = run("tokenflow", write_through=False)
    assert cold["blocks_moved"]["write_through"] == 0
    assert cold["blocks_moved"]["evict"] > 5 * max(1, wt["blocks_moved"]["evict"])


@pytest.mark.gpu
@pytest.mark.parametrize("sync_io", [True, False])
@pytest.mark.parametrize("write_through", [True, False])
def test_sim_moves_real_kv_and_keeps_it_intact(gpu, write_through, sync_io):
    """sync_io False: no host wait anywhere in the loop; evictions, loads and the model's writes are
    ordered by events only (the library's between its two streams, the loop's towards the model)."""
    import torch
    cfg, reqs = make("tokenflow", n=16, gpu_blocks=200, write_through=write_through, prefill_per_token=2e-6)
    cfg.sync_io = sync_io
    g = W.Geometry(GEOM.L, GEOM.H, GEOM.D, GEOM.B, GEOM.dtype, cfg.gpu_blocks)
    pool = torch.zeros(g.pool_bytes, dtype=torch.uint8, device=gpu)
    staging = torch.zeros(cfg.arena_blocks * g.S, dtype=torch.uint8).pin_memory()
    sim = S.Simulator(cfg, reqs, pool=pool, staging=staging, seed=77)
    out = sim.run(max_time=2000.0)
    assert out["finished"] == 16 and out["preemptions"] > 0
    assert out["kv_content_ok"], "a request's KV changed across preempt / resume cycles"
    sim.close()


@pytest.mark.gpu
@pytest.mark.parametrize("sync_io", [True, False])
def test_sim_at_8b_block_size(gpu, sync_io):
    """2 MiB blocks (Llama-3-8B shape), 32 requests, dozens of preemptions: large enough for a missing
    stream dependency between the model's writes and the write-through to show up as wrong bytes."""
    import torch
    g = W.Geometry(32, 8, 128, 16, "bf16", 1200)
    cfg = S.SimConfig(geom=g, gpu_blocks=g.N, arena_blocks=5000, max_running=16, interval=0.5, policy="tokenflow",
                      prefill_per_token=2e-4, sync_io=sync_io)
    reqs = S.burst_requests(11, 32, prompt_mean=512, out_mean=768, rates=(15.0, 20.0))
    pool = torch.zeros(g.pool_bytes, dtype=torch.uint8, device=gpu)
    staging = torch.zeros(cfg.arena_blocks * g.S, dtype=torch.uint8).pin_memory()
    sim = S.Simulator(cfg, reqs, pool=pool, staging=staging, seed=5)
    out = sim.run(max_time=4000.0)
    assert out["finished"] == 32 and out["preemptions"] > 20 and out["blocks_moved"]["load"] > 500, out
    assert out["kv_content_ok"]
    assert sorted(sim.free) == list(range(g.N))
    sim.close()
