/* The C ABI used from plain C99, without a GPU: a plan-only pool (no HIP call is made), one swap-out,
 * a budgeted write-through, a swap-in, eviction and loading in one call, the allocation-free move,
 * and one scheduling round.  Built and run by
 * tests/test_native_sanitizers.py; exits 0 when every call answers as the headers say. */
#include <stdio.h>
#include <string.h>

#include "kvsched.h"
#include "kvswap.h"

#define CHECK(cond)                                                  \
  do {                                                               \
    if (!(cond)) {                                                   \
      fprintf(stderr, "%s:%d: %s failed\n", __FILE__, __LINE__, #cond); \
      return 1;                                                      \
    }                                                                \
  } while (0)

int main(void) {
  kv_pool_config cfg;
  kv_pool* p = NULL;
  memset(&cfg, 0, sizeof(cfg));
  cfg.struct_size = sizeof(cfg);
  cfg.num_layers = 2;
  cfg.num_kv_heads = 2;
  cfg.head_dim = 16;
  cfg.block_size = 4;
  cfg.dtype = KV_F16;
  cfg.num_blocks = 32;
  cfg.block_stride = 4 * 2 * 16 * 2; /* chunk = B*H*D*e = 256 bytes */
  cfg.kv_stride = cfg.block_stride * cfg.num_blocks;
  cfg.layer_stride = 2 * cfg.kv_stride;
  cfg.flags = KV_PLAN_ONLY;
  cfg.staging_bytes = 16 * 4 * 256; /* 16 slots of 2L chunks */
  CHECK(kv_pool_create(&cfg, &p) == KV_OK && p != NULL);
  CHECK(kv_slot_bytes(p) == 4 * 256);

  {
    const uint64_t ids[2] = {7, 8};
    const int32_t off[3] = {0, 2, 5};
    const int32_t blk[5] = {3, 9, 1, 30, 12};
    const int32_t tok[2] = {8, 10}; /* 2 full blocks; 2 full blocks and a tail */
    int32_t phys[8];
    int64_t slot[8];
    int32_t moved[2] = {-1, -1};
    int64_t wrote = -1, pending = -1, used = -1;
    int32_t staged = -1, wm = -1, swapped = -1;

    CHECK(kv_swap_out(p, 1, ids, off, blk, tok, NULL) == KV_OK);
    CHECK(kv_last_plan(p, phys, slot, 8) == 2 && phys[0] == 3 && phys[1] == 9 && slot[0] == 0 && slot[1] == 1);
    CHECK(kv_swap_out(p, 1, ids, off, blk, tok, NULL) == KV_EEXIST);
    CHECK(kv_swap_out_delta(p, 1, ids + 1, off + 1, blk, tok + 1, 1, 0, moved, NULL) == KV_OK && moved[0] == 1);
    CHECK(kv_wq_post(p, 1, ids + 1, off + 1, blk, tok + 1, NULL) == KV_OK);
    CHECK(kv_wq_drain(p, 0.0, 0, KV_DELTA_INCLUDE_TAIL, &wrote, &pending, &used, NULL) == KV_OK);
    CHECK(wrote == 2 && pending == 0 && used == 0);
    CHECK(kv_req_query(p, 8, NULL, NULL, &staged, &wm, &swapped) == KV_OK && staged == 3 && wm == 2 && swapped == 0);
    {
      const int32_t roff[2] = {0, 2};
      const int32_t dst_dup[2] = {5, 5}, dst[2] = {5, 6};
      CHECK(kv_swap_in(p, 1, ids, roff, dst_dup, 0, NULL) == KV_EDUP);
      CHECK(kv_swap_in(p, 1, ids, roff, dst, 0, NULL) == KV_OK);
      CHECK(kv_req_query(p, 7, NULL, NULL, NULL, NULL, NULL) == KV_ENOENT);
    }
    {
      /* eviction and loading in one call: request 9 goes out while request 8, swapped out first, comes back into the
       * blocks request 9 gives up; the load is checked before the eviction changes anything */
      const uint64_t nine = 9, eight = 8, nobody = 77;
      const int32_t off9[2] = {0, 3}, blk9[3] = {20, 21, 22}, tok9[1] = {12};
      const int32_t off8[2] = {0, 3};
      const int32_t src[2] = {4, 4}, dst[2] = {10, 11}, dst_bad[2] = {10, 4};
      CHECK(kv_swap_out(p, 1, ids + 1, off + 1, blk, tok + 1, NULL) == KV_OK);
      CHECK(kv_evict_and_load(p, 1, &nine, off9, blk9, tok9, 1, &nobody, off8, blk9, 0, NULL) == KV_ENOENT);
      CHECK(kv_req_query(p, 9, NULL, NULL, NULL, NULL, NULL) == KV_ENOENT);
      CHECK(kv_evict_and_load(p, 1, &nine, off9, blk9, tok9, 1, &nine, off9, blk9, 0, NULL) == KV_EINVAL);
      CHECK(kv_evict_and_load(p, 1, &nine, off9, blk9, tok9, 1, &eight, off8, blk9, KV_KEEP_STAGING, NULL) == KV_OK);
      CHECK(kv_last_plan(p, phys, slot, 8) == 3 && phys[0] == 20 && phys[2] == 22);
      CHECK(kv_req_query(p, 9, NULL, NULL, &staged, &wm, &swapped) == KV_OK && staged == 3 && swapped == 1);
      CHECK(kv_req_query(p, 8, NULL, NULL, &staged, &wm, &swapped) == KV_OK && staged == 3 && swapped == 0);
      /* the move for callers that cannot allocate: same checks as kv_move_blocks, and a limit of its own */
      CHECK(kv_move_blocks_noalloc(p, 2, src, dst, NULL) == KV_OK);
      CHECK(kv_move_blocks_noalloc(p, 2, src, dst_bad, NULL) == KV_EDUP);
      CHECK(kv_move_blocks_noalloc(p, (int64_t)KV_NOALLOC_MAX_BLOCKS + 1, src, dst, NULL) == KV_E2BIG);
      CHECK(kv_move_blocks(p, 2, src, dst_bad, NULL) == KV_EDUP);
    }
    CHECK(kv_sync(p) == KV_OK);
    CHECK(strcmp(kv_strerror(KV_ENOSPC), "staging arena full") == 0);
  }

  {
    kv_sched_config sc;
    kv_sched_req rq[2];
    kv_sched_out out[2];
    int32_t mode = -1;
    double w = 0.0;
    memset(&sc, 0, sizeof(sc));
    memset(rq, 0, sizeof(rq));
    sc.struct_size = sizeof(sc);
    sc.mem_blocks = 1;
    sc.ws_blocks = 100;
    sc.max_running = 1;
    sc.interval = 1.0;
    sc.gen_rate = 40.0;
    sc.capacity = 1e9;
    sc.gamma = 1.0;
    sc.safety = 1.0;
    sc.t_critical = 1.0;
    sc.weight_tau = 1e9;
    sc.evict_gbps = sc.load_gbps = 50.0;
    sc.block_bytes = 1024.0;
    rq[0].state = KVS_RUNNING; rq[0].rate = 20.0; rq[0].buffer = 80.0; rq[0].blocks = 1; rq[0].tokens = 16;
    rq[1].state = KVS_PREEMPTED; rq[1].rate = 20.0; rq[1].buffer = 2.0; rq[1].blocks = 1; rq[1].tokens = 16;
    CHECK(kv_sched_step(&sc, 2, rq, out, &mode) == KVS_OK);
    CHECK(mode == KVS_MODE_BUFFER_AWARE && out[0].decision == KVS_PREEMPT && out[1].decision == KVS_RUN);
    CHECK(kv_metric_token_weight(15.0, 10.0, 0.1) > 0.49 && kv_metric_token_weight(15.0, 10.0, 0.1) < 0.51);
    {
      const int32_t buf[4] = {0, 0, 12, 30};
      CHECK(kv_metric_weight_sum(4, buf, 10.0, 0.1, &w) == KVS_OK && w > 2.79 && w < 2.81);
    }
  }
  CHECK(kv_pool_destroy(p) == KV_OK);
  puts("C ABI ok");
  return 0;
}
