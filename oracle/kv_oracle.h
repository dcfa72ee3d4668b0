/*
 * kv_oracle.h — TEST INFRASTRUCTURE ONLY.
 *
 * A plain, single-threaded, byte-by-byte CPU statement of what the paged
 * KV-cache swap computes: preempt / resume (paper Section 5, operations (a)
 * and (b)) and the incremental write-through of Section 5.1, over host arrays.
 * It exists so that tests, the smoke check and the benchmark's CPU baseline
 * can compare the GPU library against something that is obviously right.
 * It shares no code, header or table with the GPU library and must never be
 * called from the product path.
 *
 * Parity status: pinned.  tests/test_oracle_pins.py checks every function here
 * against things fixed outside of it: closed-form staging offsets over an
 * address-coded pool, round-trip identity, untouched complement, delta == full,
 * an element-level dictionary model under brute force on tiny pools, and the
 * block-major special case that reduces to one memcpy.
 *
 * Geometry and layout (the readings adopted where the paper is silent):
 *   chunk = B*H*D*e bytes, contiguous in the pool:
 *     pool  + l*layer_stride + c*kv_stride + p*block_stride      (c: 0 K, 1 V)
 *   scales (optional), H 32-bit words per (l, c, p):
 *     scale + l*s_layer_stride + c*s_kv_stride + p*s_block_stride
 *   staging arena = slots of S = 2*L*chunk + (scales ? 2*L*H*4 : 0) bytes.
 *   Logical block j of a request with extent base: slot base+j;
 *     data (l,c)   at slot*S + (2*l+c)*chunk
 *     scales (l,c) at slot*S + 2*L*chunk + (2*l+c)*H*4
 *   Extents are placed first-fit at the lowest free slot.
 *
 * Status codes carry the same numbers as the GPU library's so that tests can
 * compare them directly: the numbers are an interface, typed out separately
 * on each side.
 */
#ifndef KV_ORACLE_H
#define KV_ORACLE_H

#include <stdint.h>

enum {
  ORA_OK = 0,
  ORA_EINVAL = -1,
  ORA_ERANGE = -2,
  ORA_EDUP = -3,
  ORA_ENOENT = -4,
  ORA_EEXIST = -5,
  ORA_ENOSPC = -6,
  ORA_ESTATE = -8
};

enum { ORA_DELTA_INCLUDE_TAIL = 1u };
enum { ORA_KEEP_STAGING = 1u };

typedef struct {
  int32_t L, H, D, B, elem_bytes;
  int64_t N;
  uint8_t* pool;
  int64_t layer_stride, kv_stride, block_stride;
  uint8_t* scale; /* NULL: no scales */
  int64_t s_layer_stride, s_kv_stride, s_block_stride;
  uint8_t* staging;
  int64_t staging_bytes;
} ora_config;

typedef struct ora_state ora_state;

ora_state* ora_create(const ora_config* cfg);
void ora_destroy(ora_state* s);
int64_t ora_slot_bytes(const ora_state* s);

int ora_swap_out(ora_state* s, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                 const int32_t* block_ids, const int32_t* num_tokens);
int ora_swap_out_delta(ora_state* s, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                       const int32_t* block_ids, const int32_t* num_tokens, int64_t block_budget,
                       uint32_t flags, int32_t* blocks_moved);
int ora_swap_in(ora_state* s, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                const int32_t* new_block_ids, uint32_t flags);
int ora_move_blocks(ora_state* s, int64_t n, const int32_t* src_ids, const int32_t* dst_ids);

int ora_req_reserve(ora_state* s, uint64_t req_id, int32_t max_blocks);
int ora_req_release(ora_state* s, uint64_t req_id);
int ora_req_query(const ora_state* s, uint64_t req_id, int64_t* staging_offset, int32_t* cap_blocks,
                  int32_t* blocks_staged, int32_t* watermark, int32_t* swapped);

#endif
