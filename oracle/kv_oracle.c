/*
 * kv_oracle.c — TEST INFRASTRUCTURE ONLY (see kv_oracle.h).
 *
 * Every operation runs in two phases.  Phase 1 works on a private copy of the
 * bookkeeping (request table + slot occupancy), checks every argument and
 * writes down the list of (physical block, staging slot) pairs to move.  If
 * anything is wrong the copy is thrown away and nothing has changed.  Phase 2
 * installs the copy and moves the bytes, one byte at a time, pair by pair in
 * list order.
 */
#include "kv_oracle.h"

#include <stdlib.h>
#include <string.h>

typedef struct {
  uint64_t id;
  int64_t base;
  int32_t cap, staged, wm, swapped;
} entry;

typedef struct {
  entry* e;
  int32_t n;
  uint8_t* used; /* one byte per staging slot: 1 = inside some extent */
  int64_t slots;
} book;

struct ora_state {
  ora_config c;
  int64_t chunk, block_bytes, scale_chunk, block_scale_bytes, S;
  book bk;
};

typedef struct {
  int64_t* phys;
  int64_t* slot;
  int64_t n, cap;
} moves;

/* ---------------------------------------------------------------- helpers */

static int book_clone(const book* a, book* b) {
  b->n = a->n;
  b->slots = a->slots;
  b->e = (entry*)malloc(sizeof(entry) * (size_t)(a->n + 1));
  b->used = (uint8_t*)malloc((size_t)(a->slots + 1));
  if (!b->e || !b->used) return -1;
  for (int32_t i = 0; i < a->n; i++) b->e[i] = a->e[i];
  for (int64_t i = 0; i < a->slots; i++) b->used[i] = a->used[i];
  return 0;
}

static void book_free(book* b) {
  free(b->e);
  free(b->used);
  b->e = NULL;
  b->used = NULL;
}

static int32_t book_find(const book* b, uint64_t id) {
  for (int32_t i = 0; i < b->n; i++)
    if (b->e[i].id == id) return i;
  return -1;
}

static int32_t book_add(book* b, uint64_t id) {
  entry* ne = (entry*)realloc(b->e, sizeof(entry) * (size_t)(b->n + 1));
  if (!ne) return -1;
  b->e = ne;
  entry z = {id, 0, 0, 0, 0, 0};
  b->e[b->n] = z;
  return b->n++;
}

static void book_remove(book* b, int32_t i) {
  for (int64_t k = 0; k < b->e[i].cap; k++) b->used[b->e[i].base + k] = 0;
  for (int32_t k = i; k + 1 < b->n; k++) b->e[k] = b->e[k + 1];
  b->n--;
}

/* lowest start index of a run of `want` free slots, or -1 */
static int64_t first_fit(const book* b, int64_t want) {
  if (want == 0) return 0;
  for (int64_t s = 0; s + want <= b->slots; s++) {
    int64_t k = 0;
    while (k < want && !b->used[s + k]) k++;
    if (k == want) return s;
  }
  return -1;
}

/* make entry i able to hold `need` blocks; 0 or ORA_ENOSPC */
static int ensure_cap(book* b, int32_t i, int64_t need) {
  entry* e = &b->e[i];
  if (need <= e->cap) return ORA_OK;
  if (e->cap == 0) {
    int64_t s = first_fit(b, need);
    if (s < 0) return ORA_ENOSPC;
    e->base = s;
  } else {
    if (e->base + need > b->slots) return ORA_ENOSPC;
    for (int64_t k = e->cap; k < need; k++)
      if (b->used[e->base + k]) return ORA_ENOSPC;
  }
  for (int64_t k = e->cap; k < need; k++) b->used[e->base + k] = 1;
  e->cap = (int32_t)need;
  return ORA_OK;
}

static int moves_push(moves* m, int64_t phys, int64_t slot) {
  if (m->n == m->cap) {
    int64_t nc = m->cap ? m->cap * 2 : 64;
    int64_t* a = (int64_t*)realloc(m->phys, sizeof(int64_t) * (size_t)nc);
    if (!a) return -1;
    m->phys = a;
    int64_t* c = (int64_t*)realloc(m->slot, sizeof(int64_t) * (size_t)nc);
    if (!c) return -1;
    m->slot = c;
    m->cap = nc;
  }
  m->phys[m->n] = phys;
  m->slot[m->n] = slot;
  m->n++;
  return 0;
}

static void moves_free(moves* m) {
  free(m->phys);
  free(m->slot);
}

/* CSR and id checks shared by the three request-level operations */
static int check_call(const ora_state* s, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                      const int32_t* block_ids) {
  if (!s || n < 0) return ORA_EINVAL;
  if (n == 0) return ORA_OK;
  if (!req_ids || !offsets) return ORA_EINVAL;
  if (offsets[0] < 0) return ORA_EINVAL;
  for (int32_t i = 0; i < n; i++)
    if (offsets[i + 1] < offsets[i]) return ORA_EINVAL;
  if (offsets[n] > offsets[0] && !block_ids) return ORA_EINVAL;
  for (int32_t i = 0; i < n; i++)
    for (int32_t k = 0; k < i; k++)
      if (req_ids[i] == req_ids[k]) return ORA_EINVAL;
  for (int32_t k = offsets[0]; k < offsets[n]; k++)
    if (block_ids[k] < 0 || (int64_t)block_ids[k] >= s->c.N) return ORA_ERANGE;
  return ORA_OK;
}

/* ------------------------------------------------------- the byte movement */

static void block_to_slot(const ora_state* s, int64_t phys, int64_t slot) {
  const ora_config* c = &s->c;
  for (int32_t l = 0; l < c->L; l++)
    for (int32_t kv = 0; kv < 2; kv++) {
      const uint8_t* src = c->pool + l * c->layer_stride + kv * c->kv_stride + phys * c->block_stride;
      uint8_t* dst = c->staging + slot * s->S + (2 * l + kv) * s->chunk;
      for (int64_t b = 0; b < s->chunk; b++) dst[b] = src[b];
      if (c->scale) {
        const uint8_t* ss = c->scale + l * c->s_layer_stride + kv * c->s_kv_stride + phys * c->s_block_stride;
        uint8_t* sd = c->staging + slot * s->S + s->block_bytes + (2 * l + kv) * s->scale_chunk;
        for (int64_t b = 0; b < s->scale_chunk; b++) sd[b] = ss[b];
      }
    }
}

static void slot_to_block(const ora_state* s, int64_t slot, int64_t phys) {
  const ora_config* c = &s->c;
  for (int32_t l = 0; l < c->L; l++)
    for (int32_t kv = 0; kv < 2; kv++) {
      uint8_t* dst = c->pool + l * c->layer_stride + kv * c->kv_stride + phys * c->block_stride;
      const uint8_t* src = c->staging + slot * s->S + (2 * l + kv) * s->chunk;
      for (int64_t b = 0; b < s->chunk; b++) dst[b] = src[b];
      if (c->scale) {
        uint8_t* sd = c->scale + l * c->s_layer_stride + kv * c->s_kv_stride + phys * c->s_block_stride;
        const uint8_t* ss = c->staging + slot * s->S + s->block_bytes + (2 * l + kv) * s->scale_chunk;
        for (int64_t b = 0; b < s->scale_chunk; b++) sd[b] = ss[b];
      }
    }
}

static void block_to_block(const ora_state* s, int64_t from, int64_t to) {
  const ora_config* c = &s->c;
  for (int32_t l = 0; l < c->L; l++)
    for (int32_t kv = 0; kv < 2; kv++) {
      const uint8_t* src = c->pool + l * c->layer_stride + kv * c->kv_stride + from * c->block_stride;
      uint8_t* dst = c->pool + l * c->layer_stride + kv * c->kv_stride + to * c->block_stride;
      for (int64_t b = 0; b < s->chunk; b++) dst[b] = src[b];
      if (c->scale) {
        const uint8_t* ss = c->scale + l * c->s_layer_stride + kv * c->s_kv_stride + from * c->s_block_stride;
        uint8_t* sd = c->scale + l * c->s_layer_stride + kv * c->s_kv_stride + to * c->s_block_stride;
        for (int64_t b = 0; b < s->scale_chunk; b++) sd[b] = ss[b];
      }
    }
}

/* ------------------------------------------------------------- lifecycle */

ora_state* ora_create(const ora_config* cfg) {
  if (!cfg || cfg->L <= 0 || cfg->H <= 0 || cfg->D <= 0 || cfg->B <= 0 || cfg->elem_bytes <= 0 ||
      cfg->N <= 0 || !cfg->pool || !cfg->staging || cfg->staging_bytes < 0)
    return NULL;
  ora_state* s = (ora_state*)calloc(1, sizeof(ora_state));
  if (!s) return NULL;
  s->c = *cfg;
  s->chunk = (int64_t)cfg->B * cfg->H * cfg->D * cfg->elem_bytes;
  s->block_bytes = 2 * (int64_t)cfg->L * s->chunk;
  s->scale_chunk = cfg->scale ? (int64_t)cfg->H * 4 : 0;
  s->block_scale_bytes = 2 * (int64_t)cfg->L * s->scale_chunk;
  s->S = s->block_bytes + s->block_scale_bytes;
  s->bk.slots = cfg->staging_bytes / s->S;
  s->bk.n = 0;
  s->bk.e = NULL;
  s->bk.used = (uint8_t*)calloc((size_t)(s->bk.slots + 1), 1);
  if (!s->bk.used) {
    free(s);
    return NULL;
  }
  return s;
}

void ora_destroy(ora_state* s) {
  if (!s) return;
  book_free(&s->bk);
  free(s);
}

int64_t ora_slot_bytes(const ora_state* s) { return s->S; }

/* ------------------------------------------------- preempt: full swap-out
 * Section 5 (a): the whole KV cache of each listed request goes to the host. */
int ora_swap_out(ora_state* s, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                 const int32_t* block_ids, const int32_t* num_tokens) {
  int rc = check_call(s, n, req_ids, offsets, block_ids);
  if (rc) return rc;
  if (n == 0) return ORA_OK;
  if (!num_tokens) return ORA_EINVAL;
  book nb;
  if (book_clone(&s->bk, &nb)) return ORA_EINVAL;
  moves mv = {0, 0, 0, 0};
  const int64_t B = s->c.B;
  for (int32_t i = 0; i < n && !rc; i++) {
    int64_t len = num_tokens[i];
    int64_t row = offsets[i + 1] - offsets[i];
    if (len < 0 || row != (len + B - 1) / B) { rc = ORA_EINVAL; break; }
    int32_t k = book_find(&nb, req_ids[i]);
    if (k >= 0 && nb.e[k].swapped) { rc = ORA_EEXIST; break; }
    if (k < 0) k = book_add(&nb, req_ids[i]);
    if (k < 0) { rc = ORA_EINVAL; break; }
    rc = ensure_cap(&nb, k, row);
    if (rc) break;
    for (int64_t j = 0; j < row; j++)
      if (moves_push(&mv, block_ids[offsets[i] + j], nb.e[k].base + j)) { rc = ORA_EINVAL; break; }
    nb.e[k].staged = (int32_t)row;
    nb.e[k].wm = (int32_t)(len / B);
    nb.e[k].swapped = 1;
  }
  if (rc) {
    book_free(&nb);
    moves_free(&mv);
    return rc;
  }
  book_free(&s->bk);
  s->bk = nb;
  for (int64_t m = 0; m < mv.n; m++) block_to_slot(s, mv.phys[m], mv.slot[m]);
  moves_free(&mv);
  return ORA_OK;
}

/* ------------------------------------------ write-through: delta swap-out
 * Section 5.1: only blocks completed since the previous offload are written;
 * Section 5.2: writes are sized (block budget) and served in caller order. */
int ora_swap_out_delta(ora_state* s, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                       const int32_t* block_ids, const int32_t* num_tokens, int64_t block_budget,
                       uint32_t flags, int32_t* blocks_moved) {
  int rc = check_call(s, n, req_ids, offsets, block_ids);
  if (rc) return rc;
  if (block_budget < 0) return ORA_EINVAL;
  if (n == 0) return ORA_OK;
  if (!num_tokens) return ORA_EINVAL;
  book nb;
  if (book_clone(&s->bk, &nb)) return ORA_EINVAL;
  moves mv = {0, 0, 0, 0};
  int32_t* moved = (int32_t*)calloc((size_t)n, sizeof(int32_t));
  const int64_t B = s->c.B;
  int unlimited = (block_budget == 0);
  int64_t left = block_budget;
  for (int32_t i = 0; i < n && !rc; i++) {
    int64_t len = num_tokens[i];
    int64_t row = offsets[i + 1] - offsets[i];
    if (len < 0 || row < (len + B - 1) / B) { rc = ORA_EINVAL; break; }
    int32_t k = book_find(&nb, req_ids[i]);
    if (k >= 0 && nb.e[k].swapped) { rc = ORA_EEXIST; break; }
    if (k < 0) k = book_add(&nb, req_ids[i]);
    if (k < 0) { rc = ORA_EINVAL; break; }
    if (len < (int64_t)nb.e[k].wm * B) { rc = ORA_ESTATE; break; }
    rc = ensure_cap(&nb, k, row);
    if (rc) break;
    int64_t full = len / B;
    int64_t hi = (flags & ORA_DELTA_INCLUDE_TAIL) ? (len + B - 1) / B : full;
    int64_t wm = nb.e[k].wm;
    int64_t m = wm;
    if (hi > wm) {
      m = hi;
      if (!unlimited && m > wm + left) m = wm + left;
    }
    for (int64_t j = wm; j < m; j++)
      if (moves_push(&mv, block_ids[offsets[i] + j], nb.e[k].base + j)) { rc = ORA_EINVAL; break; }
    if (!unlimited) left -= (m - wm);
    moved[i] = (int32_t)(m - wm);
    if (m > nb.e[k].staged) nb.e[k].staged = (int32_t)m;
    nb.e[k].wm = (int32_t)(m < full ? m : full);
  }
  if (rc) {
    book_free(&nb);
    moves_free(&mv);
    free(moved);
    return rc;
  }
  book_free(&s->bk);
  s->bk = nb;
  for (int64_t m = 0; m < mv.n; m++) block_to_slot(s, mv.phys[m], mv.slot[m]);
  if (blocks_moved)
    for (int32_t i = 0; i < n; i++) blocks_moved[i] = moved[i];
  moves_free(&mv);
  free(moved);
  return ORA_OK;
}

/* ------------------------------------------------------- resume: swap-in
 * Section 5 (b): the staged copy goes back into freshly allocated blocks. */
int ora_swap_in(ora_state* s, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                const int32_t* new_block_ids, uint32_t flags) {
  int rc = check_call(s, n, req_ids, offsets, new_block_ids);
  if (rc) return rc;
  if (n == 0) return ORA_OK;
  book nb;
  if (book_clone(&s->bk, &nb)) return ORA_EINVAL;
  moves mv = {0, 0, 0, 0};
  for (int32_t i = 0; i < n && !rc; i++) {
    int32_t k = book_find(&nb, req_ids[i]);
    if (k < 0) { rc = ORA_ENOENT; break; }
    int64_t row = offsets[i + 1] - offsets[i];
    if (row != nb.e[k].staged) { rc = ORA_EINVAL; break; }
    for (int64_t j = 0; j < row; j++)
      if (moves_push(&mv, new_block_ids[offsets[i] + j], nb.e[k].base + j)) { rc = ORA_EINVAL; break; }
    if (flags & ORA_KEEP_STAGING)
      nb.e[k].swapped = 0;
    else
      book_remove(&nb, k);
  }
  /* destinations are freshly allocated blocks: no id may appear twice */
  for (int64_t a = 0; a < mv.n && !rc; a++)
    for (int64_t b = 0; b < a; b++)
      if (mv.phys[a] == mv.phys[b]) { rc = ORA_EDUP; break; }
  if (rc) {
    book_free(&nb);
    moves_free(&mv);
    return rc;
  }
  book_free(&s->bk);
  s->bk = nb;
  for (int64_t m = 0; m < mv.n; m++) slot_to_block(s, mv.slot[m], mv.phys[m]);
  moves_free(&mv);
  return ORA_OK;
}

/* ------------------------------------------- on-device move, pool to pool */
int ora_move_blocks(ora_state* s, int64_t n, const int32_t* src_ids, const int32_t* dst_ids) {
  if (!s || n < 0) return ORA_EINVAL;
  if (n == 0) return ORA_OK;
  if (!src_ids || !dst_ids) return ORA_EINVAL;
  for (int64_t i = 0; i < n; i++)
    if (src_ids[i] < 0 || src_ids[i] >= s->c.N || dst_ids[i] < 0 || dst_ids[i] >= s->c.N) return ORA_ERANGE;
  for (int64_t a = 0; a < n; a++) {
    for (int64_t b = 0; b < a; b++)
      if (dst_ids[a] == dst_ids[b]) return ORA_EDUP;
    for (int64_t b = 0; b < n; b++)
      if (dst_ids[a] == src_ids[b]) return ORA_EDUP;
  }
  for (int64_t i = 0; i < n; i++) block_to_block(s, src_ids[i], dst_ids[i]);
  return ORA_OK;
}

/* ----------------------------------------------------------- bookkeeping */

int ora_req_reserve(ora_state* s, uint64_t req_id, int32_t max_blocks) {
  if (!s || max_blocks < 0) return ORA_EINVAL;
  if (book_find(&s->bk, req_id) >= 0) return ORA_EEXIST;
  int64_t at = first_fit(&s->bk, max_blocks);
  if (at < 0) return ORA_ENOSPC;
  int32_t k = book_add(&s->bk, req_id);
  if (k < 0) return ORA_EINVAL;
  s->bk.e[k].base = at;
  s->bk.e[k].cap = max_blocks;
  for (int64_t j = 0; j < max_blocks; j++) s->bk.used[at + j] = 1;
  return ORA_OK;
}

int ora_req_release(ora_state* s, uint64_t req_id) {
  if (!s) return ORA_EINVAL;
  int32_t k = book_find(&s->bk, req_id);
  if (k < 0) return ORA_ENOENT;
  book_remove(&s->bk, k);
  return ORA_OK;
}

int ora_req_query(const ora_state* s, uint64_t req_id, int64_t* staging_offset, int32_t* cap_blocks,
                  int32_t* blocks_staged, int32_t* watermark, int32_t* swapped) {
  if (!s) return ORA_EINVAL;
  int32_t k = book_find(&s->bk, req_id);
  if (k < 0) return ORA_ENOENT;
  if (staging_offset) *staging_offset = s->bk.e[k].base * s->S;
  if (cap_blocks) *cap_blocks = s->bk.e[k].cap;
  if (blocks_staged) *blocks_staged = s->bk.e[k].staged;
  if (watermark) *watermark = s->bk.e[k].wm;
  if (swapped) *swapped = s->bk.e[k].swapped;
  return ORA_OK;
}
