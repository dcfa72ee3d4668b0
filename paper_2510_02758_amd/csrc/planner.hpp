// Host-side planner of the paged KV swap: request table, staging-extent
// allocator, argument validation and descriptor building.  Pure C++ (no HIP):
// the same code runs under KV_PLAN_ONLY on machines without a GPU.
//
// The paper keeps this state in its Request Offload Manager and Hierarchical
// KV Cache Manager (Section 3.1): which requests have host copies, how much of
// each has been written through (Section 5.1), and write / load queues of
// chunks.  Here a "queue" is the descriptor list one call produces: one
// (physical block, staging slot) pair per block to move, in launch order.
#pragma once

#include <algorithm>
#include <cstdint>
#include <map>
#include <unordered_map>
#include <vector>

#include "../../include/kvswap.h"

namespace kvswap {

struct Desc {
  int32_t a;  // gather/scatter: physical block;      move: source block
  int32_t b;  // gather/scatter: contiguous-side slot; move: destination block
};

// Free slots of the staging arena as disjoint, coalesced [start, start+len) runs.
// Placement is first fit at the lowest start, so it depends on the call history only.
class ExtentAlloc {
 public:
  void reset(int64_t slots) {
    free_.clear();
    slots_ = slots;
    if (slots > 0) free_[0] = slots;
  }
  int64_t slots() const { return slots_; }
  // lowest start of a free run of n slots, or -1.  n == 0 always yields 0.
  int64_t alloc(int64_t n) {
    if (n == 0) return 0;
    for (auto it = free_.begin(); it != free_.end(); ++it) {
      if (it->second >= n) {
        int64_t s = it->first, len = it->second;
        free_.erase(it);
        if (len > n) free_[s + n] = len - n;
        return s;
      }
    }
    return -1;
  }
  // take [at, at+n) if it is entirely free
  bool take(int64_t at, int64_t n) {
    if (n == 0) return true;
    auto it = free_.upper_bound(at);
    if (it == free_.begin()) return false;
    --it;
    int64_t s = it->first, len = it->second;
    if (at < s || at + n > s + len) return false;
    free_.erase(it);
    if (at > s) free_[s] = at - s;
    if (at + n < s + len) free_[at + n] = s + len - (at + n);
    return true;
  }
  void release(int64_t at, int64_t n) {
    if (n == 0) return;
    auto nx = free_.lower_bound(at);
    if (nx != free_.begin()) {
      auto pv = std::prev(nx);
      if (pv->first + pv->second == at) {
        at = pv->first;
        n += pv->second;
        free_.erase(pv);
      }
    }
    if (nx != free_.end() && at + n == nx->first) {
      n += nx->second;
      free_.erase(nx);
    }
    free_[at] = n;
  }

 private:
  std::map<int64_t, int64_t> free_;
  int64_t slots_ = 0;
};

struct Req {
  int64_t base = 0;
  int32_t cap = 0, staged = 0, wm = 0;
  bool swapped = false;
  uint64_t out_seq = 0;  // last evict-stream call that wrote this request's slots
  uint64_t in_seq = 0;   // last load-stream call that read this request's slots
};

// What a planning pass hands to the executor.
struct Plan {
  std::vector<Desc> desc;                           // (phys, staging slot) in launch order
  std::vector<std::pair<int64_t, int64_t>> fresh;   // slot runs newly taken from the arena
  std::vector<uint64_t> fresh_ids;                  // the request each of those runs went to
  std::vector<std::pair<int64_t, int64_t>> freed;   // slot runs given back (swap-in without keep)
  std::vector<uint64_t> touched;                    // request ids whose slots the call reads/writes
  std::vector<std::pair<uint64_t, size_t>> req_end; // (request id, end of its descriptors in `desc`), call order
  uint64_t wait_out_seq = 0;                        // newest earlier call the plan's slots depend on
  uint64_t wait_in_seq = 0;
};

class Planner {
 public:
  void init(int64_t num_blocks, int32_t block_size, int64_t slots) {
    N_ = num_blocks;
    B_ = block_size;
    alloc_.reset(slots);
    reqs_.clear();
  }

  int reserve(uint64_t id, int32_t max_blocks) {
    if (max_blocks < 0) return KV_EINVAL;
    if (reqs_.count(id)) return KV_EEXIST;
    int64_t at = alloc_.alloc(max_blocks);
    if (at < 0) return KV_ENOSPC;
    Req r;
    r.base = at;
    r.cap = max_blocks;
    reqs_[id] = r;
    last_fresh_ = {at, (int64_t)max_blocks};
    return KV_OK;
  }
  std::pair<int64_t, int64_t> last_fresh() const { return last_fresh_; }

  int release(uint64_t id, Req* was = nullptr) {
    auto it = reqs_.find(id);
    if (it == reqs_.end()) return KV_ENOENT;
    if (was) *was = it->second;
    alloc_.release(it->second.base, it->second.cap);
    reqs_.erase(it);
    return KV_OK;
  }

  const Req* find(uint64_t id) const {
    auto it = reqs_.find(id);
    return it == reqs_.end() ? nullptr : &it->second;
  }
  Req* find_mut(uint64_t id) {
    auto it = reqs_.find(id);
    return it == reqs_.end() ? nullptr : &it->second;
  }

  // Full swap-out (Section 5, preempt).  On error nothing has changed.
  int plan_swap_out(int32_t n, const uint64_t* ids, const int32_t* off, const int32_t* blk,
                    const int32_t* ntok, Plan* out) {
    int rc = check_call(n, ids, off, blk);
    if (rc || n == 0) return rc;
    if (!ntok) return KV_EINVAL;
    begin();
    for (int32_t i = 0; i < n && !rc; i++) {
      int64_t len = ntok[i], row = (int64_t)off[i + 1] - off[i];
      if (len < 0 || row != (len + B_ - 1) / B_) { rc = KV_EINVAL; break; }
      Req* r = touch(ids[i]);
      if (r->swapped) { rc = KV_EEXIST; break; }
      rc = ensure_cap(ids[i], r, row, out);
      if (rc) break;
      for (int64_t j = 0; j < row; j++) out->desc.push_back({blk[off[i] + j], (int32_t)(r->base + j)});
      if (row) out->req_end.push_back({ids[i], out->desc.size()});
      r->staged = (int32_t)row;
      r->wm = (int32_t)(len / B_);
      r->swapped = true;
      out->wait_in_seq = std::max(out->wait_in_seq, r->in_seq);
      out->touched.push_back(ids[i]);
    }
    if (rc) rollback(out);
    return rc;
  }

  // Incremental write-through (Section 5.1), sized and ordered (Section 5.2).
  // limited_even_if_zero: a budget of 0 then means "move nothing" instead of "unlimited".
  int plan_delta(int32_t n, const uint64_t* ids, const int32_t* off, const int32_t* blk, const int32_t* ntok,
                 int64_t budget, uint32_t flags, int32_t* moved, Plan* out, bool limited_even_if_zero = false) {
    int rc = check_call(n, ids, off, blk);
    if (rc) return rc;
    if (budget < 0) return KV_EINVAL;
    if (n == 0) return KV_OK;
    if (!ntok) return KV_EINVAL;
    begin();
    moved_.assign((size_t)n, 0);
    const bool unlimited = budget == 0 && !limited_even_if_zero;
    int64_t left = budget;
    for (int32_t i = 0; i < n && !rc; i++) {
      int64_t len = ntok[i], row = (int64_t)off[i + 1] - off[i];
      if (len < 0 || row < (len + B_ - 1) / B_) { rc = KV_EINVAL; break; }
      Req* r = touch(ids[i]);
      if (r->swapped) { rc = KV_EEXIST; break; }
      if (len < (int64_t)r->wm * B_) { rc = KV_ESTATE; break; }
      rc = ensure_cap(ids[i], r, row, out);
      if (rc) break;
      const int64_t full = len / B_;
      const int64_t hi = (flags & KV_DELTA_INCLUDE_TAIL) ? (len + B_ - 1) / B_ : full;
      const int64_t wm = r->wm;
      int64_t m = wm;
      if (hi > wm) m = unlimited ? hi : std::min(hi, wm + left);
      for (int64_t j = wm; j < m; j++) out->desc.push_back({blk[off[i] + j], (int32_t)(r->base + j)});
      if (!unlimited) left -= m - wm;
      moved_[(size_t)i] = (int32_t)(m - wm);
      r->staged = std::max<int32_t>(r->staged, (int32_t)m);
      r->wm = (int32_t)std::min(m, full);
      if (m > wm) {
        out->wait_in_seq = std::max(out->wait_in_seq, r->in_seq);
        out->touched.push_back(ids[i]);
        out->req_end.push_back({ids[i], out->desc.size()});
      }
    }
    if (rc) {
      rollback(out);
      return rc;
    }
    if (moved) std::copy(moved_.begin(), moved_.end(), moved);
    return KV_OK;
  }

  // Swap-in (Section 5, resume).  Extents are released here unless `keep`.
  // Everything plan_swap_in checks, without changing anything.
  int check_swap_in(int32_t n, const uint64_t* ids, const int32_t* off, const int32_t* blk) {
    int rc = check_call(n, ids, off, blk);
    if (rc || n == 0) return rc;
    for (int32_t i = 0; i < n; i++) {
      const Req* r = find(ids[i]);
      if (!r) return KV_ENOENT;
      if ((int64_t)off[i + 1] - off[i] != r->staged) return KV_EINVAL;
    }
    if (has_duplicates(blk + off[0], (int64_t)off[n] - off[0])) return KV_EDUP;
    return KV_OK;
  }

  int plan_swap_in(int32_t n, const uint64_t* ids, const int32_t* off, const int32_t* blk, uint32_t flags,
                   Plan* out) {
    int rc = check_swap_in(n, ids, off, blk);
    if (rc || n == 0) return rc;
    for (int32_t i = 0; i < n; i++) {
      Req* r = find_mut(ids[i]);
      for (int64_t j = 0; j < r->staged; j++) out->desc.push_back({blk[off[i] + j], (int32_t)(r->base + j)});
      if (r->staged) out->req_end.push_back({ids[i], out->desc.size()});
      out->wait_out_seq = std::max(out->wait_out_seq, r->out_seq);
      if (flags & KV_KEEP_STAGING) {
        r->swapped = false;
        out->touched.push_back(ids[i]);
      } else {
        if (r->cap) out->freed.push_back({r->base, r->cap});
        alloc_.release(r->base, r->cap);
        reqs_.erase(ids[i]);
      }
    }
    return KV_OK;
  }

  int plan_move(int64_t n, const int32_t* src, const int32_t* dst, Plan* out) {
    if (n < 0) return KV_EINVAL;
    if (n == 0) return KV_OK;
    if (!src || !dst) return KV_EINVAL;
    for (int64_t i = 0; i < n; i++)
      if (src[i] < 0 || src[i] >= N_ || dst[i] < 0 || dst[i] >= N_) return KV_ERANGE;
    if (has_duplicates(dst, n)) return KV_EDUP;
    if (sparse(n)) {  // a destination that is also a source: merge of the two sorted lists
      sorted_.assign(dst, dst + n);  // has_duplicates left `sorted_` = sorted dst, but be explicit
      std::sort(sorted_.begin(), sorted_.end());
      sorted2_.assign(src, src + n);
      std::sort(sorted2_.begin(), sorted2_.end());
      size_t i = 0, j = 0;
      while (i < sorted_.size() && j < sorted2_.size()) {
        if (sorted_[i] == sorted2_[j]) return KV_EDUP;
        sorted_[i] < sorted2_[j] ? i++ : j++;
      }
    } else {
      mark_.assign((size_t)((N_ + 63) / 64), 0);
      for (int64_t i = 0; i < n; i++) mark_[(size_t)(src[i] >> 6)] |= 1ull << (src[i] & 63);
      for (int64_t i = 0; i < n; i++)
        if (mark_[(size_t)(dst[i] >> 6)] >> (dst[i] & 63) & 1) return KV_EDUP;
    }
    for (int64_t i = 0; i < n; i++) out->desc.push_back({src[i], dst[i]});
    return KV_OK;
  }

 private:
  int check_call(int32_t n, const uint64_t* ids, const int32_t* off, const int32_t* blk) {
    if (n < 0) return KV_EINVAL;
    if (n == 0) return KV_OK;
    if (!ids || !off || off[0] < 0) return KV_EINVAL;
    for (int32_t i = 0; i < n; i++)
      if (off[i + 1] < off[i]) return KV_EINVAL;
    if (off[n] > off[0] && !blk) return KV_EINVAL;
    seen_.clear();
    seen_.reserve((size_t)n * 2);
    for (int32_t i = 0; i < n; i++)
      if (!seen_.emplace(ids[i], 0).second) return KV_EINVAL;
    for (int64_t k = off[0]; k < off[n]; k++)
      if (blk[k] < 0 || blk[k] >= N_) return KV_ERANGE;
    return KV_OK;
  }

  // A bitmap over all N blocks costs N/64 words per call; for a list that is short against the pool (token-level
  // pools have millions of blocks) sorting the list is cheaper.
  bool sparse(int64_t n) const { return n * 512 < N_; }

  bool has_duplicates(const int32_t* ids, int64_t n) {
    if (sparse(n)) {
      sorted_.assign(ids, ids + n);
      std::sort(sorted_.begin(), sorted_.end());
      return std::adjacent_find(sorted_.begin(), sorted_.end()) != sorted_.end();
    }
    mark_.assign((size_t)((N_ + 63) / 64), 0);
    for (int64_t i = 0; i < n; i++) {
      uint64_t& w = mark_[(size_t)(ids[i] >> 6)];
      const uint64_t bit = 1ull << (ids[i] & 63);
      if (w & bit) return true;
      w |= bit;
    }
    return false;
  }

  // ---- undo log: a failed call restores table and allocator exactly ----
  struct Undo {
    uint64_t id;
    bool existed;
    Req old;
  };
  void begin() { undo_.clear(); }
  Req* touch(uint64_t id) {
    auto it = reqs_.find(id);
    if (it == reqs_.end()) {
      undo_.push_back({id, false, Req()});
      return &reqs_[id];
    }
    undo_.push_back({id, true, it->second});
    return &it->second;
  }
  int ensure_cap(uint64_t id, Req* r, int64_t need, Plan* out) {
    if (need <= r->cap) return KV_OK;
    if (r->cap == 0) {
      int64_t at = alloc_.alloc(need);
      if (at < 0) return KV_ENOSPC;
      r->base = at;
      out->fresh.push_back({at, need});
    } else {
      if (r->base + need > alloc_.slots()) return KV_ENOSPC;
      if (!alloc_.take(r->base + r->cap, need - r->cap)) return KV_ENOSPC;
      out->fresh.push_back({r->base + r->cap, need - r->cap});
    }
    out->fresh_ids.push_back(id);
    r->cap = (int32_t)need;
    return KV_OK;
  }
  void rollback(Plan* out) {
    for (auto it = out->fresh.rbegin(); it != out->fresh.rend(); ++it) alloc_.release(it->first, it->second);
    for (auto it = undo_.rbegin(); it != undo_.rend(); ++it) {
      if (it->existed)
        reqs_[it->id] = it->old;
      else
        reqs_.erase(it->id);
    }
    *out = Plan();
  }

  int64_t N_ = 0, B_ = 1;
  ExtentAlloc alloc_;
  std::unordered_map<uint64_t, Req> reqs_;
  std::unordered_map<uint64_t, int> seen_;
  std::vector<Undo> undo_;
  std::vector<int32_t> moved_;
  std::vector<uint64_t> mark_;
  std::vector<int32_t> sorted_, sorted2_;
  std::pair<int64_t, int64_t> last_fresh_{0, 0};
};

}  // namespace kvswap
