// Buffer-aware request scheduler and streaming metrics (declared in include/kvsched.h).
// Host-only C++: the decision side of the paper (Section 4.2 two-step scheduler, Section 4.3
// schedulability and FCFS fallback, Section 3.2 metrics).  The swap library executes what is
// decided here.  The order of the floating-point operations is part of the contract: the test
// oracle restates the same rules and must reach the same decisions.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/kvsched.h"

extern "C" {

double kv_metric_token_weight(double B, double tau, double alpha) {
  if (B <= tau) return 1.0;
  const double w = 1.0 - alpha * (B - tau);
  return w > 0.0 ? w : 0.0;
}

int kv_metric_stream(int32_t L, const double* t_gen, double t_arrival, double rate, int32_t* buffer, double* t_read,
                     double* ttft, double* rebuffer) try {
  if (L < 0 || (L > 0 && !t_gen) || !(rate > 0.0)) return KVS_EINVAL;
  for (int32_t j = 1; j < L; j++)
    if (t_gen[j] < t_gen[j - 1]) return KVS_EINVAL;
  const double gap = 1.0 / rate;
  std::vector<double> rd((size_t)L);
  double stall = 0.0;
  for (int32_t j = 0; j < L; j++) {
    if (j == 0) {
      rd[0] = t_gen[0];
    } else {
      const double due = rd[(size_t)j - 1] + gap;
      if (t_gen[j] > due) {
        stall += t_gen[j] - due;
        rd[(size_t)j] = t_gen[j];
      } else {
        rd[(size_t)j] = due;
      }
    }
  }
  if (buffer) {
    int32_t k = 0;  // tokens read no later than t_gen[j] among those before j
    for (int32_t j = 0; j < L; j++) {
      while (k < j && rd[(size_t)k] <= t_gen[j]) k++;
      buffer[j] = j - k;
    }
  }
  if (t_read)
    for (int32_t j = 0; j < L; j++) t_read[j] = rd[(size_t)j];
  if (ttft) *ttft = L > 0 ? t_gen[0] - t_arrival : 0.0;
  if (rebuffer) *rebuffer = stall;
  return KVS_OK;
} catch (...) {
  return KVS_ENOMEM;  // only allocations can throw in here; nothing was written that the caller may use
}

int kv_metric_weight_sum(int32_t L, const int32_t* buffer, double tau, double alpha, double* sum) {
  if (L < 0 || (L > 0 && !buffer) || !sum) return KVS_EINVAL;
  double s = 0.0;
  for (int32_t j = 0; j < L; j++) s += kv_metric_token_weight((double)buffer[j], tau, alpha);
  *sum = s;
  return KVS_OK;
}

int kv_metric_effective_sum(int32_t L, const int32_t* buffer, double* sum) {
  if (L <= 0) {
    if (sum) *sum = 0.0;
    return L == 0 && sum ? KVS_OK : KVS_EINVAL;
  }
  const double tau1 = 0.1 * (double)L;
  return kv_metric_weight_sum(L, buffer, tau1, 1.0 / tau1, sum);
}

int kv_metric_qos(int32_t n, const double* weight_sum, const double* ttft, const double* rebuffer, double lambda,
                  double mu, double T, double* qos) {
  if (n < 0 || !(T > 0.0) || !qos || (n > 0 && (!weight_sum || !ttft || !rebuffer))) return KVS_EINVAL;
  double s = 0.0;
  for (int32_t i = 0; i < n; i++) s += weight_sum[i] - lambda * ttft[i] - mu * rebuffer[i];
  *qos = s / T;
  return KVS_OK;
}

int kv_sched_step(const kv_sched_config* cfg, int32_t n, const kv_sched_req* req, kv_sched_out* out, int32_t* mode) try {
  if (!cfg || cfg->struct_size != sizeof(kv_sched_config) || n < 0 || (n > 0 && (!req || !out)) || !mode)
    return KVS_EINVAL;
  if (!(cfg->interval > 0.0) || !(cfg->gen_rate > 0.0) || cfg->mem_blocks < 0 || cfg->max_running < 0 ||
      !(cfg->evict_gbps > 0.0) || !(cfg->load_gbps > 0.0) || !(cfg->block_bytes > 0.0))
    return KVS_EINVAL;
  for (int32_t i = 0; i < n; i++)
    if (req[i].state < KVS_NEW || req[i].state > KVS_PREEMPTED || !(req[i].rate > 0.0) || !(req[i].buffer >= 0.0) ||
        !(req[i].arrival == req[i].arrival) || req[i].blocks < 0 || req[i].dirty_blocks < 0 || req[i].tokens < 0)
      return KVS_EINVAL;

  // per-request estimates
  std::vector<double> t_evict((size_t)n), t_load((size_t)n), phi((size_t)n), value((size_t)n), tprime((size_t)n);
  std::vector<char> safe((size_t)n, 0);
  bool waiting = false, critical = false;
  int32_t n_running = 0, n_preempted = 0;
  double ws_rate = 0.0, sum_blocks = 0.0;
  int64_t running_blocks = 0;
  for (int32_t i = 0; i < n; i++) {
    const kv_sched_req& r = req[i];
    t_evict[(size_t)i] = r.dirty_blocks > 0 ? cfg->io_fixed + (double)r.dirty_blocks * cfg->block_bytes / (cfg->evict_gbps * 1e9) : 0.0;
    t_load[(size_t)i] = cfg->io_fixed + (double)r.blocks * cfg->block_bytes / (cfg->load_gbps * 1e9);
    double overhead = 0.0;
    int how = KVS_BY_LOAD;
    if (r.state == KVS_PREEMPTED) {
      const double t_io = (r.dirty_blocks > 0 ? cfg->evict_queue + t_evict[(size_t)i] : 0.0) + cfg->load_queue + t_load[(size_t)i];
      const double t_re = (double)r.tokens * cfg->prefill_per_token;
      if (t_re < t_io) {
        overhead = t_re;
        how = KVS_BY_RECOMPUTE;
      } else {
        overhead = t_io;
      }
    } else if (r.state == KVS_NEW) {
      overhead = (double)r.tokens * cfg->prefill_per_token;
    }
    const double tp = cfg->interval - overhead;
    tprime[(size_t)i] = tp > 0.0 ? tp : 0.0;
    phi[(size_t)i] = std::exp(-r.buffer);
    value[(size_t)i] = cfg->gen_rate * kv_metric_token_weight(r.buffer, cfg->weight_tau, cfg->weight_alpha) * tprime[(size_t)i];
    out[i].decision = KVS_KEEP;
    out[i].how = how;
    out[i].priority_buffer = phi[(size_t)i];
    out[i].value = value[(size_t)i];
    out[i].t_overhead = overhead;
    sum_blocks += (double)r.blocks;
    if (r.state == KVS_RUNNING) {
      n_running++;
      running_blocks += r.blocks;
      ws_rate += r.rate;
      if (r.buffer / r.rate < cfg->t_critical) critical = true;
      safe[(size_t)i] = r.buffer >= cfg->safety * r.rate * (t_evict[(size_t)i] + t_load[(size_t)i] + cfg->tau_schedule);
    } else {
      waiting = true;
      if (r.state == KVS_PREEMPTED) {
        n_preempted++;
        ws_rate += r.rate;
      }
    }
  }
  if (!waiting && !critical) {
    *mode = KVS_MODE_IDLE;
    return KVS_OK;
  }

  std::vector<int32_t> cand;
  std::vector<char> sel((size_t)n, 0);
  auto finish = [&](int32_t m) {
    for (int32_t i = 0; i < n; i++) {
      if (req[i].state == KVS_RUNNING)
        out[i].decision = sel[(size_t)i] ? KVS_KEEP : KVS_PREEMPT;
      else
        out[i].decision = sel[(size_t)i] ? KVS_RUN : KVS_KEEP;
    }
    *mode = m;
    return KVS_OK;
  };

  if (ws_rate > cfg->capacity) {
    // Section 4.3: not schedulable -> FCFS over the working set, no admission
    for (int32_t i = 0; i < n; i++)
      if (req[i].state != KVS_NEW) cand.push_back(i);
    std::stable_sort(cand.begin(), cand.end(), [&](int32_t a, int32_t b) { return req[a].arrival < req[b].arrival; });
    int64_t used = 0;
    int32_t cnt = 0;
    for (int32_t i : cand)
      if (cnt < cfg->max_running && used + req[i].blocks <= cfg->mem_blocks) {
        sel[(size_t)i] = 1;
        used += req[i].blocks;
        cnt++;
      }
    return finish(KVS_MODE_FCFS);
  }

  // working set size
  const double beta = n > 0 ? sum_blocks / (double)n : 1.0;
  const double w_static = std::floor((double)cfg->ws_blocks / (beta > 1.0 ? beta : 1.0));
  const double w_sched = (double)n_running < w_static ? w_static - cfg->w_adjust * (w_static - (double)n_running) : w_static;
  // admission of new requests, arrival order
  std::vector<int32_t> fresh;
  for (int32_t i = 0; i < n; i++)
    if (req[i].state == KVS_NEW) fresh.push_back(i);
  std::stable_sort(fresh.begin(), fresh.end(), [&](int32_t a, int32_t b) { return req[a].arrival < req[b].arrival; });
  int32_t safe_left = 0;
  for (int32_t i = 0; i < n; i++) safe_left += safe[(size_t)i] ? 1 : 0;
  int64_t free_blocks = cfg->mem_blocks - running_blocks;
  int32_t free_slots = cfg->max_running - n_running;
  double w_current = (double)(n_running + n_preempted);
  std::vector<char> admitted((size_t)n, 0);
  for (int32_t i : fresh) {
    if (!(w_current < w_sched)) break;
    if (free_slots > 0 && (int64_t)req[i].blocks <= free_blocks) {
      free_slots--;
      free_blocks -= req[i].blocks;
    } else if (safe_left > 0) {
      safe_left--;
    } else {
      continue;
    }
    admitted[(size_t)i] = 1;
    w_current += 1.0;
  }

  for (int32_t i = 0; i < n; i++)
    if (req[i].state != KVS_NEW || admitted[(size_t)i]) cand.push_back(i);
  std::stable_sort(cand.begin(), cand.end(), [&](int32_t a, int32_t b) {
    if (req[a].buffer != req[b].buffer) return req[a].buffer < req[b].buffer;  // phi = exp(-b) descending
    if (value[(size_t)a] != value[(size_t)b]) return value[(size_t)a] > value[(size_t)b];
    if (req[a].rate != req[b].rate) return req[a].rate > req[b].rate;
    return a < b;
  });
  int64_t used = 0;
  int32_t cnt = 0;
  for (int32_t i : cand)
    if (cnt < cfg->max_running && used + req[i].blocks <= cfg->mem_blocks) {
      sel[(size_t)i] = 1;
      used += req[i].blocks;
      cnt++;
    }
  auto objective = [&]() {
    double gain = 0.0, pen = 0.0;
    for (int32_t i : cand) {
      double b = req[i].buffer - req[i].rate * cfg->interval;
      if (sel[(size_t)i]) {
        gain += value[(size_t)i];
        b += cfg->gen_rate * tprime[(size_t)i];
      }
      if (b < 0.0) b = 0.0;
      pen += std::exp(-b);
    }
    return gain - cfg->gamma * pen;
  };
  for (size_t k = 0; k + 1 < cand.size(); k++) {
    const int32_t a = cand[k], b = cand[k + 1];
    if (sel[(size_t)a] == sel[(size_t)b]) continue;
    const int32_t on = sel[(size_t)a] ? a : b, off = sel[(size_t)a] ? b : a;
    if (used - req[on].blocks + req[off].blocks > cfg->mem_blocks) continue;
    const double before = objective();
    sel[(size_t)on] = 0;
    sel[(size_t)off] = 1;
    const double after = objective();
    if (after > before + 1e-12) {
      used += req[off].blocks - req[on].blocks;
    } else {
      sel[(size_t)on] = 1;
      sel[(size_t)off] = 0;
    }
  }
  return finish(KVS_MODE_BUFFER_AWARE);
} catch (...) {
  return KVS_ENOMEM;  // only allocations can throw in here; nothing was written that the caller may use
}

}  // extern "C"
