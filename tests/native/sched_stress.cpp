// CPU-only stress driver for the scheduler and metrics (paper_2510_02758_amd/csrc/scheduler.cpp, pure
// C++), built with AddressSanitizer + UBSan by tests/test_native_sanitizers.py.  Random request sets,
// including empty ones and degenerate configurations, go through kv_sched_step and the metric
// functions; every answer must satisfy the invariants any decision has (slots and memory respected,
// only running requests are preempted, only waiting ones are started), and rejected inputs must be
// rejected without touching the outputs' neighbours.
//
// usage: sched_stress <seed> <rounds>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../../include/kvsched.h"

static void die(const char* what, int round) {
  std::fprintf(stderr, "VIOLATION in round %d: %s\n", round, what);
  std::exit(1);
}

int main(int argc, char** argv) {
  const unsigned long long seed = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 1;
  const int rounds = argc > 2 ? std::atoi(argv[2]) : 2000;
  std::mt19937_64 rng(seed);
  auto uni = [&](double lo, double hi) { return lo + (hi - lo) * (double)(rng() >> 11) / 9007199254740992.0; };
  auto rnd = [&](long lo, long hi) { return lo + (long)(rng() % (unsigned long long)(hi - lo + 1)); };
  long modes[3] = {0, 0, 0}, rejected = 0;
  for (int round = 0; round < rounds; round++) {
    kv_sched_config c;
    std::memset(&c, 0, sizeof(c));
    c.struct_size = sizeof(c);
    c.mem_blocks = rnd(0, 80);
    c.ws_blocks = rnd(0, 300);
    c.max_running = (int32_t)rnd(0, 10);
    c.interval = uni(0.05, 2.0);
    c.gen_rate = uni(1, 80);
    c.capacity = rnd(0, 2) ? 1e9 : uni(10, 200);
    c.gamma = uni(0, 50);
    c.safety = uni(1, 3);
    c.w_adjust = uni(0, 1);
    c.t_critical = uni(0, 3);
    c.tau_schedule = uni(0, 0.5);
    c.weight_tau = uni(0, 50);
    c.weight_alpha = uni(0, 0.5);
    c.evict_gbps = uni(1, 60);
    c.load_gbps = uni(1, 60);
    c.io_fixed = uni(0, 1e-3);
    c.evict_queue = uni(0, 0.2);
    c.load_queue = uni(0, 0.2);
    c.block_bytes = 2.0 * 1048576.0;
    c.prefill_per_token = rnd(0, 1) ? 0.0 : uni(1e-6, 1e-3);
    const int n = (int)rnd(0, 40);
    // guard elements on both sides catch writes outside out[0..n)
    std::vector<kv_sched_req> req((size_t)n);
    std::vector<kv_sched_out> out((size_t)n + 2);
    kv_sched_out guard;
    std::memset(&guard, 0x5A, sizeof(guard));
    out.front() = guard;
    out.back() = guard;
    for (auto& r : req) {
      r.state = (int32_t)rnd(0, 2);
      r.arrival = uni(0, 10);
      r.rate = uni(1, 40);
      r.buffer = r.state == KVS_NEW ? 0.0 : (rnd(0, 3) ? uni(0, 300) : 0.0);
      r.blocks = (int32_t)rnd(0, 30);
      r.dirty_blocks = (int32_t)rnd(0, r.blocks);
      r.tokens = (int32_t)rnd(0, 8000);
    }
    const bool poison = rnd(0, 15) == 0 && n > 0;
    if (poison) {
      kv_sched_req& r = req[(size_t)rnd(0, n - 1)];
      switch (rnd(0, 3)) {
        case 0: r.rate = 0.0; break;
        case 1: r.buffer = -1.0; break;
        case 2: r.state = 9; break;
        default: r.buffer = std::nan(""); break;
      }
    }
    int32_t mode = -7;
    const int rc = kv_sched_step(&c, n, req.data(), out.data() + 1, &mode);
    if (std::memcmp(&out.front(), &guard, sizeof(guard)) || std::memcmp(&out.back(), &guard, sizeof(guard)))
      die("wrote outside out[0..n)", round);
    if (poison) {
      if (rc != KVS_EINVAL) die("bad request accepted", round);
      rejected++;
      continue;
    }
    if (rc != KVS_OK) die("valid input rejected", round);
    if (mode < 0 || mode > 2) die("mode", round);
    modes[mode]++;
    long run = 0, mem = 0;
    for (int i = 0; i < n; i++) {
      const kv_sched_out& o = out[(size_t)i + 1];
      const bool running = req[(size_t)i].state == KVS_RUNNING;
      if (o.decision == KVS_PREEMPT && !running) die("preempted a request that is not running", round);
      if (o.decision == KVS_RUN && running) die("started a running request", round);
      if (mode == KVS_MODE_IDLE && o.decision != KVS_KEEP) die("idle round changed something", round);
      if (mode == KVS_MODE_FCFS && o.decision == KVS_RUN && req[(size_t)i].state == KVS_NEW)
        die("admission during the fallback", round);
      if (!(o.t_overhead >= 0) || !(o.value >= 0) || !(o.priority_buffer >= 0 && o.priority_buffer <= 1))
        die("estimate out of range", round);
      if ((running && o.decision == KVS_KEEP) || o.decision == KVS_RUN) {
        run++;
        mem += req[(size_t)i].blocks;
      }
    }
    if (mode != KVS_MODE_IDLE && (run > c.max_running || mem > c.mem_blocks)) die("slots or memory exceeded", round);

    // metrics on a random trace
    const int L = (int)rnd(0, 200);
    std::vector<double> t_gen((size_t)L), t_read((size_t)L);
    std::vector<int32_t> buf((size_t)L);
    double t = uni(0, 1);
    for (auto& x : t_gen) x = (t += uni(0, 0.2));
    double ttft = -1, reb = -1, ws = -1, es = -1;
    const double rate = uni(1, 50);
    if (kv_metric_stream(L, t_gen.data(), 0.0, rate, buf.data(), t_read.data(), &ttft, &reb) != KVS_OK) die("stream", round);
    for (int j = 0; j < L; j++) {
      if (buf[(size_t)j] < 0 || buf[(size_t)j] > j) die("buffer out of range", round);
      if (t_read[(size_t)j] < t_gen[(size_t)j]) die("read before generated", round);
      if (j && t_read[(size_t)j] < t_read[(size_t)j - 1] + 1.0 / rate - 1e-9) die("read faster than the rate", round);
    }
    if (reb < 0) die("negative rebuffering", round);
    if (kv_metric_weight_sum(L, buf.data(), c.weight_tau, c.weight_alpha, &ws) != KVS_OK || ws < 0 || ws > L + 1e-9)
      die("weight sum", round);
    if (kv_metric_effective_sum(L, buf.data(), &es) != KVS_OK || es < 0 || es > L + 1e-9) die("effective sum", round);
  }
  std::printf("seed %llu: %d rounds ok (idle %ld, buffer-aware %ld, fcfs %ld, rejected %ld)\n", seed, rounds, modes[0],
              modes[1], modes[2], rejected);
  return modes[0] > 0 && modes[1] > 0 && modes[2] > 0 && rejected > 0 ? 0 : 2;
}
