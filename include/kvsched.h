/*
 * kvsched.h — C ABI of the buffer-aware request scheduler and the streaming metrics
 * (host-only: plain CPU code, no GPU call; lives in the same shared library as kvswap.h).
 *
 * This is the decision side of the paper: which requests run, which are preempted, which are
 * resumed (Section 4, "Buffer-Aware Request Scheduling"), and the metrics that score a serving
 * run (Section 3.2, Eq. 1-2, and the effective throughput of Section 7.1).  The swap library
 * executes the decisions; its telemetry (kv_io_stats_get) feeds the I/O estimates used here.
 *
 * All arrays are HOST pointers, read or written during the call only.  Times are seconds,
 * rates tokens per second, memory is counted in KV blocks.  Every function returns 0 or a
 * negative code (KVS_EINVAL).
 */
#ifndef KVSCHED_H
#define KVSCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { KVS_OK = 0, KVS_EINVAL = -1, KVS_ENOMEM = -2 /* working arrays could not be allocated */ };

/* ------------------------------------------------------------------ metrics */

/* Reader model of Section 3.2: request i delivers L tokens at times t_gen[0..L) (non-decreasing);
 * the user starts reading when the first token exists and reads one token every 1/rate seconds,
 * waiting whenever the next token is not there yet.
 *   t_read[j]   = max(t_gen[j], t_read[j-1] + 1/rate),  t_read[0] = t_gen[0]
 *   ttft        = t_gen[0] - t_arrival
 *   rebuffer    = sum over j >= 1 of max(0, t_gen[j] - (t_read[j-1] + 1/rate))
 *   buffer[j]   = B_{i,j}: tokens generated before token j and still unread at t_gen[j]
 *                 (token j itself is not counted)
 * Any output pointer may be NULL. */
int kv_metric_stream(int32_t L, const double* t_gen, double t_arrival, double rate, int32_t* buffer,
                     double* t_read, double* ttft, double* rebuffer);

/* Token weight, Eq. 1: 1 if B <= tau, else max(1 - alpha*(B - tau), 0). */
double kv_metric_token_weight(double B, double tau, double alpha);

/* Sum of Eq. 1 weights over a request's tokens. */
int kv_metric_weight_sum(int32_t L, const int32_t* buffer, double tau, double alpha, double* sum);

/* Effective-throughput weight sum of one request (Section 7.1): a token counts fully while the
 * buffer is below tau1 = 10 % of the request's output length L, decays linearly to zero at
 * tau2 = 20 % of L, and not at all beyond: Eq. 1 with tau = 0.1 L and alpha = 1 / (0.1 L). */
int kv_metric_effective_sum(int32_t L, const int32_t* buffer, double* sum);

/* QoS, Eq. 2: (1/T) * sum_i (weight_sum_i - lambda*ttft_i - mu*rebuffer_i). */
int kv_metric_qos(int32_t n, const double* weight_sum, const double* ttft, const double* rebuffer, double lambda,
                  double mu, double T, double* qos);

/* ---------------------------------------------------------------- scheduler */

enum { KVS_NEW = 0, KVS_RUNNING = 1, KVS_PREEMPTED = 2 }; /* request state seen by the scheduler */
enum { KVS_KEEP = 0, KVS_RUN = 1, KVS_PREEMPT = 2 };      /* decision per request */
enum { KVS_BY_LOAD = 0, KVS_BY_RECOMPUTE = 1 };           /* how a preempted request comes back */
enum { KVS_MODE_IDLE = 0, KVS_MODE_BUFFER_AWARE = 1, KVS_MODE_FCFS = 2 };

typedef struct {
  uint32_t struct_size;
  int64_t mem_blocks;        /* KV blocks the GPU pool can hold for requests (the memory constraint) */
  int64_t ws_blocks;         /* M of the working-set rule: blocks the whole hierarchy (GPU pool + host
                                arena) can hold, since the working set overcommits the GPU */
  int32_t max_running;       /* B: most requests decoding at once */
  double interval;           /* t_schedule_interval */
  double gen_rate;           /* tokens/s each running request receives (decode speed) */
  double capacity;           /* Gamma: tokens/s the system can sustain over the working set */
  double gamma;              /* weight of the low-buffer penalty phi(b) = exp(-b) */
  double safety;             /* mu >= 1: buffer conservativeness of the preemption test */
  double w_adjust;           /* lambda of the working-set rule, in [0, 1] */
  double t_critical;         /* a request whose buffer lasts less than this many seconds is critical */
  double tau_schedule;       /* fixed cost of a scheduling round */
  double weight_tau, weight_alpha; /* Eq. 1 parameters used for the token value v_i */
  /* I/O and compute estimates (from kv_io_stats_get and from the serving loop's history) */
  double evict_gbps, load_gbps;  /* measured payload rates */
  double io_fixed;               /* fixed cost per transfer */
  double evict_queue, load_queue; /* seconds of work already queued on each stream */
  double block_bytes;            /* bytes per KV block (one staging slot) */
  double prefill_per_token;      /* sliding-window average prefill latency per token */
} kv_sched_config;

typedef struct {
  int32_t state;        /* KVS_NEW / KVS_RUNNING / KVS_PREEMPTED */
  double arrival;       /* seconds */
  double rate;          /* r_i, tokens/s the user reads */
  double buffer;        /* b_i^rem: unread tokens */
  int32_t blocks;       /* l_i in KV blocks (context so far, or the prompt for a new request) */
  int32_t dirty_blocks; /* blocks not yet written through (what an eviction still has to move) */
  int32_t tokens;       /* context length in tokens (for the recompute estimate) */
} kv_sched_req;

typedef struct {
  int32_t decision; /* KVS_KEEP / KVS_RUN / KVS_PREEMPT */
  int32_t how;      /* for KVS_RUN of a preempted request: KVS_BY_LOAD or KVS_BY_RECOMPUTE */
  double priority_buffer; /* sort keys, for inspection: phi(b), v*t', r */
  double value;
  double t_overhead; /* min(t_IO, t_recompute) for a preempted request, prefill time for a new one */
} kv_sched_out;

/* One scheduling round over n requests (Section 4.2).  Fills out[0..n) and *mode.
 *  1. Trigger: nothing changes (KVS_MODE_IDLE, all KVS_KEEP) unless a request is waiting (new or
 *     preempted) or a running request is critical (buffer / rate < t_critical).
 *  2. Schedulability (Section 4.3): if the rates of the working set (running + preempted) exceed
 *     `capacity`, fall back to FCFS: requests run in arrival order while memory and max_running
 *     allow; no new request is admitted (KVS_MODE_FCFS).
 *  3. Working set: W_static = floor(ws_blocks / mean blocks per request), W_scheduled =
 *     W_static - w_adjust * (W_static - N_running) while N_running < W_static.  New requests join the
 *     candidate list in arrival order while the working set (running + preempted + admitted) is
 *     below W_scheduled, and only if they can be placed: either a free decode slot and enough free
 *     GPU blocks exist, or some running request is safe to preempt, i.e. its buffer covers the
 *     round trip: buffer >= safety * rate * (t_evict + t_load + tau_schedule).  Each safe request
 *     backs one admission.
 *  4. Buffer balancing: candidates (running, preempted, admitted new) are ordered by phi(b) =
 *     exp(-b) descending, i.e. emptiest buffer first, then by v*t' descending, then by rate
 *     descending, then by index; v = gen_rate * Eq.1 weight of the buffer, t' = max(0, interval -
 *     t_overhead).  Greedy selection in that order under mem_blocks and max_running, then one pass
 *     of adjacent swaps (a selected request next to an unselected one) kept when feasible and when
 *     it raises J = sum over selected of v*t' - gamma * sum over all candidates of phi(b_pred),
 *     b_pred = max(0, b + (selected ? gen_rate*t' : 0) - rate*interval).
 *  5. A preempted request that is selected comes back by load or by recompute, whichever estimate
 *     is smaller: t_IO = evict_queue + t_evict + load_queue + t_load, t_recompute = tokens *
 *     prefill_per_token. */
int kv_sched_step(const kv_sched_config* cfg, int32_t n, const kv_sched_req* req, kv_sched_out* out, int32_t* mode);

#ifdef __cplusplus
}
#endif
#endif /* KVSCHED_H */
