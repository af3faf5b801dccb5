// Scheduler rules as pure host functions: Bubble Monitor zero-count, Algorithm 1 (Adaptive Kernel Scheduling),
// the Kernel Barrier's offline token rule and online pull rule (Sec. 3.3), the collocation principles
// (Sec. 3.2) and the bubble model.  The runtime threads call these; they touch no GPU state.
#include "launch.h"
#include "kb_rules.h"

extern "C" {

uint32_t sif_zero_count(const uint32_t* counts, uint32_t n) {
  uint32_t z = 0;
  if (counts == nullptr) return 0;
  while (z < n && counts[n - 1 - z] == 0) ++z;
  return z;
}

sif_status sif_alg1_step(const sif_alg1_params* p, uint32_t zc, uint64_t* pool, uint64_t* grant, int32_t* status) {
  if (!p || !pool || !grant || !status) return sif::fail(SIF_E_INVAL, "alg1: null pointer");
  if (p->m == 0 || p->gamma_den == 0) return sif::fail(SIF_E_INVAL, "alg1: m and gamma_den must be positive");
  if (zc <= p->alpha) {                     // conservative phase: keep the GPU logically busy
    *pool = 0; *grant = 0; *status = SIF_STATUS_BUSY;
    return SIF_OK;
  }
  const uint64_t base = *pool > p->t0 ? *pool : p->t0;
  const uint64_t grown = base * p->gamma_num / p->gamma_den;
  if (zc <= p->beta) {                      // incremental phase: grow towards LL, still busy for online
    *pool = grown < p->ll ? grown : p->ll;
    *status = SIF_STATUS_BUSY;
  } else {                                  // stable phase: grow towards UL, idle
    *pool = grown < p->ul ? grown : p->ul;
    *status = SIF_STATUS_IDLE;
  }
  *grant = *pool / p->m;
  return SIF_OK;
}

uint32_t sif_kb_release(const uint32_t* costs, uint32_t n, uint64_t balance, uint64_t* balance_left) {
  uint32_t i = 0;
  while (costs != nullptr && i < n && balance >= costs[i]) balance -= costs[i++];
  if (balance_left) *balance_left = balance;
  return i;
}

uint32_t sif_kb_charge(uint64_t predicted_us, uint64_t ul, uint32_t m) {
  const uint64_t cap = (m != 0 && ul / m > 0) ? ul / m : 1;
  const uint64_t c = predicted_us < cap ? predicted_us : cap;
  return (uint32_t)(c > 0xFFFFFFFFull ? 0xFFFFFFFFull : c);
}

sif_status sif_sched_run_trace(const sif_alg1_params* p, uint32_t window, const uint32_t* counts, uint32_t n_periods,
                               const uint32_t* costs, uint32_t n_costs, uint32_t* zc_out, uint64_t* pool_out,
                               uint64_t* grant_out, int32_t* status_out, uint32_t* released_out) {
  if (!p || window == 0 || (n_periods > 0 && !counts) || (n_costs > 0 && !costs)) return sif::fail(SIF_E_INVAL, "run_trace: null or empty argument");
  // the objects the monitor thread and the barrier thread keep, driven by the trace instead of by a device
  sif::BmWindow bm(window);
  sif::KbTokens tok;
  uint64_t pool = 0;
  uint32_t head = 0;
  for (uint32_t t = 0; t < n_periods; ++t) {
    const uint32_t zc = bm.push(counts[t]);
    uint64_t grant = 0;
    int32_t status = SIF_STATUS_BUSY;
    const sif_status st = sif_alg1_step(p, zc, &pool, &grant, &status);
    if (st != SIF_OK) return st;
    tok.new_period(grant);
    uint32_t n = 0;
    while (head < n_costs && tok.covers(costs[head])) { tok.spend(costs[head]); ++head; ++n; }
    if (zc_out) zc_out[t] = zc;
    if (pool_out) pool_out[t] = pool;
    if (grant_out) grant_out[t] = grant;
    if (status_out) status_out[t] = status;
    if (released_out) released_out[t] = n;
  }
  return SIF_OK;
}

int32_t sif_gate_violation(uint64_t t0, uint64_t bubble_begin, uint64_t bubble_end) {
  return t0 < bubble_begin || (bubble_end != 0 && t0 > bubble_end);
}

uint32_t sif_latency_bucket(uint64_t ns) {
  if (ns < 16) return (uint32_t)ns;
  const uint32_t top = 63u - (uint32_t)__builtin_clzll(ns);        // position of the leading one, >= 4
  return (top - 3u) * 16u + (uint32_t)((ns >> (top - 4u)) & 15u);
}

uint64_t sif_latency_bucket_lower_ns(uint32_t bucket) {
  if (bucket < 16) return bucket;
  if (bucket >= sif::LatencyHist::kBuckets) bucket = sif::LatencyHist::kBuckets - 1;
  const uint32_t top = bucket / 16u + 3u;
  return (uint64_t)(16u + bucket % 16u) << (top - 4u);
}

uint32_t sif_latency_buckets(void) { return sif::LatencyHist::kBuckets; }

uint64_t sif_latency_percentile(const uint64_t* counts, uint32_t n_buckets, double p) {
  if (!counts || n_buckets == 0 || !(p > 0.0)) return 0;
  if (n_buckets > sif::LatencyHist::kBuckets) n_buckets = sif::LatencyHist::kBuckets;
  if (p > 1.0) p = 1.0;
  uint64_t total = 0;
  for (uint32_t b = 0; b < n_buckets; ++b) total += counts[b];
  if (total == 0) return 0;
  uint64_t rank = (uint64_t)(p * (double)total);                    // nearest rank: ceil(p * total), at least 1
  if ((double)rank < p * (double)total) ++rank;
  if (rank == 0) rank = 1;
  uint64_t seen = 0;
  for (uint32_t b = 0; b < n_buckets; ++b) {
    seen += counts[b];
    if (seen >= rank) {
      const uint64_t lo = sif_latency_bucket_lower_ns(b);
      const uint64_t hi = b + 1 < sif::LatencyHist::kBuckets ? sif_latency_bucket_lower_ns(b + 1) : lo + 1;
      return lo + (hi - 1 - lo) / 2;                                  // middle of the values the bucket holds
    }
  }
  return sif_latency_bucket_lower_ns(n_buckets - 1);
}

int32_t sif_online_pull_ok(int32_t status, uint32_t queue_len, uint64_t predicted_remaining_ns, uint64_t predicted_request_ns) {
  return status == SIF_STATUS_IDLE && queue_len > 0 && predicted_remaining_ns >= predicted_request_ns;
}

int32_t sif_principle_1(const uint64_t* peak_bytes, uint32_t n, uint64_t capacity_bytes) {
  uint64_t s = 0;
  for (uint32_t i = 0; peak_bytes != nullptr && i < n; ++i) {
    if (s + peak_bytes[i] < s) return 0;    // overflow
    s += peak_bytes[i];
  }
  return s < capacity_bytes;
}

int32_t sif_principle_2(uint64_t min_exec_ns, uint64_t max_bubble_ns) { return min_exec_ns < max_bubble_ns; }

uint64_t sif_collective_ns(uint64_t n_bytes, uint64_t bw_bytes_per_s) {
  if (bw_bytes_per_s == 0) return 0;
  return (uint64_t)(((unsigned __int128)n_bytes * 1000000000ull) / bw_bytes_per_s);
}

int32_t sif_pp_1f1b_bubbles(uint32_t stage, uint32_t n_stages, uint32_t n_micro, uint64_t tf_ns, uint64_t tb_ns,
                            int32_t* kind, int32_t* index, uint64_t* ns, uint32_t max) {
  if (n_stages == 0 || stage >= n_stages || n_micro < n_stages) return sif::fail(SIF_E_INVAL, "pp: need stage < n_stages <= n_micro");
  if (max > 0 && (!kind || !index || !ns)) return sif::fail(SIF_E_INVAL, "pp: null output");
  const uint32_t w = n_stages - 1 - stage;   // warm-up forwards = cool-down backwards
  uint32_t cnt = 0;
  auto put = [&](int32_t k, int32_t i, uint64_t t) {
    if (cnt < max) { kind[cnt] = k; index[cnt] = i; ns[cnt] = t; }
    ++cnt;
  };
  if (stage > 0) put(0, 0, (uint64_t)stage * tf_ns);            // wait for the first activation
  if (w > 0) {
    put(1, 0, (uint64_t)w * tb_ns);                             // first gradient travels back through w stages
    for (uint32_t k = n_micro - w; k < n_micro; ++k) put(1, (int32_t)k, tf_ns);   // cool-down: one forward slot empty
  }
  if (stage > 0) put(2, -1, (uint64_t)stage * tb_ns);           // earlier stages still draining
  return (int32_t)cnt;
}

int32_t sif_dp_gradient_buckets(const uint64_t* group_bytes, uint32_t n_groups, uint64_t cap_bytes, uint32_t* bucket_of_group) {
  if (cap_bytes == 0 || (n_groups > 0 && (!group_bytes || !bucket_of_group))) return sif::fail(SIF_E_INVAL, "dp buckets: zero cap or null array");
  uint32_t bucket = 0;
  uint64_t held = 0;
  bool open = false;
  for (uint32_t i = 0; i < n_groups; ++i) {
    bucket_of_group[i] = bucket;
    held += group_bytes[i];
    open = true;
    if (held >= cap_bytes) { ++bucket; held = 0; open = false; }
  }
  return (int32_t)(bucket + (open ? 1u : 0u));
}

uint64_t sif_dp_overlapped_wait(const uint64_t* ready_ns, const uint64_t* dur_ns, uint32_t n, uint64_t end_ns) {
  uint64_t finish = 0;
  for (uint32_t k = 0; ready_ns != nullptr && dur_ns != nullptr && k < n; ++k) finish = (ready_ns[k] > finish ? ready_ns[k] : finish) + dur_ns[k];
  return finish > end_ns ? finish - end_ns : 0;
}

uint32_t sif_feedback_share(uint32_t share_ppm, uint64_t step_ns, uint64_t ref_ns, uint32_t eps_ppm, uint32_t add_ppm, uint32_t cap_ppm) {
  const unsigned __int128 lhs = (unsigned __int128)step_ns * 1000000u, rhs = (unsigned __int128)ref_ns * (1000000ull + eps_ppm);
  if (lhs > rhs) return share_ppm / 2;
  const uint64_t up = (uint64_t)share_ppm + add_ppm;
  return (uint32_t)(up < cap_ppm ? up : cap_ppm);
}

uint64_t sif_concurrent_account(uint64_t balance_ns, uint32_t share_ppm, uint64_t period_ns, uint64_t burst_ns) {
  const uint64_t gain = (uint64_t)(((unsigned __int128)period_ns * share_ppm) / 1000000u);
  const uint64_t b = balance_ns + gain;
  return b < burst_ns ? b : burst_ns;
}

}  // extern "C"
