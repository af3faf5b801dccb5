// Host-side scheduler state machines that the monitor and barrier threads run, kept free of any GPU call so that
// the same code can be driven over recorded traces on a CPU: the Bubble Monitor's sliding window, the Kernel
// Barrier's token account (Sec. 3.3), the rules this build adds around the token rule, the check of the invariant
// "an inference kernel starts only inside a detected bubble", and the latency histogram of the statistics.
#pragma once
#include <atomic>
#include <stdint.h>
#include <vector>

#include "specinf.h"

namespace sif {

// Bubble Monitor (Sec. 3.3): the per-period counts of training kernels in a sliding window of W entries; push()
// records the newest count and returns Z_c, the number of consecutive zero counts that end with it.
class BmWindow {
 public:
  explicit BmWindow(uint32_t cap) : cap_(cap ? cap : 1) { w_.reserve(cap_); }
  uint32_t push(uint32_t count) {
    if (w_.size() == cap_) w_.erase(w_.begin());
    w_.push_back(count);
    return sif_zero_count(w_.data(), (uint32_t)w_.size());
  }
 private:
  uint32_t cap_;
  std::vector<uint32_t> w_;
};

// Kernel Barrier, offline token mechanism (Sec. 3.3), for one inference instance.  The grant of a new period replaces
// what was left of the last one; the kernel at the head of the instance's queue is forwarded iff the balance covers
// its charge, which is then taken off (sif_kb_release on that one kernel).
struct KbTokens {
  uint64_t balance = 0;
  void new_period(uint64_t grant) { balance = grant; }
  bool covers(uint32_t charge) const { return sif_kb_release(&charge, 1, balance, nullptr) == 1; }
  void spend(uint32_t charge) { (void)sif_kb_release(&charge, 1, balance, &balance); }
  void clear() { balance = 0; }
};

// ---- rules of this build around the token rule (none of them is the paper's) ---------------------------------
// Speculation depth: the predicted time of forwarded but unfinished kernels stays within max_ahead tokens (the
// paper's barrier forwards at the CPU launch site and is effectively of depth one); a kernel is never held back
// by this rule when nothing is in flight.
inline bool kb_depth_ok(uint64_t outstanding_us, uint64_t charge, uint64_t max_ahead, size_t n_inflight) {
  return !(outstanding_us + charge > max_ahead && n_inflight > 0);
}
// What the device gate is bound to refuse is not launched: behind what is in flight (its predicted time plus the
// gap of kGapNs after each kernel) this kernel would end after the predicted end of the bubble.
constexpr uint64_t kGapNs = 5000;
inline bool kb_fits_bubble(uint64_t rest_ns, uint64_t outstanding_us, size_t n_inflight, double cost_us) {
  return rest_ns >= 1000ull * outstanding_us + kGapNs * n_inflight + (uint64_t)(cost_us * 1000.0);
}

// ---- latency histogram ------------------------------------------------------------------------------------------
// Fixed buckets, sixteen per power of two (a bucket is at most 1/16 wider than its lower edge), values below 16 ns
// one bucket each: adding and reading are lock-free, so the statistics call never waits for a thread that records.
struct LatencyHist {
  static constexpr uint32_t kBuckets = 61 * 16;
  std::atomic<uint64_t> n[kBuckets];
  LatencyHist() { clear(); }
  void clear() { for (auto& c : n) c.store(0, std::memory_order_relaxed); }
  void add(uint64_t ns) { n[sif_latency_bucket(ns)].fetch_add(1, std::memory_order_relaxed); }
  // nearest-rank percentile over the recorded values (sif_latency_percentile on a snapshot of the counts)
  uint64_t percentile(double p) const {
    uint64_t snap[kBuckets];
    for (uint32_t b = 0; b < kBuckets; ++b) snap[b] = n[b].load(std::memory_order_relaxed);
    return sif_latency_percentile(snap, kBuckets, p);
  }
};

}  // namespace sif
