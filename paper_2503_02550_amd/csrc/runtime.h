// Host-side structures of the collocation runtime: streams with their activity records, kernel plans of the
// registered models, and the context that owns the monitor and barrier threads.
#pragma once
#include <atomic>
#include <condition_variable>
#include <deque>
#include <functional>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <unordered_map>
#include <vector>

#include "launch.h"

namespace sif {

// One stream and its device-side bookkeeping.
struct StreamState {
  hipStream_t stream = nullptr;
  StreamRec* rec = nullptr;        // HBM
  Slot* ring = nullptr;            // HBM, kRingSlots entries
  uint32_t next_kseq = 1;          // launch numbers start at 1
  uint32_t kind = 0;
};

// One kernel launch of a plan.
struct Op {
  std::function<sif_status(hipStream_t, const KCtl&)> fn;
  const char* name = "";
  double cost_us = 5.0;            // predicted duration (analytic estimate, replaced by calibration)
  int32_t bubble_site = -1;        // training plans: >= 0 means "bubble of bubble_ns here" instead of a kernel
  uint64_t bubble_ns = 0;
  int32_t prof_class = -1;         // >= 0: GEMM layout variant (a_layout*2 + b_layout), timed with events when profiling
  double flops = 0.0;              // algorithmic floating-point operations of the launch
  // pipeline-stage plans: a kernel belongs to pass 2*micro_batch + (0 forward, 1 backward); a bubble is the idle
  // interval (pp_kind, pp_index) of the 1F1B schedule (see sif_pp_1f1b_bubbles)
  int32_t pp_pass = -1, pp_kind = -1, pp_index = 0;
  bool dp_overlap = false;         // bubble whose length the device derives from the bucketed gradient exchange
  // a matrix product whose rows are independent (A [M][K] row-major, one batch) can be cut into two launches over
  // row ranges, with the same bits: `gemm` holds its arguments
  bool row_split = false;
  sif_gemm_args gemm{};
};
typedef std::vector<Op> Plan;

// Bump allocator over a caller-owned workspace; with base == nullptr it only measures.
struct Arena {
  unsigned char* base = nullptr;
  uint64_t off = 0;
  void* take(uint64_t bytes) {
    off = (off + 255) & ~uint64_t(255);
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
};

struct NamedTensor { void* ptr; uint64_t elems; };

struct TrainModel {
  sif_train_desc desc;
  uint64_t n_params = 0;
  Plan plan;                                        // one training step, bubbles included
  std::unordered_map<std::string, NamedTensor> tensors;   // "name" or "name.<layer>"
  const void** p_inputs = nullptr;                  // host cells the plan's closures read at launch time
  const void* cur_inputs = nullptr;
  const void* cur_targets = nullptr;
  float* cur_loss = nullptr;
  uint64_t max_bubble_ns = 0;
  uint64_t workspace_bytes = 0;
  std::vector<uint32_t> last_kseq;                  // launch number of each op in the most recent step
  bool pp_times_estimated = false;                  // pipeline bubbles were sized from the cost model, not from the caller
  // bucketed gradient exchange beside backward (dp_bucket_bytes > 0): per bucket its bytes, the op whose end makes
  // it final and how long the exchange of the bucket takes
  struct DpBucket { uint64_t bytes; uint32_t ready_op; uint64_t dur_ns; };
  std::vector<DpBucket> dp_buckets;
};

struct InferModel {
  sif_infer_desc desc;
  uint64_t n_params = 0;
  void* work = nullptr;                             // working copy of the weights
  std::unordered_map<std::string, void*> bufs;
  // cost per op of the plan for the registered (batch, seq), measured by calibration: [n - 1] for n coalesced
  // requests (calib_cost_us = the single-request plan)
  std::vector<double> calib_cost_us;
  std::vector<std::vector<double>> calib_cost_us_n;
  double calib_total_us = 0.0;
  uint32_t calib_batch = 0, calib_seq = 0;
  void* calib_in = nullptr;
  void* calib_out = nullptr;
};

struct Job {
  sif_ticket ticket = 0;
  int32_t model = -1;
  bool online = false;
  uint32_t batch = 0, seq = 0;
  uint64_t t_arrival_ns = 0, t_done_ns = 0;
  const void* in_dev = nullptr;
  void* out_dev = nullptr;
  std::vector<Job*> parts;       // a coalesced job: the submitted requests it runs (it has no ticket of its own)
  Plan plan;
  uint32_t next_op = 0;          // next op to launch
  uint32_t done_ops = 0;         // ops known to have run
  int32_t result = 1;            // 1 pending, 0 done, < 0 error
};

// cost_us: what the launch added to outstanding_us; ev: index of the completion event recorded behind it (the last
// kernel of a job) or -1; check_gate: admitted into a bubble, so its start is checked against that bubble's stamps
struct InFlight { uint32_t kseq; Job* job; uint32_t op; uint32_t idle_seq; uint64_t cost_us; int32_t ev; bool check_gate; };

// Layout / plan builders (models.hip)
uint64_t model_n_params(const sif_model_shape& s);
sif_status build_train_model(TrainModel& tm, hipStream_t stream);
uint64_t infer_workspace_bytes(const sif_infer_desc& d);
sif_status build_infer_model(InferModel& im, hipStream_t stream);
struct InferIO { const void* in_dev; void* out_dev; uint32_t seq = 0; };      // seq: this request's own length (0 = the common one)
// One kernel sequence for `n_io` requests of `batch` x `seq` each (n_io > 1: encoder models only).  Requests of one
// sequence each (batch = 1) may differ in length (InferIO::seq); `seq` is then the longest.
sif_status build_infer_plan(const InferModel& im, const InferIO* io, uint32_t n_io, uint32_t batch, uint32_t seq,
                            uint32_t kernel_us_max, Plan& out);
uint32_t infer_coalesce(const sif_infer_desc& d);
// Rows of a row-splittable product that fill the chip with one whole round of tiles (the unit it is cut in)
uint32_t gemm_round_rows(const sif_gemm_args& a);
// Cuts `op` (row_split) into its first `rows_first` rows (a multiple of 128, 0 < rows_first < m) and the rest
void split_gemm_rows(const Op& op, uint32_t rows_first, Op& first, Op& rest);
constexpr uint32_t kMaxCoalesce = 32;     // most requests one coalesced kernel sequence serves

// markers.hip
sif_status launch_bubble(hipStream_t s, StreamRec* rec, Mirror* mir, Slot* slot, uint32_t seq, uint32_t site, uint64_t ticks,
                         uint64_t max_ticks, uint32_t device_timed, uint32_t kind_id);
// Buckets of an overlapped gradient exchange as the bubble kernel sees them: how many launches before the bubble
// each bucket's last producer ran, and how many ticks its exchange takes.
constexpr uint32_t kMaxDpBuckets = 48;
struct DpBucketArgs { uint32_t n; uint32_t back[kMaxDpBuckets]; uint64_t ticks[kMaxDpBuckets]; };
sif_status launch_bubble_overlap(hipStream_t s, StreamRec* rec, Mirror* mir, Slot* ring, uint32_t kseq, const DpBucketArgs& b, uint32_t seq,
                                 uint32_t site, uint64_t max_ticks, uint32_t device_timed, uint32_t kind_id);
sif_status launch_step_marker(hipStream_t s, StreamRec* rec, Mirror* mir, Slot* slot, uint32_t end, uint32_t kind_id);
sif_status launch_probe(hipStream_t spin_stream, hipStream_t stamp_stream, uint64_t ticks, uint64_t* out);
sif_status launch_reset_skip(hipStream_t s, StreamRec* rec, Mirror* mir, uint32_t epoch);

}  // namespace sif
