// The collocation runtime behind the C ABI: context, Bubble Monitor thread, Kernel Barrier thread, job queues.
//
// Mapping to the paper's components (Sec. 3.1, 3.3):
//   monitoring library + Bubble Monitor : prologue/epilogue of every training kernel (monitor.h) keep the launch
//       count in HBM and in a pinned host mailbox; the monitor thread samples it every period, keeps the sliding
//       window and computes the zero-count Z_c.
//   CUDA Kernel Scheduler               : the monitor thread evaluates Algorithm 1 on Z_c each period and
//       publishes (tokens, status).  One process, so a pair of atomics replaces the UNIX socket.
//   Kernel Barrier                      : the barrier thread owns the inference stream.  Offline: forwards queued
//       kernels while the period's tokens last.  Online: pulls requests in arrival order while the status is
//       idle and the predicted rest of the bubble holds them.  Launches are speculative: each kernel re-checks the
//       training stream's state on the device (gate) and the first one that finds it busy poisons the rest of
//       the window; the barrier then rewinds to that kernel and waits for the next grant.
#include <algorithm>
#include <chrono>
#include <string.h>

#include "runtime.h"
#include "kb_rules.h"

using namespace sif;

static inline uint64_t host_now_ns() {
  return (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now().time_since_epoch()).count();
}
static inline void cpu_relax(int n) { for (int i = 0; i < n; ++i) __builtin_ia32_pause(); }

constexpr uint32_t kBubbleTable = 4096;

struct sif_ctx {
  sif_config cfg;
  int device = 0;
  StreamState T, I;
  Mirror* mir = nullptr;
  uint64_t tick_hz = 100000000ull;
  uint64_t capacity = 0;

  std::unique_ptr<TrainModel> train;
  std::vector<std::unique_ptr<InferModel>> models;

  std::atomic<uint64_t> bubble_ns[kBubbleTable];
  uint32_t bubble_seq = 0;
  uint32_t step_no = 0;

  std::thread mon, bar;
  std::atomic<bool> stop{false};
  std::atomic<bool> paused{false};
  std::atomic<uint32_t> collocate{1};

  // published by the monitor thread
  std::atomic<uint64_t> grant{0}, pool{0}, period_no{0};
  std::atomic<int32_t> status{SIF_STATUS_BUSY};
  std::atomic<uint32_t> zc{0};
  std::atomic<uint64_t> edge_host_ns{0}, edge_len_ns{0};
  std::atomic<uint32_t> edge_seq{0};

  // jobs
  std::mutex mu;
  std::condition_variable cv;
  std::deque<Job*> online_q;
  std::vector<std::deque<Job*>> offline_q;      // one FIFO per inference instance (indexed like models)
  size_t offline_queued = 0;
  std::unordered_map<sif_ticket, std::unique_ptr<Job>> jobs;
  sif_ticket next_ticket = 1;
  LatencyHist latency;                 // online request latencies (lock-free: the statistics call never waits)
  std::mutex infer_mu;                 // serialises launches on the inference stream

  // barrier thread state
  std::deque<InFlight> inflight;
  uint64_t head_since_ns = 0;       // host time at which the kernel at the head of `inflight` got there
  const Job* rerun_job = nullptr;   // the launch that found the gate closed or was given back: its job and op
  uint32_t rerun_op = 0;
  std::deque<Job*> run_online, run_offline;
  std::vector<std::unique_ptr<Job>> groups;      // coalesced jobs in flight (guarded by mu)
  std::vector<KbTokens> tokens;                  // per offline instance: what is left of the period's grant
  // events recorded behind the last kernel of each job: a job is reported done once its event has completed, i.e.
  // once the stream has passed that kernel and its results are visible to every later reader
  std::vector<hipEvent_t> done_ev;
  std::vector<int32_t> done_ev_free;
  // starts of gated kernels that have completed, waiting to be checked against their bubble's own stamps
  struct GateCheck { uint32_t kseq, b8; uint64_t give_up_ns, t0, begin; bool have; };
  std::deque<GateCheck> gate_pending;
  // what the barrier forwarded, newest kReleaseLog entries (written by the barrier thread only)
  std::vector<sif_release_rec> release_log;
  uint64_t release_n = 0;
  uint64_t period_grant = 0;                     // the grant that the balances were last set to
  size_t rr_next = 0;                            // instance the next offline kernel is looked for first
  uint64_t outstanding_us = 0, last_period = 0;
  bool awaiting_reset = false;
  bool hold = false;                   // after a skipped launch: release nothing until a new bubble begins
  uint32_t hold_seq = 0;
  uint32_t reset_epoch = 0;

  std::atomic<uint64_t> offline_samples{0}, offline_batches{0}, online_done{0}, kernels_launched{0}, periods{0};
  std::atomic<uint64_t> gate_violations{0}, gate_checked{0}, gate_unchecked{0};
  uint64_t step_solo_ns = 0;
  uint32_t train_kernels_base = 0;          // completed training kernels at the last sif_reset_stats
  // concurrent filling with feedback: the share is set by the monitor thread after every training iteration, the
  // time account is kept by the barrier thread
  std::atomic<uint32_t> share_ppm{0};
  uint64_t conc_account_ns = 0;

  // optional event timing of the GEMM launches (sif_profile_gemm)
  std::atomic<uint32_t> prof_on{0};        // 0 off, 1 every GEMM launch, 2 only the variant with both operands K-contiguous
  std::vector<hipEvent_t> prof_ev;      // 2 per timed launch
  uint32_t prof_third[2] = {0, 0};      // eligible launches seen per stream (training, inference) in mode 3
  std::vector<int32_t> prof_class;
  std::vector<double> prof_flops;
  std::vector<uint32_t> prof_kseq;      // launch number on the inference stream, 0 for a training launch
  std::atomic<uint32_t> prof_n{0};

  uint64_t ticks_to_ns(uint64_t t) const { return (uint64_t)((unsigned __int128)t * 1000000000ull / tick_hz); }
  uint64_t ns_to_ticks(uint64_t ns) const { return (uint64_t)((unsigned __int128)ns * tick_hz / 1000000000ull); }
};

static KCtl make_ctl(sif_ctx* c, StreamState& st, uint32_t kind, uint32_t id, const StreamRec* gate, uint32_t cost_ticks) {
  KCtl k{};
  k.rec = st.rec; k.mir = c->mir; k.kseq = st.next_kseq++;
  k.slot = st.ring + (k.kseq % kRingSlots);
  k.gate = gate; k.cost_ticks = cost_ticks;
  k.kind_id = (kind << 28) | (id & 0x0FFFFFFFu);
  return k;
}

constexpr uint32_t kProfMax = 16384;
constexpr uint32_t kReleaseLog = 1u << 16;

// Launches one op; when GEMM profiling is on, brackets it with two events on its own stream.
static sif_status launch_op(sif_ctx* c, Op& op, hipStream_t s, const KCtl& k) {
  const uint32_t prof_mode = c->prof_on.load(std::memory_order_relaxed);
  bool timed = op.prof_class >= 0 && (prof_mode == 1 || (prof_mode >= 2 && op.prof_class == 0));
  // mode 3: every third eligible launch of a stream (each stream is launched by one thread and counts for itself)
  if (timed && prof_mode == 3) timed = (s == c->T.stream ? c->prof_third[0] : c->prof_third[1])++ % 3 == 0;
  if (timed) {
    const uint32_t i = c->prof_n.fetch_add(1, std::memory_order_relaxed);
    if (i < kProfMax) {
      c->prof_class[i] = op.prof_class;
      c->prof_flops[i] = op.flops;
      c->prof_kseq[i] = k.gate != nullptr ? k.kseq : 0;      // gated launches may be skipped on the device: checked when read
      (void)hipEventRecord(c->prof_ev[2 * i], s);
      const sif_status st = op.fn(s, k);
      (void)hipEventRecord(c->prof_ev[2 * i + 1], s);
      return st;
    }
  }
  return op.fn(s, k);
}

constexpr uint64_t kLenFromDevice = ~0ull;     // bubble table entry: the device decides the length and reports it

static inline uint32_t mload(const uint32_t* p) { return __atomic_load_n(p, __ATOMIC_ACQUIRE); }
static inline uint64_t mload(const uint64_t* p) { return __atomic_load_n(p, __ATOMIC_ACQUIRE); }

// ------------------------------------------------------------------------------------------------ monitor
static void monitor_main(sif_ctx* c) {
  (void)hipSetDevice(c->device);
  const uint64_t period_ns = (uint64_t)c->cfg.period_us * 1000ull;
  BmWindow window(c->cfg.window);
  // The mailbox starts zeroed and bubble numbers start at 1.  These must not be read from the mailbox here: the
  // thread may first run after the first bubble has begun, and would then never release it.
  uint32_t prev_launched = 0;
  uint32_t last_idle_seen = 0;
  uint32_t pending_release = 0;
  uint64_t release_at = 0, pool = 0;
  uint64_t next_sample = host_now_ns() + period_ns;
  uint64_t steps_seen = mload(&c->mir->steps), launched_seen = c->kernels_launched.load(std::memory_order_relaxed);
  uint64_t cal_seen = 0, ref = 0;        // feedback: calibrated solo iteration time last seen, reference in use
  while (!c->stop.load(std::memory_order_relaxed)) {
    const uint64_t now = host_now_ns();
    if (c->cfg.feedback) {                 // a training iteration ended: has it lengthened?
      const uint64_t steps = mload(&c->mir->steps);
      if (steps != steps_seen) {
        steps_seen = steps;
        // Reference: the shortest iteration seen since the last calibration, starting from the calibrated solo time
        // (the first iterations of a process run long, and a reference taken from them alone would hide a slowdown).
        const uint64_t cal = __atomic_load_n(&c->step_solo_ns, __ATOMIC_RELAXED);
        if (cal != cal_seen) { cal_seen = cal; ref = cal; }
        const uint64_t step_ns = c->ticks_to_ns(mload(&c->mir->step_ticks_last));
        if (!c->paused.load(std::memory_order_relaxed)) {
          if (ref == 0 || step_ns < ref) ref = step_ns;
          // an iteration during which the barrier forwarded nothing says nothing about the share
          const uint64_t launched = c->kernels_launched.load(std::memory_order_relaxed);
          const bool served = launched != launched_seen;
          launched_seen = launched;
          if (served && c->collocate.load(std::memory_order_relaxed))
            c->share_ppm.store(sif_feedback_share(c->share_ppm.load(std::memory_order_relaxed), step_ns, ref, c->cfg.feedback_eps_ppm,
                                                  c->cfg.feedback_add_ppm, c->cfg.feedback_cap_ppm), std::memory_order_relaxed);
        }
      }
    }
    const uint32_t is = mload(&c->mir->idle_seq);
    if (is != last_idle_seen) {            // a bubble began: time its release on the host clock
      last_idle_seen = is;
      uint64_t len = c->bubble_ns[is % kBubbleTable].load(std::memory_order_acquire);
      if (len == kLenFromDevice) len = c->ticks_to_ns(mload(&c->mir->idle_len_ticks));     // written before idle_seq
      pending_release = is;
      release_at = now + len;
      c->edge_len_ns.store(len, std::memory_order_relaxed);
      c->edge_host_ns.store(now, std::memory_order_relaxed);
      c->edge_seq.store(is, std::memory_order_release);
    }
    if (pending_release != 0 && now >= release_at) {
      __atomic_store_n(&c->mir->release_seq, pending_release, __ATOMIC_RELEASE);
      pending_release = 0;
    }
    if (now >= next_sample) {
      const uint32_t launched = mload(&c->mir->t_launched), completed = mload(&c->mir->t_completed);
      uint32_t count = launched - prev_launched;
      prev_launched = launched;
      if (c->cfg.count_running && count == 0 && launched != completed) count = 1;
      const uint32_t zc = window.push(count);
      uint64_t grant = 0;
      int32_t status = SIF_STATUS_BUSY;
      sif_alg1_step(&c->cfg.alg1, zc, &pool, &grant, &status);
      c->zc.store(zc, std::memory_order_relaxed);
      c->pool.store(pool, std::memory_order_relaxed);
      c->grant.store(grant, std::memory_order_relaxed);
      c->status.store(status, std::memory_order_relaxed);
      c->period_no.fetch_add(1, std::memory_order_release);
      c->periods.fetch_add(1, std::memory_order_relaxed);
      next_sample += period_ns;
      if (next_sample < now) next_sample = now + period_ns;
    }
    cpu_relax(20);
  }
  // never leave a bubble waiting for a host that is gone
  __atomic_store_n(&c->mir->release_seq, 0xFFFFFFFFu, __ATOMIC_RELEASE);
}

// ------------------------------------------------------------------------------------------------ barrier
static void apply_calibration(const InferModel& im, Job& j);

static void finish_job(sif_ctx* c, Job* j, int32_t result) {
  if (!j->parts.empty()) {          // a coalesced job: its requests finish together, then it is dropped
    const std::vector<Job*> parts = j->parts;
    for (Job* p : parts) finish_job(c, p, result);
    std::lock_guard<std::mutex> lk(c->mu);
    c->groups.erase(std::remove_if(c->groups.begin(), c->groups.end(), [&](const std::unique_ptr<Job>& g) { return g.get() == j; }), c->groups.end());
    return;
  }
  std::lock_guard<std::mutex> lk(c->mu);
  j->t_done_ns = host_now_ns();
  j->result = result;
  if (result == 0) {
    if (j->online) {
      c->online_done.fetch_add(1);
      c->latency.add(j->t_done_ns > j->t_arrival_ns ? j->t_done_ns - j->t_arrival_ns : 0);
    } else {
      c->offline_batches.fetch_add(1);
      c->offline_samples.fetch_add(j->batch);
    }
  }
  j->plan.clear();
  c->cv.notify_all();
}

static uint64_t predicted_remaining_ns(sif_ctx* c) {
  const uint32_t seq = c->edge_seq.load(std::memory_order_acquire);
  if (seq == 0 || mload(&c->mir->busy_seq) == seq || mload(&c->mir->idle_seq) != seq) return 0;
  const uint64_t end = c->edge_host_ns.load(std::memory_order_relaxed) + c->edge_len_ns.load(std::memory_order_relaxed);
  const uint64_t now = host_now_ns();
  return end > now ? end - now : 0;
}

// ---- the invariant "an inference kernel starts only inside a detected bubble", checked from the stamps -------------
// A gated kernel that ran left its start time and the number of the bubble its gate saw in the mailbox; the bubble
// kernel left its own begin and end stamps there.  Stage one (as soon as the kernel is known to have completed) reads
// the kernel's word and the bubble's begin; stage two waits for the bubble's end.
static void gate_check_stage_one(const Mirror* m, sif_ctx::GateCheck& g) {
  const uint64_t w = mload(&m->i_gate[g.kseq % kGateStamps]);
  if (((w >> 8) & 0xFFFFu) != (g.kseq & 0xFFFFu)) return;            // the word has not arrived yet
  const uint32_t b8 = (uint32_t)(w & 0xFFu), e = b8 % kBubbleStamps;
  if ((mload(&m->bub_tag[e]) & 0xFFu) != b8) return;
  const uint64_t begin = mload(&m->bub_begin[e]);
  if ((mload(&m->bub_tag[e]) & 0xFFu) != b8) return;                  // the entry was not recycled meanwhile
  // the start time travels as its low 40 bits: rebuild it next to the bubble's begin
  const int64_t rel = (int64_t)(((w >> 24) - (begin & 0xFFFFFFFFFFull)) << 24) >> 24;
  g.t0 = begin + (uint64_t)rel; g.begin = begin; g.b8 = b8; g.have = true;
}

static void process_gate_checks(sif_ctx* c, bool last_pass) {
  const uint64_t now = host_now_ns();
  const Mirror* m = c->mir;
  while (!c->gate_pending.empty()) {
    sif_ctx::GateCheck& g = c->gate_pending.front();
    if (!g.have) gate_check_stage_one(m, g);
    int verdict = -1;                                                   // -1 undecided, 0 inside, 1 violation
    if (g.have) {
      if (sif_gate_violation(g.t0, g.begin, 0)) verdict = 1;
      else {
        const uint32_t e = g.b8 % kBubbleStamps;
        const uint64_t end = mload(&m->bub_end[e]);
        if (end != 0 && (mload(&m->bub_tag[e]) & 0xFFu) == g.b8 && mload(&m->bub_begin[e]) == g.begin) verdict = sif_gate_violation(g.t0, g.begin, end);
        // a kernel that is known to have completed while its bubble is still not over began before that end
        else if (last_pass || now >= g.give_up_ns) verdict = 0;
      }
    } else if (last_pass || now >= g.give_up_ns) {
      c->gate_unchecked.fetch_add(1, std::memory_order_relaxed);        // its stamps never arrived
      c->gate_pending.pop_front();
      continue;
    }
    if (verdict < 0) break;
    if (verdict == 1) c->gate_violations.fetch_add(1, std::memory_order_relaxed);
    c->gate_checked.fetch_add(1, std::memory_order_relaxed);
    c->gate_pending.pop_front();
  }
}

// Of the predicted time of what is in flight, the part the kernel at the head has behind it: it runs since it got to
// the head, inside a bubble not before the bubble's edge; at most nine tenths of its prediction are taken off.
static uint64_t head_elapsed_ns(sif_ctx* c) {
  if (c->inflight.empty()) return 0;
  const uint64_t begin = std::max(c->head_since_ns, c->edge_host_ns.load(std::memory_order_relaxed)), now = host_now_ns();
  return now > begin ? std::min<uint64_t>(now - begin, 900ull * c->inflight.front().cost_us) : 0;
}

static double job_cost_us(const Job* j) {
  double s = 0;
  for (const Op& o : j->plan) s += o.cost_us;
  return s;
}

static void barrier_main(sif_ctx* c) {
  (void)hipSetDevice(c->device);
  while (!c->stop.load(std::memory_order_relaxed)) {
    if (c->paused.load(std::memory_order_acquire)) { std::this_thread::sleep_for(std::chrono::microseconds(50)); continue; }
    std::unique_lock<std::mutex> il(c->infer_mu);
    bool progressed = false;
    const bool gated = (bool)c->train;
    // 1. completions, in launch order
    const uint32_t done = mload(&c->mir->i_done), skip = mload(&c->mir->i_skip_from);
    while (!c->inflight.empty() && c->inflight.front().kseq <= done && (skip == kNone || c->inflight.front().kseq < skip)) {
      InFlight f = c->inflight.front();
      if (f.ev >= 0) {
        // the last kernel of a job: the job is done when the stream has passed it (its results are then visible to
        // whoever reads them next), not when its last block says it is about to leave
        const hipError_t q = hipEventQuery(c->done_ev[f.ev]);
        if (q == hipErrorNotReady) { (void)hipGetLastError(); break; }      // "not ready" must not show up as the next launch's error
        c->done_ev_free.push_back(f.ev);
        if (q != hipSuccess) {
          c->inflight.pop_front();
          auto drop = [&](std::deque<Job*>& qq) { qq.erase(std::remove(qq.begin(), qq.end(), f.job), qq.end()); };
          drop(c->run_online); drop(c->run_offline);
          c->inflight.erase(std::remove_if(c->inflight.begin(), c->inflight.end(), [&](const InFlight& g) { return g.job == f.job; }), c->inflight.end());
          finish_job(c, f.job, fail_hip(q, "barrier: completion event"));
          progressed = true;
          continue;
        }
      }
      c->inflight.pop_front();
      c->head_since_ns = host_now_ns();
      c->outstanding_us = c->outstanding_us > f.cost_us ? c->outstanding_us - f.cost_us : 0;      // exactly what its launch added
      if (f.check_gate) c->gate_pending.push_back(sif_ctx::GateCheck{f.kseq, 0, host_now_ns() + 200000000ull, 0, 0, false});
      if (++f.job->done_ops == f.job->plan.size()) {
        auto drop = [&](std::deque<Job*>& q) { q.erase(std::remove(q.begin(), q.end(), f.job), q.end()); };
        drop(c->run_online); drop(c->run_offline);
        finish_job(c, f.job, 0);
      }
      progressed = true;
    }
    if (!c->gate_pending.empty()) process_gate_checks(c, false);
    // 2. a kernel found the gate closed: everything from it on was (or will be) skipped; rewind and clear the poison
    if (!c->awaiting_reset && skip != kNone) {
      while (!c->inflight.empty() && c->inflight.back().kseq >= skip) {
        InFlight f = c->inflight.back();
        c->inflight.pop_back();
        if (f.ev >= 0) c->done_ev_free.push_back(f.ev);
        if (f.op < f.job->next_op) f.job->next_op = f.op;
        if (f.kseq == skip) { c->rerun_job = f.job; c->rerun_op = f.op; }
        c->hold = true;                   // the bubble this launch was aimed at has no room left
        c->hold_seq = f.idle_seq;
      }
      c->outstanding_us = 0;
      for (const InFlight& f : c->inflight) c->outstanding_us += f.cost_us;
      for (KbTokens& t : c->tokens) t.clear();
      launch_reset_skip(c->I.stream, c->I.rec, c->mir, ++c->reset_epoch);
      c->awaiting_reset = true;
      progressed = true;
    }
    if (c->awaiting_reset) {
      if (mload(&c->mir->i_reset_ack) == c->reset_epoch) c->awaiting_reset = false;
      else { il.unlock(); cpu_relax(50); continue; }
    }
    // 3. a new period: the grant replaces the balance
    const uint64_t pn = c->period_no.load(std::memory_order_acquire);
    // (the grant is already the per-instance share pool / m of Algorithm 1; every offline instance gets it)
    if (pn != c->last_period) {
      if (c->cfg.feedback) {      // the periods that went by feed the time account (one call per period, as the rule is stated)
        const uint64_t burst = 1000ull * std::max<uint64_t>(c->cfg.kernel_us_max, c->cfg.alg1.ul);
        const uint32_t share = c->share_ppm.load(std::memory_order_relaxed);
        for (uint64_t k = std::min<uint64_t>(pn - c->last_period, 64); k > 0; --k)
          c->conc_account_ns = sif_concurrent_account(c->conc_account_ns, share, (uint64_t)c->cfg.period_us * 1000ull, burst);
      }
      c->last_period = pn;
      c->period_grant = c->grant.load(std::memory_order_relaxed);
      for (KbTokens& t : c->tokens) t.new_period(c->period_grant);
    }
    if (c->hold && (!gated || mload(&c->mir->idle_seq) != c->hold_seq)) c->hold = false;
    // 4. admit jobs.  Two ways lead to the inference stream: into a bubble (Algorithm 1's tokens, the device gate
    // checks the bubble; closed after a skipped launch until the next bubble begins), and, with concurrent filling,
    // beside training against the time account (the device gate checks only the order of the launches).
    const bool feedback = gated && c->cfg.feedback != 0 && c->collocate.load(std::memory_order_relaxed);
    const bool into_bubbles = (c->collocate.load(std::memory_order_relaxed) && !c->hold) || !gated;
    if (into_bubbles || feedback) {
      {
        std::lock_guard<std::mutex> lk(c->mu);
        // Online pull-and-execute: requests are pulled one at a time, in arrival order, each only if the status is
        // idle and the predicted rest of the bubble, less what the requests already pulled still need, holds it.
        // With concurrent filling an online request need not wait for a bubble: outside one it is pulled as soon as the
        // time account is in credit, and its kernels are paid from that account one by one as they are released.
        const bool beside_ok = feedback && c->status.load(std::memory_order_relaxed) != SIF_STATUS_IDLE && c->conc_account_ns > 0;
        while ((into_bubbles || beside_ok) && !c->online_q.empty() && c->run_online.size() < 8) {
          Job* j = c->online_q.front();
          uint64_t pending = 0;
          for (const Job* q : c->run_online)
            for (size_t i = q->done_ops; i < q->plan.size(); ++i) pending += (uint64_t)(q->plan[i].cost_us * 1000.0);
          const uint64_t rest = predicted_remaining_ns(c);
          const uint64_t room = rest > pending ? rest - pending : 0;
          // Requests of the same instance that wait behind it may run with it as one kernel sequence (their rows back
          // to back, whatever their lengths): as many as are queued, fewer if the rest of the bubble does not hold them.
          const InferModel& im = *c->models[j->model];
          size_t n = 1;
          while (n < infer_coalesce(im.desc) && n < c->online_q.size() && c->online_q[n]->model == j->model) ++n;
          std::unique_ptr<Job> g;
          for (; n > 1; n = (n + 1) / 2) {
            g.reset(new Job());
            g->ticket = j->ticket; g->model = j->model; g->online = true; g->batch = 1; g->t_arrival_ns = j->t_arrival_ns;
            InferIO io[kMaxCoalesce];
            uint32_t longest = 0, rows = 0;
            for (size_t r = 0; r < n; ++r) {
              const Job* q = c->online_q[r];
              io[r].in_dev = q->in_dev; io[r].out_dev = q->out_dev; io[r].seq = q->seq;
              longest = std::max(longest, q->seq);
              rows += q->seq;
            }
            if (build_infer_plan(im, io, (uint32_t)n, 1, longest, c->cfg.kernel_us_max, g->plan) != SIF_OK) { g.reset(); continue; }
            g->seq = rows;                 // the calibrated costs scale with the rows the sequence covers
            g->parts.assign(c->online_q.begin(), c->online_q.begin() + (ptrdiff_t)n);
            apply_calibration(im, *g);
            if (!gated || beside_ok || sif_online_pull_ok(c->status.load(std::memory_order_relaxed), (uint32_t)c->online_q.size(), room, (uint64_t)(job_cost_us(g.get()) * 1000.0))) break;
            g.reset();
          }
          if (g) {
            for (size_t r = 0; r < n; ++r) { c->online_q.front()->plan.clear(); c->online_q.pop_front(); }
            c->run_online.push_back(g.get());
            c->groups.push_back(std::move(g));
            continue;
          }
          const uint64_t need = (uint64_t)(job_cost_us(j) * 1000.0);
          if (gated && !beside_ok && !sif_online_pull_ok(c->status.load(std::memory_order_relaxed), (uint32_t)c->online_q.size(), room, need)) break;
          c->online_q.pop_front();
          c->run_online.push_back(j);
        }
        // at most two jobs per offline instance are admitted at a time, so that no instance's backlog keeps another out
        for (size_t mdl = 0; mdl < c->offline_q.size(); ++mdl) {
          std::deque<Job*>& oq = c->offline_q[mdl];
          auto admitted = [&] { size_t n = 0; for (Job* q : c->run_offline) n += (size_t)q->model == mdl; return n; };
          while (!oq.empty() && admitted() < 2) {
            Job* j = oq.front();
            oq.pop_front();
            --c->offline_queued;
            // requests of equal shape that are queued behind it join it (never waited for)
            const InferModel& im = *c->models[j->model];
            std::vector<Job*> parts{j};
            while (parts.size() < infer_coalesce(im.desc) && !oq.empty()) {
              Job* n = oq.front();
              if (n->batch != j->batch || n->seq != j->seq) break;
              oq.pop_front();
              --c->offline_queued;
              parts.push_back(n);
            }
            if (parts.size() > 1) {
              std::unique_ptr<Job> g(new Job());
              g->ticket = j->ticket; g->model = j->model; g->batch = j->batch * (uint32_t)parts.size(); g->seq = j->seq;
              g->t_arrival_ns = j->t_arrival_ns;
              InferIO io[kMaxCoalesce];
              for (size_t r = 0; r < parts.size(); ++r) io[r] = InferIO{parts[r]->in_dev, parts[r]->out_dev};
              if (build_infer_plan(im, io, (uint32_t)parts.size(), j->batch, j->seq, c->cfg.kernel_us_max, g->plan) == SIF_OK) {
                g->parts = parts;
                apply_calibration(im, *g);
                for (Job* p : parts) p->plan.clear();
                c->run_offline.push_back(g.get());
                c->groups.push_back(std::move(g));
                continue;
              }
              for (size_t r = parts.size(); r-- > 1;) { oq.push_front(parts[r]); ++c->offline_queued; }      // could not be merged: one by one
            }
            c->run_offline.push_back(j);
          }
        }
      }
      // 5. release kernels
      const uint64_t max_ahead = gated ? c->cfg.alg1.ul : ~0ull;
      int budget = 64;
      while (budget-- > 0) {
        Job* j = nullptr;
        bool online = false, beside = false;
        // what the next kernel of a job is charged: its predicted microseconds, at most the largest possible grant
        auto cost_of = [&](const Job* q) { return (uint64_t)sif_kb_charge((uint64_t)(q->plan[q->next_op].cost_us + 0.999), c->cfg.alg1.ul, c->cfg.alg1.m); };
        if (into_bubbles || feedback)
          for (Job* q : c->run_online) if (q->next_op < q->plan.size()) { j = q; online = true; break; }
        // online kernels without tokens only while idle (and not after a skipped launch, until the next bubble begins);
        // otherwise, with concurrent filling, beside training against the time account
        if (j && gated && (!into_bubbles || c->status.load(std::memory_order_relaxed) != SIF_STATUS_IDLE)) {
          if (feedback && c->conc_account_ns >= 1000ull * cost_of(j)) beside = true;
          else j = nullptr;
        }
        if (!j) {
          // Offline: every instance spends its own balance, FIFO within the instance (its head kernel blocks the
          // rest of its queue); the instances take turns, and one that is out of tokens does not hold up the others.
          online = false;
          const size_t nm = c->tokens.size();
          for (size_t r = 0; r < nm && !j; ++r) {
            const size_t mdl = (c->rr_next + r) % nm;
            for (Job* q : c->run_offline) {
              if ((size_t)q->model != mdl || q->next_op >= q->plan.size()) continue;
              if (!gated || (into_bubbles && c->tokens[mdl].covers((uint32_t)cost_of(q)))) { j = q; c->rr_next = (mdl + 1) % nm; }   // token rule
              else if (feedback && c->conc_account_ns >= 1000ull * cost_of(q)) { j = q; beside = true; c->rr_next = (mdl + 1) % nm; }
              break;
            }
          }
        }
        if (!j) break;
        // The end of a bubble: a product that the predicted rest of the bubble does not hold any more, but whole
        // rounds of its tiles would, is cut in two along its rows (same bits); the first part goes out now.
        if (gated && !online && !beside && j->plan[j->next_op].row_split) {
          const Op& whole = j->plan[j->next_op];
          // what is in flight takes its predicted time plus the gap between dependent kernels of a stream, each
          // (less what the kernel at the head has already run)
          const uint64_t rest_ns = predicted_remaining_ns(c), ahead_ns = c->outstanding_us * 1000ull + 5000ull * c->inflight.size() - head_elapsed_ns(c);
          if (rest_ns > ahead_ns) {
            const double avail_us = (double)(rest_ns - ahead_ns) / 1000.0 - 10.0;
            const uint32_t unit = gemm_round_rows(whole.gemm);
            // (a part is predicted a tenth longer than its share of the whole plus the fixed part of a launch, see
            // split_gemm_rows: the part is sized so that this prediction, not the bare share, fits what is left)
            const double per_unit = 1.1 * whole.cost_us * unit / (double)whole.gemm.m;
            if (whole.cost_us > avail_us && avail_us >= per_unit + 6.0) {
              const uint64_t rows_first = (uint64_t)((avail_us - 6.0) / per_unit) * unit;
              if (rows_first > 0 && rows_first < whole.gemm.m) {
                Op first, rest;
                split_gemm_rows(whole, (uint32_t)rows_first, first, rest);
                j->plan[j->next_op] = std::move(first);
                j->plan.insert(j->plan.begin() + (ptrdiff_t)j->next_op + 1, std::move(rest));
              }
            }
          }
        }
        Op& op = j->plan[j->next_op];
        const uint64_t cost = cost_of(j);
        if (gated && !kb_depth_ok(c->outstanding_us, cost, max_ahead, c->inflight.size())) break;   // bounded speculation depth
        // What the device gate is bound to refuse is not launched: behind what is in flight (its predicted time and the
        // gap after each kernel), this kernel would end after the predicted end of the bubble.  The gate still decides;
        // this spares launches whose empty blocks would pass through the CUs beside the training kernels that follow.
        if (gated && !beside && !kb_fits_bubble(predicted_remaining_ns(c), c->outstanding_us - head_elapsed_ns(c) / 1000ull, c->inflight.size(), op.cost_us)) break;
        const uint32_t id = (uint32_t)(((j->ticket & 0xFFF) << 16) | (j->next_op & 0xFFFF));
        KCtl k = make_ctl(c, c->I, kKindInfer, id, gated ? c->T.rec : nullptr, (uint32_t)c->ns_to_ticks((uint64_t)(op.cost_us * 1000.0)));
        const bool last_of_job = j->next_op + 1 == j->plan.size();
        if (last_of_job) k.flags |= 1u;
        if (beside) k.flags |= 2u;        // paid from the time account: starts whatever the training stream does
        // (with gate_spin_every the run of a launch that came back waits the default time, whatever its number)
        const bool rerun = c->rerun_job == j && c->rerun_op == j->next_op;
        if (rerun) c->rerun_job = nullptr;
        if (c->cfg.gate_spin_log2 && (c->cfg.gate_spin_every < 2 || (k.kseq % c->cfg.gate_spin_every == 0 && !rerun)))
          k.flags |= (std::min<uint32_t>(c->cfg.gate_spin_log2, 30u) + 1u) << 8;
        sif_status st = launch_op(c, op, c->I.stream, k);
        int32_t ev = -1;
        if (st == SIF_OK && last_of_job) {
          if (c->done_ev_free.empty()) {
            hipEvent_t e = nullptr;
            if (hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess) { c->done_ev.push_back(e); c->done_ev_free.push_back((int32_t)c->done_ev.size() - 1); }
          }
          if (c->done_ev_free.empty()) st = fail(SIF_E_DEVICE, "barrier: no completion event");
          else {
            ev = c->done_ev_free.back();
            c->done_ev_free.pop_back();
            const hipError_t e = hipEventRecord(c->done_ev[ev], c->I.stream);
            if (e != hipSuccess) { c->done_ev_free.push_back(ev); ev = -1; st = fail_hip(e, "barrier: hipEventRecord"); }
          }
        }
        if (st != SIF_OK) {
          auto drop = [&](std::deque<Job*>& q) { q.erase(std::remove(q.begin(), q.end(), j), q.end()); };
          drop(c->run_online); drop(c->run_offline);
          // launches of this job already in flight complete normally; forget them
          c->inflight.erase(std::remove_if(c->inflight.begin(), c->inflight.end(), [&](const InFlight& f) { return f.job == j; }), c->inflight.end());
          finish_job(c, j, st);
          break;
        }
        c->kernels_launched.fetch_add(1, std::memory_order_relaxed);
        if (c->inflight.empty()) c->head_since_ns = host_now_ns();
        c->inflight.push_back(InFlight{k.kseq, j, j->next_op, mload(&c->mir->idle_seq), cost, ev, gated && !beside});
        j->next_op++;
        c->outstanding_us += cost;
        const bool by_tokens = !beside && gated && !online;
        if (beside) c->conc_account_ns -= std::min<uint64_t>(c->conc_account_ns, 1000ull * cost);
        else if (by_tokens) c->tokens[j->model].spend((uint32_t)cost);
        if (gated) {
          sif_release_rec& r = c->release_log[c->release_n++ % kReleaseLog];
          r.period = c->last_period; r.grant = c->period_grant;
          r.model = (uint32_t)j->model; r.charge = (uint32_t)cost; r.launch = k.kseq; r.kind = beside ? 2u : (online ? 1u : 0u);
        }
        progressed = true;
      }
    }
    il.unlock();
    if (!progressed) cpu_relax(100);
  }
}

// ------------------------------------------------------------------------------------------------ helpers
static sif_status run_step(sif_ctx* c, const void* inputs, const void* targets, float* loss) {
  TrainModel& tm = *c->train;
  tm.cur_inputs = inputs; tm.cur_targets = targets; tm.cur_loss = loss;
  hipStream_t s = c->T.stream;
  KCtl k0 = make_ctl(c, c->T, kKindStep, c->step_no, nullptr, 0);
  sif_status st = launch_step_marker(s, c->T.rec, c->mir, k0.slot, 0, k0.kind_id);
  if (st != SIF_OK) return st;
  tm.last_kseq.assign(tm.plan.size(), 0);
  for (size_t i = 0; i < tm.plan.size(); ++i) {
    Op& op = tm.plan[i];
    if (op.bubble_site >= 0) {
      const uint32_t seq = ++c->bubble_seq;
      KCtl kb = make_ctl(c, c->T, kKindBubble, (uint32_t)op.bubble_site, nullptr, 0);
      tm.last_kseq[i] = kb.kseq;
      if (op.dp_overlap) {
        // what is left of the bucketed gradient exchange: the device works it out from the end stamps of the
        // launches that finalized the buckets, and reports the length to the monitor thread
        c->bubble_ns[seq % kBubbleTable].store(kLenFromDevice, std::memory_order_release);
        DpBucketArgs ba{};
        ba.n = (uint32_t)tm.dp_buckets.size();
        uint64_t total = 0;
        for (uint32_t b = 0; b < ba.n; ++b) {
          ba.back[b] = kb.kseq - tm.last_kseq[tm.dp_buckets[b].ready_op];
          ba.ticks[b] = c->ns_to_ticks(tm.dp_buckets[b].dur_ns);
          total += ba.ticks[b];
        }
        st = launch_bubble_overlap(s, c->T.rec, c->mir, c->T.ring, kb.kseq, ba, seq, (uint32_t)op.bubble_site,
                                   4 * total + c->ns_to_ticks(100000000ull), c->cfg.device_timed_bubbles, kb.kind_id);
      } else {
        c->bubble_ns[seq % kBubbleTable].store(op.bubble_ns, std::memory_order_release);
        const uint64_t ticks = c->ns_to_ticks(op.bubble_ns);
        st = launch_bubble(s, c->T.rec, c->mir, kb.slot, seq, (uint32_t)op.bubble_site, ticks, 4 * ticks + c->ns_to_ticks(100000000ull),
                           c->cfg.device_timed_bubbles, kb.kind_id);
      }
    } else {
      const KCtl k = make_ctl(c, c->T, kKindTrain, (uint32_t)i, nullptr, 0);
      tm.last_kseq[i] = k.kseq;
      st = launch_op(c, op, s, k);
    }
    if (st != SIF_OK) return st;
  }
  KCtl k1 = make_ctl(c, c->T, kKindStep, c->step_no, nullptr, 0);
  ++c->step_no;
  return launch_step_marker(s, c->T.rec, c->mir, k1.slot, 1, k1.kind_id);
}

static uint64_t workspace_layout(uint64_t* rec_t, uint64_t* rec_i, uint64_t* ring_t, uint64_t* ring_i) {
  uint64_t off = 0;
  auto take = [&](uint64_t b) { off = (off + 255) & ~uint64_t(255); uint64_t o = off; off += b; return o; };
  uint64_t a = take(sizeof(StreamRec)), b = take(sizeof(StreamRec)), r1 = take((uint64_t)kRingSlots * sizeof(Slot)), r2 = take((uint64_t)kRingSlots * sizeof(Slot));
  if (rec_t) { *rec_t = a; *rec_i = b; *ring_t = r1; *ring_i = r2; }
  return off;
}

#define HIPCHK(call, what) do { hipError_t e_ = (call); if (e_ != hipSuccess) return fail_hip(e_, what); } while (0)

// ------------------------------------------------------------------------------------------------ C ABI
extern "C" {

uint64_t sif_now_ns(void) { return host_now_ns(); }

sif_status sif_default_config(sif_config* cfg) {
  if (!cfg) return fail(SIF_E_INVAL, "default_config: null");
  memset(cfg, 0, sizeof(*cfg));
  cfg->struct_size = sizeof(*cfg);
  cfg->period_us = 5; cfg->window = 64; cfg->count_running = 1;
  cfg->alg1.alpha = 1; cfg->alg1.beta = 3; cfg->alg1.gamma_num = 2; cfg->alg1.gamma_den = 1; cfg->alg1.m = 1;
  cfg->alg1.t0 = 200; cfg->alg1.ll = 400; cfg->alg1.ul = 800;
  cfg->kernel_us_max = 300; cfg->collocate = 1; cfg->device_timed_bubbles = 0; cfg->device_capacity_bytes = 0;
  cfg->gate_spin_log2 = 0; cfg->gate_spin_every = 0;
  cfg->feedback = 0; cfg->feedback_eps_ppm = 20000; cfg->feedback_add_ppm = 20000; cfg->feedback_cap_ppm = 1000000;
  return SIF_OK;
}

uint64_t sif_ctx_workspace_bytes(void) { return workspace_layout(nullptr, nullptr, nullptr, nullptr); }

sif_status sif_create(const sif_config* cfg, void* train_stream, void* infer_stream, void* workspace_dev, uint64_t workspace_bytes, sif_ctx** out) {
  if (!cfg || !out || !workspace_dev) return fail(SIF_E_INVAL, "create: null argument");
  if (cfg->struct_size != sizeof(sif_config)) return fail(SIF_E_INVAL, "create: config struct_size mismatch");
  if (!train_stream || !infer_stream || train_stream == infer_stream) return fail(SIF_E_INVAL, "create: need two distinct streams");
  if (cfg->period_us == 0 || cfg->window == 0 || cfg->window > 1024) return fail(SIF_E_INVAL, "create: period_us > 0 and 1 <= window <= 1024");
  if (cfg->alg1.m == 0 || cfg->alg1.gamma_den == 0 || cfg->alg1.gamma_num == 0) return fail(SIF_E_INVAL, "create: alg1 m, gamma_num and gamma_den must be positive");
  if (cfg->alg1.alpha > cfg->alg1.beta || cfg->alg1.ll > cfg->alg1.ul) return fail(SIF_E_INVAL, "create: need alpha <= beta and LL <= UL");
  if (cfg->feedback_cap_ppm > 1000000) return fail(SIF_E_INVAL, "create: feedback_cap_ppm is a share, at most 1000000");
  if ((uintptr_t)workspace_dev & 255) return fail(SIF_E_INVAL, "create: workspace must be 256-byte aligned");
  if (workspace_bytes < sif_ctx_workspace_bytes()) return fail(SIF_E_NOMEM, "create: workspace too small");
  std::unique_ptr<sif_ctx> c(new sif_ctx());
  c->cfg = *cfg;
  c->collocate.store(cfg->collocate);
  HIPCHK(hipGetDevice(&c->device), "hipGetDevice");
  int khz = 0;
  HIPCHK(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, c->device), "wall clock rate");
  if (khz <= 0) return fail(SIF_E_DEVICE, "create: device reports no wall clock rate");
  c->tick_hz = (uint64_t)khz * 1000ull;
  size_t free_b = 0, total_b = 0;
  HIPCHK(hipMemGetInfo(&free_b, &total_b), "hipMemGetInfo");
  c->capacity = cfg->device_capacity_bytes ? cfg->device_capacity_bytes : (uint64_t)total_b;
  for (auto& b : c->bubble_ns) b.store(0);
  uint64_t o_rt, o_ri, o_gt, o_gi;
  workspace_layout(&o_rt, &o_ri, &o_gt, &o_gi);
  unsigned char* base = (unsigned char*)workspace_dev;
  c->T.stream = (hipStream_t)train_stream; c->I.stream = (hipStream_t)infer_stream;
  c->T.rec = (StreamRec*)(base + o_rt); c->I.rec = (StreamRec*)(base + o_ri);
  c->T.ring = (Slot*)(base + o_gt); c->I.ring = (Slot*)(base + o_gi);
  HIPCHK(hipMemset(workspace_dev, 0, sif_ctx_workspace_bytes()), "clear workspace");
  StreamRec init{};
  init.state = kStateBusy; init.skip_from = kNone;
  HIPCHK(hipMemcpy(c->T.rec, &init, sizeof(init), hipMemcpyHostToDevice), "init record");
  HIPCHK(hipMemcpy(c->I.rec, &init, sizeof(init), hipMemcpyHostToDevice), "init record");
  void* mp = nullptr;
  HIPCHK(hipHostMalloc(&mp, sizeof(Mirror), hipHostMallocCoherent), "hipHostMalloc mailbox");
  // whatever fails from here on gives the mailbox and the events back
  struct Undo {
    void* mp; sif_ctx* c; bool armed;
    ~Undo() { if (!armed) return; for (hipEvent_t e : c->done_ev) (void)hipEventDestroy(e); c->done_ev.clear(); (void)hipHostFree(mp); c->mir = nullptr; }
  } undo{mp, c.get(), true};
  memset(mp, 0, sizeof(Mirror));
  c->mir = (Mirror*)mp;
  c->mir->i_skip_from = kNone;
  for (int i = 0; i < 64; ++i) {
    hipEvent_t e = nullptr;
    HIPCHK(hipEventCreateWithFlags(&e, hipEventDisableTiming), "create: hipEventCreate");
    c->done_ev.push_back(e);
    c->done_ev_free.push_back(i);
  }
  c->release_log.assign(kReleaseLog, sif_release_rec{});
  HIPCHK(hipDeviceSynchronize(), "create: synchronize");
  // The two streams must be able to run concurrently: spin 300 us on the training stream and stamp the time on
  // the inference stream; the stamp has to fall inside the spin.
  {
    uint64_t* probe = (uint64_t*)c->I.ring;
    sif_status st = launch_probe(c->T.stream, c->I.stream, c->ns_to_ticks(300000), probe);
    if (st != SIF_OK) return st;
    uint64_t h[3] = {0, 0, 0};
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(h, probe, sizeof(h), hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemset(probe, 0, sizeof(h));
    if (e != hipSuccess) return fail_hip(e, "create: stream probe");
    if (!(h[2] > h[0] && h[2] < h[1]) && !cfg->allow_serial_streams) {
      return fail(SIF_E_AGAIN, "create: the two streams do not run concurrently (they share a hardware queue); pass another pair");
    }
  }
  undo.armed = false;
  sif_ctx* raw = c.release();
  raw->mon = std::thread(monitor_main, raw);
  raw->bar = std::thread(barrier_main, raw);
  *out = raw;
  return SIF_OK;
}

sif_status sif_destroy(sif_ctx* c) {
  if (!c) return fail(SIF_E_INVAL, "destroy: null");
  c->paused.store(true);
  c->stop.store(true);
  if (c->bar.joinable()) c->bar.join();
  if (c->mon.joinable()) c->mon.join();
  (void)hipSetDevice(c->device);
  hipError_t e1 = hipStreamSynchronize(c->T.stream), e2 = hipStreamSynchronize(c->I.stream);
  {
    std::lock_guard<std::mutex> lk(c->mu);
    for (auto& kv : c->jobs) if (kv.second->result == 1) kv.second->result = SIF_E_CANCELLED;
    c->cv.notify_all();
  }
  process_gate_checks(c, true);
  if (c->mir) (void)hipHostFree(c->mir);
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->done_ev) (void)hipEventDestroy(e);
  delete c;
  if (e1 != hipSuccess) return fail_hip(e1, "destroy: training stream");
  if (e2 != hipSuccess) return fail_hip(e2, "destroy: inference stream");
  return SIF_OK;
}

sif_status sif_set_collocate(sif_ctx* c, uint32_t on) {
  if (!c) return fail(SIF_E_INVAL, "set_collocate: null");
  c->collocate.store(on ? 1 : 0);
  return SIF_OK;
}

uint64_t sif_model_n_params(const sif_model_shape* s) { return s ? model_n_params(*s) : 0; }

uint64_t sif_train_workspace_bytes(const sif_train_desc* d) {
  if (!d || d->struct_size != sizeof(sif_train_desc)) return 0;
  TrainModel tm;
  tm.desc = *d;
  tm.desc.workspace_dev = nullptr;
  if (build_train_model(tm, nullptr) != SIF_OK) return 0;
  return tm.workspace_bytes;
}

sif_status sif_register_training_step(sif_ctx* c, const sif_train_desc* d, sif_handle* out) {
  if (!c || !d || !out) return fail(SIF_E_INVAL, "register_training_step: null argument");
  if (d->struct_size != sizeof(sif_train_desc)) return fail(SIF_E_INVAL, "register_training_step: struct_size mismatch");
  if (c->train) return fail(SIF_E_INVAL, "register_training_step: a training instance is already registered");
  if (!d->master_dev || !d->workspace_dev || ((uintptr_t)d->workspace_dev & 255) || ((uintptr_t)d->master_dev & 15)) return fail(SIF_E_INVAL, "register_training_step: master/workspace null or misaligned");
  const uint64_t need = sif_train_workspace_bytes(d);
  if (need == 0) return SIF_E_INVAL;      // text set by the builder
  if (d->workspace_bytes < need) return fail(SIF_E_NOMEM, "register_training_step: workspace too small: need %llu bytes", (unsigned long long)need);
  std::unique_ptr<TrainModel> tm(new TrainModel());
  tm->desc = *d;
  sif_status st = build_train_model(*tm, c->T.stream);
  if (st != SIF_OK) return st;
  HIPCHK(hipStreamSynchronize(c->T.stream), "register_training_step: synchronize");
  std::lock_guard<std::mutex> il(c->infer_mu);
  c->train = std::move(tm);
  *out = 0;
  return SIF_OK;
}

sif_status sif_run_training_step(sif_ctx* c, sif_handle h, const void* inputs_dev, const void* targets_dev, float* loss_dev) {
  if (!c || !c->train || h != 0) return fail(SIF_E_INVAL, "run_training_step: no such training instance");
  if (!inputs_dev || !targets_dev) return fail(SIF_E_INVAL, "run_training_step: null inputs or targets");
  return run_step(c, inputs_dev, targets_dev, loss_dev);
}

sif_status sif_sync_training(sif_ctx* c) {
  if (!c) return fail(SIF_E_INVAL, "sync_training: null");
  HIPCHK(hipStreamSynchronize(c->T.stream), "sync_training");
  return SIF_OK;
}

sif_status sif_train_tensor(sif_ctx* c, sif_handle h, const char* name, int32_t layer, void** ptr_dev, uint64_t* elems) {
  if (!c || !c->train || h != 0 || !name || !ptr_dev) return fail(SIF_E_INVAL, "train_tensor: bad argument");
  std::string key = name;
  auto it = c->train->tensors.find(key);
  if (it == c->train->tensors.end()) it = c->train->tensors.find(key + "." + std::to_string(layer));
  if (it == c->train->tensors.end()) return fail(SIF_E_INVAL, "train_tensor: unknown tensor '%s'", name);
  *ptr_dev = it->second.ptr;
  if (elems) *elems = it->second.elems;
  return SIF_OK;
}

sif_status sif_train_dp_bucket(sif_ctx* c, sif_handle h, uint32_t index, uint64_t* bytes, uint32_t* ready_launch) {
  if (!c || !c->train || h != 0 || !bytes || !ready_launch) return fail(SIF_E_INVAL, "train_dp_bucket: bad handle or null output");
  if (index >= c->train->dp_buckets.size()) return fail(SIF_E_INVAL, "train_dp_bucket: the step has %zu buckets", c->train->dp_buckets.size());
  *bytes = c->train->dp_buckets[index].bytes;
  *ready_launch = c->train->dp_buckets[index].ready_op;
  return SIF_OK;
}

const char* sif_train_op_name(sif_ctx* c, sif_handle h, uint32_t index) {
  if (!c || !c->train || h != 0 || index >= c->train->plan.size()) return nullptr;
  return c->train->plan[index].name;
}

uint64_t sif_infer_workspace_bytes(const sif_infer_desc* d) {
  if (!d || d->struct_size != sizeof(sif_infer_desc)) return 0;
  return infer_workspace_bytes(*d);
}

sif_status sif_register_inference_model(sif_ctx* c, const sif_infer_desc* d, sif_handle* out) {
  if (!c || !d || !out) return fail(SIF_E_INVAL, "register_inference_model: null argument");
  if (d->struct_size != sizeof(sif_infer_desc)) return fail(SIF_E_INVAL, "register_inference_model: struct_size mismatch");
  if (!d->master_dev || !d->workspace_dev || ((uintptr_t)d->workspace_dev & 255) || ((uintptr_t)d->master_dev & 15)) return fail(SIF_E_INVAL, "register_inference_model: master/workspace null or misaligned");
  // Principle-I: the peaks of all collocated instances must sum below the device capacity
  std::vector<uint64_t> peaks;
  if (c->train) peaks.push_back(c->train->workspace_bytes + c->train->n_params * 4);
  for (auto& m : c->models) peaks.push_back(m->desc.peak_bytes);
  peaks.push_back(d->peak_bytes);
  if (!sif_principle_1(peaks.data(), (uint32_t)peaks.size(), c->capacity)) return fail(SIF_E_NOMEM, "register_inference_model: collocated peaks exceed the device capacity");
  std::unique_ptr<InferModel> im(new InferModel());
  im->desc = *d;
  std::lock_guard<std::mutex> il(c->infer_mu);
  sif_status st = build_infer_model(*im, c->I.stream);
  if (st != SIF_OK) return st;
  HIPCHK(hipStreamSynchronize(c->I.stream), "register_inference_model: synchronize");
  c->models.push_back(std::move(im));
  {
    std::lock_guard<std::mutex> lk(c->mu);
    c->offline_q.emplace_back();
    c->tokens.emplace_back();
  }
  *out = (sif_handle)(c->models.size() - 1);
  return SIF_OK;
}

static void apply_calibration(const InferModel& im, Job& j) {
  const size_t n = j.parts.empty() ? 1 : j.parts.size();
  if (n > im.calib_cost_us_n.size() || im.calib_batch == 0) return;
  const std::vector<double>& cal = im.calib_cost_us_n[n - 1];
  if (cal.size() != j.plan.size()) return;
  // rows this job covers against the rows the calibration run of n requests covered (a coalesced offline job carries
  // n times the batch, one of online requests of different lengths its total row count in seq with batch 1)
  const double scale = ((double)j.batch * (j.seq ? j.seq : 1)) / ((double)im.calib_batch * n * (im.calib_seq ? im.calib_seq : 1));
  for (size_t i = 0; i < j.plan.size(); ++i) {
    const double base = cal[i];
    j.plan[i].cost_us = std::max(1.0, 2.0 + (base - 2.0) * scale);
  }
}

static sif_status submit(sif_ctx* c, sif_handle model, const void* in_dev, void* out_dev, uint32_t batch, uint32_t seq, bool online,
                         uint64_t t_arrival_ns, sif_ticket* out) {
  if (!c || !out) return fail(SIF_E_INVAL, "submit: null argument");
  if (model < 0 || (size_t)model >= c->models.size()) return fail(SIF_E_INVAL, "submit: no such model");
  InferModel& im = *c->models[model];
  if ((im.desc.online != 0) != online) return fail(SIF_E_INVAL, "submit: model was registered for the other mode");
  std::unique_ptr<Job> j(new Job());
  j->model = model; j->online = online; j->batch = batch; j->seq = im.desc.shape.kind == SIF_MODEL_MLP ? 1 : seq;
  j->t_arrival_ns = t_arrival_ns ? t_arrival_ns : host_now_ns();
  j->in_dev = in_dev; j->out_dev = out_dev;
  const InferIO io{in_dev, out_dev};
  sif_status st = build_infer_plan(im, &io, 1, batch, seq, c->cfg.kernel_us_max, j->plan);
  if (st != SIF_OK) return st;
  apply_calibration(im, *j);
  std::lock_guard<std::mutex> lk(c->mu);
  if (c->offline_queued + c->online_q.size() >= 4096) return fail(SIF_E_AGAIN, "submit: queue full");
  j->ticket = c->next_ticket++;
  *out = j->ticket;
  if (online) c->online_q.push_back(j.get());
  else { c->offline_q[model].push_back(j.get()); ++c->offline_queued; }
  c->jobs[j->ticket] = std::move(j);
  return SIF_OK;
}

sif_status sif_submit_offline_batch(sif_ctx* c, sif_handle model, const void* in_dev, void* out_dev, uint32_t batch, uint32_t seq, sif_ticket* out) {
  return submit(c, model, in_dev, out_dev, batch, seq, false, 0, out);
}

sif_status sif_submit_online_request(sif_ctx* c, sif_handle model, const void* in_dev, void* out_dev, uint32_t seq, uint64_t t_arrival_ns, sif_ticket* out) {
  return submit(c, model, in_dev, out_dev, 1, seq, true, t_arrival_ns, out);
}

sif_status sif_wait(sif_ctx* c, sif_ticket t, uint64_t timeout_ns) {
  if (!c) return fail(SIF_E_INVAL, "wait: null");
  std::unique_lock<std::mutex> lk(c->mu);
  auto it = c->jobs.find(t);
  if (it == c->jobs.end()) return fail(SIF_E_INVAL, "wait: unknown ticket");
  Job* j = it->second.get();
  const bool ok = c->cv.wait_for(lk, std::chrono::nanoseconds(timeout_ns), [&] { return j->result != 1; });
  if (!ok) return fail(SIF_E_TIMEOUT, "wait: ticket %llu still pending", (unsigned long long)t);
  const int32_t r = j->result;
  c->jobs.erase(it);
  if (r < 0) return fail(r, "wait: job failed or was cancelled");
  return SIF_OK;
}

sif_status sif_calibrate(sif_ctx* c, uint32_t iters, const void* train_inputs_dev, const void* train_targets_dev) {
  if (!c || iters == 0) return fail(SIF_E_INVAL, "calibrate: null context or zero iterations");
  c->paused.store(true, std::memory_order_release);
  std::unique_lock<std::mutex> il(c->infer_mu);
  struct Unpause { sif_ctx* c; ~Unpause() { c->paused.store(false, std::memory_order_release); } } unpause{c};
  HIPCHK(hipStreamSynchronize(c->I.stream), "calibrate: synchronize");
  sif_status result = SIF_OK;
  if (c->train && train_inputs_dev && train_targets_dev) {
    sif_status st = run_step(c, train_inputs_dev, train_targets_dev, nullptr);
    if (st != SIF_OK) return st;
    HIPCHK(hipStreamSynchronize(c->T.stream), "calibrate: synchronize");
    // A pipeline stage whose per-micro-batch times were not given: take them from the step just run (first to last
    // kernel of micro-batch 0's forward and backward pass) and size the schedule's idle intervals from them.
    if (c->train->desc.par_mode == SIF_PAR_PP && c->train->pp_times_estimated) {
      TrainModel& tm = *c->train;
      std::vector<Slot> ring(kRingSlots);
      HIPCHK(hipMemcpy(ring.data(), c->T.ring, (size_t)kRingSlots * sizeof(Slot), hipMemcpyDeviceToHost), "calibrate: read the trace");
      uint64_t lo[2] = {~0ull, ~0ull}, hi[2] = {0, 0};
      for (size_t i = 0; i < tm.plan.size(); ++i) {
        const int32_t pass = tm.plan[i].pp_pass;
        if (pass != 0 && pass != 1) continue;
        const Slot& sl = ring[tm.last_kseq[i] % kRingSlots];
        lo[pass] = std::min(lo[pass], sl.t0); hi[pass] = std::max(hi[pass], sl.t1);
      }
      if (hi[0] > lo[0] && hi[1] > lo[1]) {
        const uint64_t tf = c->ticks_to_ns(hi[0] - lo[0]), tb = c->ticks_to_ns(hi[1] - lo[1]);
        int32_t kind[64], index[64];
        uint64_t gap[64];
        const int32_t ng = sif_pp_1f1b_bubbles(tm.desc.pp_stage, tm.desc.pp_stages, tm.desc.pp_micro, tf, tb, kind, index, gap, 64);
        if (ng > 0 && ng <= 64) {
          tm.max_bubble_ns = 0;
          for (Op& op : tm.plan) {
            if (op.bubble_site < 0 || op.pp_kind < 0) continue;
            for (int32_t g = 0; g < ng; ++g)
              if (kind[g] == op.pp_kind && (op.pp_kind == 2 || index[g] == op.pp_index)) { op.bubble_ns = gap[g]; op.cost_us = gap[g] / 1000.0; }
            tm.max_bubble_ns = std::max(tm.max_bubble_ns, op.bubble_ns);
          }
          tm.pp_times_estimated = false;
          st = run_step(c, train_inputs_dev, train_targets_dev, nullptr);      // once with the new intervals before timing
          if (st != SIF_OK) return st;
          HIPCHK(hipStreamSynchronize(c->T.stream), "calibrate: synchronize");
        }
      }
    }
    // the solo iteration time: the shortest of `iters` steps, each measured on the device between its two markers
    // (the first step after a pause of the stream tends to run long, which a mean over few steps would carry)
    uint64_t best = ~0ull;
    for (uint32_t i = 0; i < iters; ++i) {
      st = run_step(c, train_inputs_dev, train_targets_dev, nullptr);
      if (st != SIF_OK) return st;
      HIPCHK(hipStreamSynchronize(c->T.stream), "calibrate: synchronize");
      best = std::min(best, mload(&c->mir->step_ticks_last));
    }
    __atomic_store_n(&c->step_solo_ns, c->ticks_to_ns(best), __ATOMIC_RELAXED);
    // a bubble whose length the device decides: keep what the last solo step showed as its predicted length
    for (size_t i = 0; i < c->train->plan.size(); ++i) {
      Op& op = c->train->plan[i];
      if (!op.dp_overlap) continue;
      Slot sl;
      HIPCHK(hipMemcpy(&sl, c->T.ring + (c->train->last_kseq[i] % kRingSlots), sizeof(Slot), hipMemcpyDeviceToHost), "calibrate: read slot");
      op.bubble_ns = c->ticks_to_ns(sl.t1 - sl.t0);
      op.cost_us = op.bubble_ns / 1000.0;
      c->train->max_bubble_ns = op.bubble_ns;
    }
  }
  for (auto& mp : c->models) {
    InferModel& im = *mp;
    const sif_model_shape& s = im.desc.shape;
    const uint32_t batch = im.desc.online ? 1 : s.batch;
    const uint32_t n_max = infer_coalesce(im.desc);
    im.calib_cost_us_n.assign(n_max, std::vector<double>());
    for (uint32_t n = 1; n <= n_max; ++n) {        // the plan of one request and of each number of coalesced requests
      Plan plan;
      InferIO io[kMaxCoalesce];
      const uint64_t rows1 = (uint64_t)batch * s.seq;
      for (uint32_t r = 0; r < n; ++r) {
        io[r].in_dev = (const unsigned char*)im.calib_in + (s.kind == SIF_MODEL_MLP ? 0 : r * rows1 * 4);
        io[r].out_dev = (unsigned char*)im.calib_out + (s.kind == SIF_MODEL_MLP ? 0 : r * rows1 * s.d_model * 2);
      }
      sif_status st = build_infer_plan(im, io, n, batch, s.seq, c->cfg.kernel_us_max, plan);
      if (st != SIF_OK) return st;
      std::vector<double> sum(plan.size(), 0.0);
      std::vector<uint32_t> kseqs(plan.size());
      for (uint32_t it = 0; it <= iters; ++it) {
        for (size_t i = 0; i < plan.size(); ++i) {
          KCtl k = make_ctl(c, c->I, kKindInfer, (uint32_t)i, nullptr, 0);
          kseqs[i] = k.kseq;
          st = plan[i].fn(c->I.stream, k);
          if (st != SIF_OK) return st;
        }
        HIPCHK(hipStreamSynchronize(c->I.stream), "calibrate: synchronize");
        if (it == 0) continue;       // warm-up
        for (size_t i = 0; i < plan.size(); ++i) {
          Slot sl;
          HIPCHK(hipMemcpy(&sl, c->I.ring + (kseqs[i] % kRingSlots), sizeof(Slot), hipMemcpyDeviceToHost), "calibrate: read slot");
          sum[i] += (double)c->ticks_to_ns(sl.t1 - sl.t0) / 1000.0;
        }
      }
      std::vector<double>& cal = im.calib_cost_us_n[n - 1];
      cal.resize(plan.size());
      for (size_t i = 0; i < plan.size(); ++i) cal[i] = std::max(1.0, sum[i] / iters + 2.0);
    }
    im.calib_cost_us = im.calib_cost_us_n[0];
    im.calib_total_us = 0;
    for (double v : im.calib_cost_us) im.calib_total_us += v;
    im.calib_batch = batch; im.calib_seq = s.kind == SIF_MODEL_MLP ? 1 : s.seq;
    if (im.desc.online && c->train && c->train->max_bubble_ns && !sif_principle_2((uint64_t)(im.calib_total_us * 1000.0), c->train->max_bubble_ns)) {
      fail(SIF_W_SLO_RISK, "calibrate: an online request (%.0f us) is longer than the longest bubble", im.calib_total_us);
      result = SIF_W_SLO_RISK;
    }
  }
  return result;
}

sif_status sif_poll_stats(sif_ctx* c, sif_stats* out) {
  if (!c || !out) return fail(SIF_E_INVAL, "poll_stats: null");
  if (out->struct_size != sizeof(sif_stats)) return fail(SIF_E_INVAL, "poll_stats: struct_size mismatch");
  const Mirror* m = c->mir;
  out->status_now = (uint32_t)c->status.load(); out->zc_now = c->zc.load(); out->tokens_now = c->grant.load();
  out->concurrent_share_ppm = c->share_ppm.load();
  out->steps = mload(&m->steps);
  out->step_ns_sum = c->ticks_to_ns(mload(&m->step_ticks_sum));
  out->step_ns_last = c->ticks_to_ns(mload(&m->step_ticks_last));
  out->step_solo_ns = c->step_solo_ns;
  out->bubble_ns = c->ticks_to_ns(mload(&m->bubble_ticks));
  out->filled_ns = c->ticks_to_ns(mload(&m->filled_ticks));
  out->infer_busy_ns = c->ticks_to_ns(mload(&m->infer_ticks));
  out->offline_samples = c->offline_samples.load(); out->offline_batches = c->offline_batches.load();
  out->online_done = c->online_done.load();
  out->kernels_launched = c->kernels_launched.load();
  out->kernels_skipped = mload(&m->kernels_skipped);
  out->kernels_run = mload(&m->kernels_run);
  out->train_kernels = (uint32_t)(mload(&m->t_completed) - c->train_kernels_base);
  out->gate_violations = c->gate_violations.load();
  out->gate_checked = c->gate_checked.load();
  out->gate_unchecked = c->gate_unchecked.load();
  out->gate_timeouts = mload(&m->gate_timeouts);
  out->periods = c->periods.load();
  // nearest-rank percentiles from the histogram (bucket middles: within 1/32 of the exact value); no lock is taken
  out->online_p50_ns = c->latency.percentile(0.50);
  out->online_p95_ns = c->latency.percentile(0.95);
  return SIF_OK;
}

sif_status sif_reset_stats(sif_ctx* c) {
  if (!c) return fail(SIF_E_INVAL, "reset_stats: null");
  c->paused.store(true, std::memory_order_release);
  std::unique_lock<std::mutex> il(c->infer_mu);
  struct Unpause { sif_ctx* c; ~Unpause() { c->paused.store(false, std::memory_order_release); } } unpause{c};
  HIPCHK(hipStreamSynchronize(c->T.stream), "reset_stats: training stream");
  HIPCHK(hipStreamSynchronize(c->I.stream), "reset_stats: inference stream");
  // zero the accumulators of both records (from `steps` up to the completion counters) and of the mailbox
  const size_t off = offsetof(StreamRec, steps), len = offsetof(StreamRec, done_top) - off;
  HIPCHK(hipMemset((unsigned char*)c->T.rec + off, 0, len), "reset_stats");
  HIPCHK(hipMemset((unsigned char*)c->I.rec + off, 0, len), "reset_stats");
  Mirror* m = c->mir;
  m->steps = m->step_ticks_sum = m->step_ticks_last = m->bubble_ticks = m->filled_ticks = m->infer_ticks = 0;
  m->kernels_run = m->kernels_skipped = 0;
  c->train_kernels_base = mload(&m->t_completed);
  process_gate_checks(c, true);               // both streams are idle: every pending start can be judged now
  c->offline_samples = 0; c->offline_batches = 0; c->online_done = 0; c->kernels_launched = 0; c->periods = 0;
  c->gate_violations = 0; c->gate_checked = 0; c->gate_unchecked = 0;
  m->gate_timeouts = 0;
  c->latency.clear();
  c->release_n = 0;
  return SIF_OK;
}

sif_status sif_profile_gemm(sif_ctx* c, uint32_t on) {
  if (!c) return fail(SIF_E_INVAL, "profile_gemm: null");
  if (on && c->prof_ev.empty()) {
    c->prof_ev.resize(2 * kProfMax);
    for (auto& e : c->prof_ev) HIPCHK(hipEventCreate(&e), "profile_gemm: hipEventCreate");
    c->prof_class.assign(kProfMax, -1);
    c->prof_flops.assign(kProfMax, 0.0);
    c->prof_kseq.assign(kProfMax, 0);
  }
  if (on) { c->prof_n.store(0); c->prof_third[0] = c->prof_third[1] = 0; }
  c->prof_on.store(on > 3 ? 1u : on);
  return SIF_OK;
}

sif_status sif_profile_read(sif_ctx* c, uint64_t launches[4], double flops[4], double seconds[4]) {
  if (!c || !launches || !flops || !seconds) return fail(SIF_E_INVAL, "profile_read: null");
  if (c->prof_on.load()) return fail(SIF_E_INVAL, "profile_read: switch profiling off first");
  HIPCHK(hipStreamSynchronize(c->T.stream), "profile_read: training stream");
  HIPCHK(hipStreamSynchronize(c->I.stream), "profile_read: inference stream");
  for (int i = 0; i < 4; ++i) { launches[i] = 0; flops[i] = 0; seconds[i] = 0; }
  const uint32_t n = std::min(c->prof_n.load(), kProfMax);
  // a launch the device gate skipped did no work: leave it out (its re-run is timed by itself)
  std::vector<Slot> ring(kRingSlots);
  HIPCHK(hipMemcpy(ring.data(), c->I.ring, (size_t)kRingSlots * sizeof(Slot), hipMemcpyDeviceToHost), "profile_read: copy ring");
  for (uint32_t i = 0; i < n; ++i) {
    if (c->prof_kseq[i] != 0) {
      const Slot& sl = ring[c->prof_kseq[i] % kRingSlots];
      if ((sl.decision >> 2) != c->prof_kseq[i] || (sl.decision & 3u) != 1u) continue;
    }
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]) != hipSuccess) continue;
    const int k = c->prof_class[i];
    if (k < 0 || k > 3) continue;
    launches[k] += 1; flops[k] += c->prof_flops[i]; seconds[k] += (double)ms * 1e-3;
  }
  return SIF_OK;
}

sif_status sif_read_trace(sif_ctx* c, uint32_t which, sif_trace_rec* out, uint32_t max, uint32_t* n) {
  if (!c || !n || which > 1 || (max && !out)) return fail(SIF_E_INVAL, "read_trace: bad argument");
  c->paused.store(true, std::memory_order_release);
  std::unique_lock<std::mutex> il(c->infer_mu);
  struct Unpause { sif_ctx* c; ~Unpause() { c->paused.store(false, std::memory_order_release); } } unpause{c};
  HIPCHK(hipStreamSynchronize(c->T.stream), "read_trace: training stream");
  HIPCHK(hipStreamSynchronize(c->I.stream), "read_trace: inference stream");
  StreamState& st = which == 0 ? c->T : c->I;
  const uint32_t launched = st.next_kseq - 1;
  uint32_t cnt = launched < kRingSlots - 1 ? launched : kRingSlots - 1;
  if (cnt > max) cnt = max;
  std::vector<Slot> ring(kRingSlots);
  HIPCHK(hipMemcpy(ring.data(), st.ring, (size_t)kRingSlots * sizeof(Slot), hipMemcpyDeviceToHost), "read_trace: copy ring");
  for (uint32_t i = 0; i < cnt; ++i) {
    const uint32_t kseq = launched - cnt + 1 + i;
    const Slot& s = ring[kseq % kRingSlots];
    out[i].kind = s.kind_id >> 28; out[i].id = s.kind_id & 0x0FFFFFFFu;
    out[i].decision = (out[i].kind == kKindTrain || out[i].kind == kKindInfer) ? (s.decision & 3u) : 1u;
    out[i].reserved = kseq;
    out[i].t0_ns = c->ticks_to_ns(s.t0); out[i].t1_ns = c->ticks_to_ns(s.t1);
  }
  *n = cnt;
  return SIF_OK;
}

sif_status sif_read_release_log(sif_ctx* c, sif_release_rec* out, uint32_t max, uint32_t* n) {
  if (!c || !n || (max && !out)) return fail(SIF_E_INVAL, "read_release_log: bad argument");
  c->paused.store(true, std::memory_order_release);
  std::unique_lock<std::mutex> il(c->infer_mu);
  struct Unpause { sif_ctx* c; ~Unpause() { c->paused.store(false, std::memory_order_release); } } unpause{c};
  const uint64_t have = std::min<uint64_t>(c->release_n, kReleaseLog);
  const uint32_t cnt = (uint32_t)std::min<uint64_t>(have, max);
  for (uint32_t i = 0; i < cnt; ++i) out[i] = c->release_log[(c->release_n - cnt + i) % kReleaseLog];
  *n = cnt;
  return SIF_OK;
}

sif_status sif_read_latency_histogram(sif_ctx* c, uint64_t* counts, uint32_t max, uint32_t* n) {
  if (!c || !n || (max && !counts)) return fail(SIF_E_INVAL, "read_latency_histogram: bad argument");
  const uint32_t cnt = std::min<uint32_t>(max, LatencyHist::kBuckets);
  for (uint32_t b = 0; b < cnt; ++b) counts[b] = c->latency.n[b].load(std::memory_order_relaxed);
  *n = cnt;
  return SIF_OK;
}

}  // extern "C"
