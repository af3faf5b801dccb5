// Device-side activity monitor: the record every hot-path kernel keeps up to date in HBM, the per-launch trace
// slot, and the pinned host mailbox the monitor and barrier threads read.
//
// Role in the method (Sec. 3.3): the paper's monitoring library counts the kernels a training instance issues
// and its Kernel Barrier blocks or forwards each inference kernel at the CPU launch site.  Here the count is
// kept by a prologue/epilogue inside each kernel, and an inference kernel that was launched speculatively
// re-checks the training stream's state on the device before it does any work: the first block of the launch
// decides (run or skip), publishes the decision, and every other block follows it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sif {

constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr uint32_t kRingSlots = 1u << 16;   // trace slots per stream
constexpr uint32_t kStateIdle = 0, kStateBusy = 1;
enum : uint32_t { kKindTrain = 1, kKindInfer = 2, kKindBubble = 3, kKindStep = 4 };

struct alignas(128) StreamRec {     // one per stream, in HBM
  uint32_t state;                   // training stream: kStateBusy / kStateIdle (inside a bubble)
  uint32_t seq;                     // number of the current / last bubble (state and seq: one aligned 64-bit word)
  uint32_t site;                    // its site in the step
  uint32_t launched;                // kernels started on this stream
  uint32_t completed;               // kernels finished
  uint32_t skip_from;               // inference stream: first skipped launch (poison), kNone if clear
  uint32_t pad0, pad1;
  uint64_t t_start, t_end;          // last kernel start / end (device wall clock ticks)
  uint64_t t_idle_begin;            // start of the current / last bubble
  uint64_t t_busy_begin;            // end of the last finished bubble
  uint64_t t_expected_end;          // predicted end of the current bubble
  uint64_t step_t0;
  // accumulators (ticks / counts), mirrored to the host mailbox by whoever updates them
  uint64_t steps, step_ticks_sum, step_ticks_last;
  uint64_t bubble_ticks, filled_ticks, infer_ticks;
  uint64_t kernels_run, kernels_skipped, train_kernels;
  // completion counters of the kernel currently running on this stream (see kernel_end)
  uint32_t done_top;
  alignas(128) uint32_t done_sub[64 * 32];
  // work counters of the kernel currently running on this stream (kernels that hand out their tiles dynamically: one
  // counter per XCD, each on a cache line of its own); zero between kernels, re-armed like the completion counters
  alignas(128) uint32_t tile_next[8 * 32];
};

struct alignas(32) Slot {           // one per launch, ring indexed by launch number
  uint32_t pad0, pad1;
  uint32_t decision;                // (launch number << 2) | 1 run | 2 skip
  uint32_t kind_id;                 // (kind << 28) | id
  uint64_t t0, t1;
};

struct Mirror {                     // pinned, coherent host memory
  // device -> host
  uint32_t t_launched, t_completed;
  uint32_t idle_seq, busy_seq, idle_site, pad0;
  uint32_t i_done, i_skip_from, i_reset_ack, gate_timeouts;
  uint64_t steps, step_ticks_sum, step_ticks_last;
  uint64_t bubble_ticks, filled_ticks, infer_ticks;
  uint64_t kernels_run, kernels_skipped, train_kernels;
  // host -> device
  uint32_t release_seq, pad2;
  // device -> host: length of the bubble announced by idle_seq, where the device decides it (written before idle_seq)
  uint64_t idle_len_ticks;
  // device -> host, for the check of "an inference kernel starts only inside a detected bubble" (the barrier thread
  // makes it when a kernel completes).  Bubble b (numbered from 1) stamps its begin and end, on the device clock, into
  // entry b % kBubbleStamps; bub_tag says which bubble an entry belongs to and bub_end is 0 until that bubble is over.
  // A gated inference kernel that runs leaves one word in i_gate[launch number % kGateStamps]:
  //   bits 63..24 its start time (low 40 bits), 23..8 its launch number (low 16 bits), 7..0 the number of the bubble
  //   the gate saw (low 8 bits)
  // - one store, so the host never sees half of it.
  uint64_t bub_begin[64], bub_end[64];
  uint32_t bub_tag[64];
  uint64_t i_gate[1024];
};
constexpr uint32_t kBubbleStamps = 64, kGateStamps = 1024;

struct KCtl {                       // by-value kernel argument
  StreamRec* rec;                   // this stream's record; nullptr = unmonitored launch
  Mirror* mir;
  Slot* slot;
  const StreamRec* gate;            // training record an inference kernel is gated on, or nullptr
  uint32_t kseq;                    // launch number on this stream (>= 1)
  uint32_t cost_ticks;              // predicted duration
  uint32_t kind_id;
  uint32_t flags;                   // bit 0: last kernel of its job; bit 1: gated on the poison only (runs beside training);
                                    // bits 8..15: 0, or 1 + log2 of the bound on the spins a block waits for block 0's decision
};
constexpr uint32_t kDefaultSpinLog2 = 18;

__device__ __forceinline__ uint64_t now_ticks() { return wall_clock64(); }

template <typename T>
__device__ __forceinline__ T ld_agent(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void st_agent(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void st_sys(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}
// Relaxed agent-scope accesses: they bypass the per-XCD L2 for this one word but imply no cache write-back or
// invalidate (an acquire/release at agent scope costs a pass over the whole L2, too much to pay per block).
template <typename T>
__device__ __forceinline__ T ld_relaxed(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void st_relaxed(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void st_sys_relaxed(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
template <typename T>
__device__ __forceinline__ T ld_sys(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__device__ __forceinline__ uint32_t grid_blocks() { return gridDim.x * gridDim.y * gridDim.z; }
__device__ __forceinline__ bool first_thread() { return threadIdx.x == 0 && threadIdx.y == 0 && threadIdx.z == 0; }

// Decision of the first block of a gated launch: run only if no earlier launch of this speculation window was
// skipped, the training stream is inside a bubble, the predicted rest of the bubble holds this kernel, and
// the bubble is still the same one after the start time was stamped.
__device__ __forceinline__ bool gate_decide(const KCtl& c, uint64_t* t0, uint32_t* bubble) {
  // Relaxed device-scope loads (an acquire would sweep the L2 on every inference kernel start).  state and seq are
  // read as one 64-bit word; the three loads of the first round are independent and travel together, so the
  // decision costs two memory round trips: {state|seq, predicted end, poison} -> clock -> {state|seq} again.  A
  // predicted end that belongs to an older bubble than the state just read lies in the past and only makes the
  // decision conservative.
  const uint64_t* ss = reinterpret_cast<const uint64_t*>(&c.gate->state);
  const uint64_t s0 = ld_relaxed(ss);
  const uint64_t t_end = ld_relaxed(&c.gate->t_expected_end);
  const uint32_t poison = ld_relaxed(&c.rec->skip_from);
  if (c.flags & 2u) {               // concurrent filling: only the order within the speculation window is kept
    if (poison != kNone) return false;
    *t0 = now_ticks();
    return true;
  }
  if (poison != kNone || (uint32_t)s0 != kStateIdle) return false;
  const uint64_t t = now_ticks();
  if (t + c.cost_ticks > t_end) return false;
  if (ld_relaxed(ss) != s0) return false;
  *t0 = t;
  *bubble = (uint32_t)(s0 >> 32);
  return true;
}

// Kernel prologue.  Every thread calls it; returns false when the launch is skipped (the kernel must then do
// nothing but call kernel_end(c, false)).
//   * Block 0 of the grid stamps the start time and, for a gated launch, takes the decision and publishes it.
//   * The other blocks of a gated launch read the published decision (a load, no read-modify-write: same-address
//     atomics from thousands of blocks serialise at ~50 ns each).  Workgroups are dispatched in grid order, so
//     block 0 is resident whenever any block is and waits for nothing; should the decision still not appear
//     within the spin bound, the block poisons the window and skips, and the host re-runs the launch (every
//     inference kernel writes only buffers it does not read, so a partial run can be repeated).  A block that gave
//     up does not count itself in kernel_end, so a launch that block 0 then lets run never reaches its full count:
//     it is never reported done, and the kernel that clears the poison (it runs alone on the stream) re-arms the
//     completion counters it left behind.
//   * Blocks of an ungated launch never wait.
__device__ __forceinline__ uint32_t linear_block() { return blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z); }

__device__ __forceinline__ bool kernel_begin(const KCtl& c) {
  if (c.rec == nullptr) return true;
  __shared__ int s_run;
  if (first_thread()) {
    int run = 1;
    if (linear_block() == 0) {
      uint64_t t0 = now_ticks();
      uint32_t bubble = 0;
      if (c.gate != nullptr) run = gate_decide(c, &t0, &bubble) ? 1 : 0;
      c.slot->kind_id = c.kind_id;
      st_relaxed(&c.slot->t0, t0);
      if (run) {
        // what the host needs to check this start against the bubble's own stamps (not for launches beside training)
        if (c.gate != nullptr && !(c.flags & 2u))
          st_sys_relaxed(&c.mir->i_gate[c.kseq % kGateStamps], (t0 << 24) | ((uint64_t)(c.kseq & 0xFFFFu) << 8) | (bubble & 0xFFu));
        st_relaxed(&c.rec->t_start, t0);
        const uint32_t l = c.rec->launched + 1;
        st_relaxed(&c.rec->launched, l);
        if ((c.kind_id >> 28) == kKindTrain) st_sys_relaxed(&c.mir->t_launched, l);
      } else {
        c.slot->t1 = t0;
        if (ld_relaxed(&c.rec->skip_from) == kNone) {
          st_relaxed(&c.rec->skip_from, c.kseq);
          st_sys_relaxed(&c.mir->i_skip_from, c.kseq);
        }
        st_sys_relaxed(&c.mir->kernels_skipped, ++c.rec->kernels_skipped);
      }
      st_relaxed(&c.slot->decision, (c.kseq << 2) | (run ? 1u : 2u));
    } else if (c.gate != nullptr) {
      const uint32_t lg = (c.flags >> 8) & 0xFFu, bound = 1u << (lg ? (lg - 1u > 30u ? 30u : lg - 1u) : kDefaultSpinLog2);
      uint32_t d = 0, spins = 0;
      while (((d = ld_relaxed(&c.slot->decision)) >> 2) != c.kseq && ++spins < bound) __builtin_amdgcn_s_sleep(4);
      if ((d >> 2) == c.kseq) {
        run = (d & 3u) == 1u;
      } else {                           // block 0 never showed up: give the launch back to the host
        run = 0;
        if (ld_agent(&c.rec->skip_from) == kNone || ld_agent(&c.rec->skip_from) > c.kseq) {
          st_agent(&c.rec->skip_from, c.kseq);
          st_sys(&c.mir->i_skip_from, c.kseq);
        }
        st_sys(&c.mir->gate_timeouts, 1u);
      }
    }
    s_run = run;
  }
  __syncthreads();
  return s_run != 0;
}

// Kernel epilogue.  Every thread calls it after its last global store.  The last block of the grid to leave
// stamps the end time and bumps the counters.  "Last" is found with a two-level count (64 sub-counters on
// separate cache lines, then one top counter) so that no address sees more than blocks/64 + 64 atomics;
// kernels of one stream never overlap, so the counters belong to the stream and the last block re-arms them.
__device__ __forceinline__ void kernel_end(const KCtl& c, bool ran) {
  if (c.rec == nullptr || !ran) return;
  __syncthreads();
  if (!first_thread()) return;
  const uint32_t total = grid_blocks(), id = linear_block(), sub = id & 63u;
  const uint32_t in_sub = (total - sub + 63u) >> 6;
  uint32_t* cnt = c.rec->done_sub + sub * 32u;
  if (atomicAdd(cnt, 1u) + 1u != in_sub) return;
  *cnt = 0;
  const uint32_t subs = total < 64u ? total : 64u;
  if (atomicAdd(&c.rec->done_top, 1u) + 1u != subs) return;
  c.rec->done_top = 0;
#pragma unroll
  for (int x = 0; x < 8; ++x) st_relaxed(&c.rec->tile_next[x * 32], 0u);
  Mirror* m = c.mir;
  StreamRec* r = c.rec;
  const uint64_t t1 = now_ticks();
  const uint64_t t0 = ld_relaxed(&c.slot->t0);
  c.slot->t1 = t1;
  st_relaxed(&r->t_end, t1);
  const uint32_t done = r->completed + 1;
  st_relaxed(&r->completed, done);
  if ((c.kind_id >> 28) == kKindTrain) {
    st_sys_relaxed(&m->t_completed, done);          // also the count of training kernels run (the host takes differences)
  } else {
    uint64_t dur = t1 - t0, fill = dur;
    if (c.gate != nullptr) {
      const uint64_t ib = ld_relaxed(&c.gate->t_idle_begin);
      const uint64_t end = (ld_relaxed(&c.gate->state) == kStateIdle) ? t1 : ld_relaxed(&c.gate->t_busy_begin);
      const uint64_t lo = t0 > ib ? t0 : ib, hi = t1 < end ? t1 : end;
      fill = hi > lo ? hi - lo : 0;
    }
    r->infer_ticks += dur;
    r->filled_ticks += fill;
    ++r->kernels_run;
    // The statistics travel to the host mailbox with the last kernel of a job and with every eighth launch (each
    // store to host memory lengthens the end of the kernel); the progress word travels every time.  It says that the
    // last block is about to leave, not that the kernel's results are visible: the host reports a job done only after
    // an event recorded behind its last kernel has completed.
    if ((c.flags & 1u) || (c.kseq & 7u) == 0u) {
      st_sys_relaxed(&m->infer_ticks, r->infer_ticks);
      st_sys_relaxed(&m->filled_ticks, r->filled_ticks);
      st_sys_relaxed(&m->kernels_run, r->kernels_run);
    }
    st_sys_relaxed(&m->i_done, c.kseq);
  }
}

}  // namespace sif
