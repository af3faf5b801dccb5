// Marker kernels of the training stream: the modelled bubble (a timed wait that occupies one wavefront and no
// other compute resource), step begin/end stamps, and the poison reset of the inference stream.
//
// A bubble stands for the wait on a collective of the distributed training job (Sec. 2.1: communication leaves
// the GPU idle).  On entry the kernel stamps the time and then declares the stream idle; on exit it declares the
// stream busy and then stamps the time, so an inference kernel that saw "idle" before and after stamping its own
// start time started strictly inside the stamped interval.  The wait always ends: either the host releases it,
// or the device deadline passes.
#include "common.h"
#include "launch.h"
#include "runtime.h"

namespace sif {

// t0: when the stream went idle; ticks: how long the bubble lasts (device-timed) or is expected to last.
__device__ __forceinline__ void bubble_wait(StreamRec* rec, Mirror* mir, Slot* slot, uint32_t seq, uint32_t site, uint64_t t0, uint64_t ticks,
                                            uint64_t max_ticks, uint32_t device_timed, uint32_t kind_id) {
  st_agent(&rec->seq, seq);
  st_agent(&rec->site, site);
  st_agent(&rec->t_idle_begin, t0);
  st_agent(&rec->t_expected_end, t0 + ticks);
  st_agent(&rec->state, kStateIdle);
  // the bubble's own stamps for the host's check of inference kernel starts: entry cleared, then tagged
  st_sys(&mir->bub_end[seq % kBubbleStamps], (uint64_t)0);
  st_sys(&mir->bub_begin[seq % kBubbleStamps], t0);
  st_sys(&mir->bub_tag[seq % kBubbleStamps], seq);
  st_sys(&mir->idle_site, site);
  st_sys(&mir->idle_len_ticks, ticks);
  st_sys(&mir->idle_seq, seq);
  const uint64_t deadline = t0 + (device_timed ? ticks : max_ticks);
  while (now_ticks() < deadline) {
    if (!device_timed && ld_sys(&mir->release_seq) >= seq) break;
    __builtin_amdgcn_s_sleep(64);
  }
  st_agent(&rec->state, kStateBusy);
  const uint64_t t1 = now_ticks();
  st_agent(&rec->t_busy_begin, t1);
  st_sys(&mir->bub_end[seq % kBubbleStamps], t1);
  rec->bubble_ticks += t1 - t0;
  st_sys(&mir->bubble_ticks, rec->bubble_ticks);
  st_sys(&mir->busy_seq, seq);
  slot->kind_id = kind_id;
  slot->decision = 1;
  slot->t0 = t0;
  slot->t1 = t1;
}

__global__ __launch_bounds__(64) void bubble_kernel(StreamRec* rec, Mirror* mir, Slot* slot, uint32_t seq, uint32_t site,
                                                    uint64_t ticks, uint64_t max_ticks, uint32_t device_timed, uint32_t kind_id) {
  if (threadIdx.x != 0) return;
  bubble_wait(rec, mir, slot, seq, site, now_ticks(), ticks, max_ticks, device_timed, kind_id);
}

// The wait at the end of backward when the gradients are exchanged in buckets beside it.  Bucket k can be sent once
// the launch that finalized it has ended (its end stamp lies in the trace ring, `back[k]` launches before this
// one) and bucket k-1 has been sent, and takes ticks[k]; the stream idles for what is left of the exchange now.
// If the exchange is already over there is no bubble: the stream never goes idle and the record has zero length.
__global__ __launch_bounds__(64) void bubble_overlap_kernel(StreamRec* rec, Mirror* mir, Slot* ring, uint32_t kseq, DpBucketArgs b, uint32_t seq,
                                                            uint32_t site, uint64_t max_ticks, uint32_t device_timed, uint32_t kind_id) {
  if (threadIdx.x != 0) return;
  const uint64_t t0 = now_ticks();
  uint64_t finish = 0;
  for (uint32_t k = 0; k < b.n; ++k) {
    const uint64_t ready = ld_relaxed(&ring[(kseq - b.back[k]) % kRingSlots].t1);
    finish = (ready > finish ? ready : finish) + b.ticks[k];
  }
  Slot* slot = ring + (kseq % kRingSlots);
  if (finish <= t0) {
    slot->kind_id = kind_id;
    slot->decision = 1;
    slot->t0 = t0;
    slot->t1 = t0;
    return;
  }
  bubble_wait(rec, mir, slot, seq, site, t0, finish - t0, max_ticks, device_timed, kind_id);
}

__global__ __launch_bounds__(64) void step_marker_kernel(StreamRec* rec, Mirror* mir, Slot* slot, uint32_t end, uint32_t kind_id) {
  if (threadIdx.x != 0) return;
  const uint64_t t = now_ticks();
  if (!end) {
    rec->step_t0 = t;
    st_agent(&rec->state, kStateBusy);
    slot->kind_id = 0;      // the begin marker leaves no trace record of its own
    slot->decision = 0;
    slot->t0 = t;
    slot->t1 = t;
    return;
  }
  const uint64_t dt = t - rec->step_t0;
  rec->steps += 1;
  rec->step_ticks_sum += dt;
  rec->step_ticks_last = dt;
  st_sys(&mir->step_ticks_last, dt);
  st_sys(&mir->step_ticks_sum, rec->step_ticks_sum);
  st_sys(&mir->steps, rec->steps);
  slot->kind_id = kind_id;
  slot->decision = 1;
  slot->t0 = rec->step_t0;
  slot->t1 = t;
}

// Clears the poison of the inference stream after the host has taken note of the first skipped launch.
// It runs alone on the stream, so it also re-arms the completion counters: a launch some of whose blocks gave up
// waiting for the gate decision leaves them short of their full count.
__global__ __launch_bounds__(64) void reset_skip_kernel(StreamRec* rec, Mirror* mir, uint32_t epoch) {
  st_relaxed(&rec->done_sub[threadIdx.x * 32u], 0u);
  if (threadIdx.x < 8) st_relaxed(&rec->tile_next[threadIdx.x * 32u], 0u);
  __syncthreads();
  if (threadIdx.x != 0) return;
  st_relaxed(&rec->done_top, 0u);
  st_agent(&rec->skip_from, kNone);
  st_sys(&mir->i_skip_from, kNone);
  st_sys(&mir->i_reset_ack, epoch);
}

// Probe pair used once at context creation: does a kernel on the inference stream run while the training stream
// is occupied?  (Two HIP streams can share one hardware queue, which would serialise them.)
__global__ __launch_bounds__(64) void probe_spin_kernel(uint64_t ticks, uint64_t* out) {
  if (threadIdx.x != 0) return;
  const uint64_t t0 = now_ticks();
  while (now_ticks() - t0 < ticks) __builtin_amdgcn_s_sleep(32);
  out[0] = t0;
  out[1] = now_ticks();
}
__global__ __launch_bounds__(64) void probe_stamp_kernel(uint64_t* out) {
  if (threadIdx.x == 0) out[2] = now_ticks();
}

sif_status launch_probe(hipStream_t spin_stream, hipStream_t stamp_stream, uint64_t ticks, uint64_t* out) {
  hipLaunchKernelGGL(probe_spin_kernel, dim3(1), dim3(64), 0, spin_stream, ticks, out);
  sif_status st = check_launch("probe_spin");
  if (st != SIF_OK) return st;
  hipLaunchKernelGGL(probe_stamp_kernel, dim3(1), dim3(64), 0, stamp_stream, out);
  return check_launch("probe_stamp");
}

sif_status launch_bubble(hipStream_t s, StreamRec* rec, Mirror* mir, Slot* slot, uint32_t seq, uint32_t site, uint64_t ticks,
                         uint64_t max_ticks, uint32_t device_timed, uint32_t kind_id) {
  hipLaunchKernelGGL(bubble_kernel, dim3(1), dim3(64), 0, s, rec, mir, slot, seq, site, ticks, max_ticks, device_timed, kind_id);
  return check_launch("bubble");
}

sif_status launch_bubble_overlap(hipStream_t s, StreamRec* rec, Mirror* mir, Slot* ring, uint32_t kseq, const DpBucketArgs& b, uint32_t seq,
                                 uint32_t site, uint64_t max_ticks, uint32_t device_timed, uint32_t kind_id) {
  if (b.n == 0 || b.n > kMaxDpBuckets) return fail(SIF_E_INVAL, "bubble: bucket count out of range");
  for (uint32_t k = 0; k < b.n; ++k)
    if (b.back[k] == 0 || b.back[k] >= kRingSlots || b.back[k] >= kseq) return fail(SIF_E_INVAL, "bubble: a bucket's producer lies outside the trace ring");
  hipLaunchKernelGGL(bubble_overlap_kernel, dim3(1), dim3(64), 0, s, rec, mir, ring, kseq, b, seq, site, max_ticks, device_timed, kind_id);
  return check_launch("bubble_overlap");
}

sif_status launch_step_marker(hipStream_t s, StreamRec* rec, Mirror* mir, Slot* slot, uint32_t end, uint32_t kind_id) {
  hipLaunchKernelGGL(step_marker_kernel, dim3(1), dim3(64), 0, s, rec, mir, slot, end, kind_id);
  return check_launch("step_marker");
}

sif_status launch_reset_skip(hipStream_t s, StreamRec* rec, Mirror* mir, uint32_t epoch) {
  hipLaunchKernelGGL(reset_skip_kernel, dim3(1), dim3(64), 0, s, rec, mir, epoch);
  return check_launch("reset_skip");
}

}  // namespace sif
