/*
 * specinf.h -- C ABI of libspecinf.so: the per-GPU hot path of SpecInF (speculative inference filling,
 * arxiv 2503.02550) on one MI355X (gfx950).
 *
 * One training instance runs its compute on a caller-supplied HIP stream; a Bubble Monitor counts its kernels
 * per period and reports the zero-count Z_c (Sec. 3.3 "Bubble Monitor"); Algorithm 1 turns Z_c into tokens
 * and a busy/idle status (Sec. 3.3 "CUDA Kernel Scheduler"); a Kernel Barrier forwards queued inference
 * kernels to a second stream while tokens last, or pulls online requests one by one while idle (Sec. 3.3
 * "Kernel Barrier").  Every kernel carries a prologue/epilogue that keeps a per-stream activity record in
 * HBM; inference kernels are launched speculatively and re-check that record on the device before they run.
 * Collective waits of the distributed training job are modelled as timed waits of the training stream.
 *
 * Conventions
 *   - All pointers named *_dev are device (HBM) addresses, all others are host addresses.
 *   - The caller owns every device buffer and both streams; the library borrows them from register/submit
 *     until the ticket completes or sif_destroy returns.  The library allocates only host control state and
 *     one small pinned host mailbox per context; nothing is allocated on the hot path.
 *   - Matrices are row-major.  Weights are stored [out_features, in_features].  bf16 = upper 16 bits of an
 *     IEEE binary32, rounded to nearest even; accumulation is fp32.
 *   - Every function returns a sif_status: 0 = SIF_OK, > 0 = warning (work was done), < 0 = error (nothing
 *     was done).  No function throws or aborts.  sif_last_error() gives the text of the last error of the
 *     calling thread.
 *   - Structs start with `struct_size` = sizeof(the struct) as the caller compiled it.
 */
#ifndef SPECINF_H
#define SPECINF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sif_ctx sif_ctx;
typedef int32_t sif_status;
typedef uint64_t sif_ticket;
typedef int32_t sif_handle;

enum {
  SIF_OK = 0,
  SIF_W_SLO_RISK = 1,   /* Principle-II violated: batch-1 request longer than the longest bubble */
  SIF_E_INVAL = -1,
  SIF_E_NOMEM = -2,     /* workspace too small, or Principle-I violated */
  SIF_E_AGAIN = -3,     /* queue full */
  SIF_E_CANCELLED = -4,
  SIF_E_TIMEOUT = -5,
  SIF_E_DEVICE = -6     /* a HIP call failed; text in sif_last_error() */
};

enum { SIF_F32 = 0, SIF_BF16 = 1 };
enum { SIF_STATUS_BUSY = 0, SIF_STATUS_IDLE = 1 };

const char* sif_last_error(void);
int32_t sif_abi_version(void);

/* ====================================================================================================
 * 1. Scheduler rules as pure host functions (no GPU needed).  The monitor thread calls sif_zero_count and
 *    sif_alg1_step once per period; the barrier thread takes the offline token decision with sif_kb_release (one
 *    kernel at a time, charged sif_kb_charge) and the online decision with sif_online_pull_ok.  Around the token
 *    rule the barrier applies rules of its own, none of them the paper's: a bound on the predicted time of
 *    forwarded but unfinished kernels, no launch that the device gate is bound to refuse, nothing after a skipped
 *    launch until the next bubble begins, and turns between several instances.  sif_sched_run_trace drives the
 *    monitor -> Algorithm 1 -> token chain, the very objects the threads keep, over a recorded trace.
 * ==================================================================================================== */

/* Constants of Algorithm 1 (inputs alpha, beta, gamma, m, UL, LL of the listing) plus the seed t0 that the
 * multiplicative update restarts from after the conservative phase.  Tokens are integers; one token is one
 * microsecond of predicted inference-kernel time.  gamma = gamma_num / gamma_den. */
typedef struct sif_alg1_params {
  uint32_t alpha, beta;
  uint32_t gamma_num, gamma_den;
  uint32_t m;
  uint32_t reserved;
  uint64_t ll, ul, t0;
} sif_alg1_params;

/* Bubble Monitor: number of consecutive zero counts ending at counts[n-1] (the newest sample). */
uint32_t sif_zero_count(const uint32_t* counts, uint32_t n);

/* Algorithm 1, one evaluation.  *pool is the per-GPU token state carried between periods (starts at 0);
 * *grant receives the tokens handed to each of the m instances, *status SIF_STATUS_BUSY / _IDLE.
 *   Z_c <= alpha         : pool = 0,                                       busy   (conservative)
 *   alpha < Z_c <= beta  : pool = min(LL, floor(max(pool,t0)*gamma)),      busy   (incremental)
 *   Z_c > beta           : pool = min(UL, floor(max(pool,t0)*gamma)),      idle   (stable)
 *   grant = floor(pool / m)
 * Returns SIF_E_INVAL for null pointers, m = 0 or gamma_den = 0. */
sif_status sif_alg1_step(const sif_alg1_params* p, uint32_t zc, uint64_t* pool, uint64_t* grant, int32_t* status);

/* Kernel Barrier, offline rule: with `balance` tokens, how many kernels from the head of the FIFO of costs
 * are forwarded (a kernel is forwarded iff balance >= cost, then balance -= cost; the head blocks the rest).
 * *balance_left may be null. */
uint32_t sif_kb_release(const uint32_t* costs, uint32_t n, uint64_t balance, uint64_t* balance_left);

/* What a kernel predicted to run predicted_us microseconds is charged: one token per microsecond, but never more
 * than the largest grant an instance can receive, floor(UL / m) (at least 1), so that the head of a queue can always
 * be forwarded in the stable phase (this build's reading: the paper says only "proportionate to its size"). */
uint32_t sif_kb_charge(uint64_t predicted_us, uint64_t ul, uint32_t m);

/* The chain Bubble Monitor -> Algorithm 1 -> offline Kernel Barrier (Sec. 3.3) over a trace, without a GPU: for each
 * of the n_periods per-period counts of training kernels the window of `window` entries gives Z_c, Algorithm 1 the
 * pool, grant and status, the grant replaces the balance of the one inference instance, and kernels are forwarded
 * from the head of the FIFO `costs` (tokens each) while the balance covers them.  Runs the same window and token
 * objects the monitor and barrier threads keep.  Per period t (null outputs are skipped): zc_out[t], pool_out[t],
 * grant_out[t], status_out[t], released_out[t] = kernels forwarded in that period. */
sif_status sif_sched_run_trace(const sif_alg1_params* p, uint32_t window, const uint32_t* counts, uint32_t n_periods,
                               const uint32_t* costs, uint32_t n_costs, uint32_t* zc_out, uint64_t* pool_out,
                               uint64_t* grant_out, int32_t* status_out, uint32_t* released_out);

/* The invariant "no inference kernel starts outside a detected bubble": 1 iff a kernel that started at t0 violated
 * it, given the interval [bubble_begin, bubble_end] of the bubble the device gate admitted it to (all three on the
 * device clock; bubble_end = 0: the bubble was not over yet when the check was made). */
int32_t sif_gate_violation(uint64_t t0, uint64_t bubble_begin, uint64_t bubble_end);

/* Latency histogram of the statistics: sixteen buckets per power of two (values below 16 ns one bucket each), so a
 * bucket is at most 1/16 wider than its lower edge.  sif_latency_bucket: the bucket a latency falls into;
 * sif_latency_bucket_lower_ns: a bucket's lower edge; sif_latency_buckets: how many there are. */
uint32_t sif_latency_bucket(uint64_t ns);
uint64_t sif_latency_bucket_lower_ns(uint32_t bucket);
uint32_t sif_latency_buckets(void);
/* Nearest-rank percentile (0 < p <= 1) of the values counted in counts[0..n_buckets): the rank-ceil(p * total) value's
 * bucket, reported as the middle of the values that bucket holds; 0 if nothing was counted. */
uint64_t sif_latency_percentile(const uint64_t* counts, uint32_t n_buckets, double p);

/* Kernel Barrier, online rule: 1 iff status is idle, a request waits and the predicted rest of the bubble
 * holds the predicted request time. */
int32_t sif_online_pull_ok(int32_t status, uint32_t queue_len, uint64_t predicted_remaining_ns,
                           uint64_t predicted_request_ns);

/* Collocation principles (Sec. 3.2).  1 = satisfied. */
int32_t sif_principle_1(const uint64_t* peak_bytes, uint32_t n, uint64_t capacity_bytes);
int32_t sif_principle_2(uint64_t min_exec_ns, uint64_t max_bubble_ns);

/* Bubble model: duration of a modelled collective, floor(bytes * 1e9 / bw). */
uint64_t sif_collective_ns(uint64_t n_bytes, uint64_t bw_bytes_per_s);

/* Idle intervals of one 1F1B pipeline stage (uniform per-micro-batch forward time tf and backward time tb,
 * n_micro >= n_stages).  Writes up to `max` entries: kind[i] 0 = gap before forward pass index[i],
 * 1 = gap before backward pass index[i], 2 = wait at the end of the step; ns[i] its length.
 * Returns the number of gaps (may exceed max; then only max were written), or a negative sif_status. */
int32_t sif_pp_1f1b_bubbles(uint32_t stage, uint32_t n_stages, uint32_t n_micro, uint64_t tf_ns, uint64_t tb_ns,
                            int32_t* kind, int32_t* index, uint64_t* ns, uint32_t max);

/* Data parallel with a bucketed gradient exchange that runs beside backward (a reading that goes beyond the single
 * exposed all-reduce; Sec. 2.1 names communication as the source of the idle time).  group_bytes[i] = gradient bytes
 * that become final together, in the order backward finalizes them.  A bucket is closed as soon as it holds at
 * least cap_bytes; what is open at the end is the last bucket.  Writes the bucket number of every group and returns
 * the number of buckets, or a negative sif_status (cap_bytes = 0, null array). */
int32_t sif_dp_gradient_buckets(const uint64_t* group_bytes, uint32_t n_groups, uint64_t cap_bytes,
                                uint32_t* bucket_of_group);

/* Exposed wait of that exchange: bucket k is sent once it is ready (ready_ns[k]) and bucket k-1 has been sent, and
 * takes dur_ns[k]; returns what is left of the exchange when backward ends at end_ns (0 if it is over by then). */
uint64_t sif_dp_overlapped_wait(const uint64_t* ready_ns, const uint64_t* dur_ns, uint32_t n, uint64_t end_ns);

/* Concurrent filling with feedback (Sec. 5.2: the outlook for pipeline parallelism is to run inference beside
 * training as much as possible until the Bubble Monitor sees the training iterations lengthen; the rule itself is
 * this library's reading).  share_ppm = the fraction of a busy period, in parts per million, during which an
 * inference kernel may run.  After an iteration of step_ns against the reference ref_ns: halved if
 * step_ns > ref_ns * (1 + eps), else raised by add_ppm up to cap_ppm. */
uint32_t sif_feedback_share(uint32_t share_ppm, uint64_t step_ns, uint64_t ref_ns, uint32_t eps_ppm, uint32_t add_ppm,
                            uint32_t cap_ppm);
/* The barrier's time account for the busy phases after one period: + period_ns * share, never above burst_ns.  A
 * kernel that Algorithm 1's tokens do not cover is forwarded iff the account holds its predicted time, which is
 * then taken off. */
uint64_t sif_concurrent_account(uint64_t balance_ns, uint32_t share_ppm, uint64_t period_ns, uint64_t burst_ns);

/* ====================================================================================================
 * 2. Single kernels (raw launchers).  Each enqueues one kernel on `stream` (a hipStream_t, may be null =
 *    default stream) and returns without synchronising.  Used by the model code below and by the parity
 *    tests.  All operand pointers are device addresses, 16-byte aligned; see each function for shapes.
 * ==================================================================================================== */

/* Operand layouts of the general matrix product  C[M,N] = alpha * sum_k A(m,k) B(k,n)  (+ epilogue). */
enum {
  SIF_A_ROW_K = 0,  /* A stored [M][K], lda = row stride      (activations in a forward product)        */
  SIF_A_ROW_M = 1   /* A stored [K][M], lda = row stride      (left operand of a weight gradient)       */
};
enum {
  SIF_B_ROW_K = 0,  /* B stored [N][K], ldb = row stride      (weights [out,in] in a forward product)   */
  SIF_B_ROW_N = 1   /* B stored [K][N], ldb = row stride      (weights in a data gradient, V in P*V)    */
};
enum {
  SIF_EPI_NONE = 0,
  SIF_EPI_BIAS = 1,        /* + bias[n]                                                        */
  SIF_EPI_GELU = 2,        /* C = GELU(acc + bias); if aux_dev != null also aux[m,n] = acc + bias (pre-activation) */
  SIF_EPI_RESIDUAL = 4,    /* + res[m,n] (same layout and dtype as C, ld = ldc)                        */
  SIF_EPI_GELU_GRAD = 8,   /* C = acc * GELU'(aux[m,n])  (aux bf16, ld = ldc)                          */
  SIF_EPI_OUT_F32 = 16,    /* C is fp32 instead of bf16                                                */
  SIF_EPI_CAUSAL_SKIP = 32 /* square per-batch problem: tiles strictly above the diagonal are not computed
                              nor written                                                             */
};

typedef struct sif_gemm_args {
  uint32_t struct_size;
  uint32_t a_layout, b_layout, epilogue;
  uint32_t m, n, k;            /* logical extents.  The extent along an operand's contiguous dimension may
                                  be ragged only if the row is padded (ld >= extent rounded up to 8) with
                                  zeros; ld must be a multiple of 8 elements.                          */
  uint32_t lda, ldb, ldc;      /* leading dimensions in elements; lda, ldb: multiples of 8, at most 4194304 */
  uint32_t batch_outer, batch_inner;             /* grid z = batch_outer * batch_inner (>= 1 each)     */
  int64_t a_stride_outer, a_stride_inner;        /* element offsets per batch index                    */
  int64_t b_stride_outer, b_stride_inner;
  int64_t c_stride_outer, c_stride_inner;
  float alpha;
  uint32_t k_causal;           /* 0 = full K.  1: contract only k <  row-tile end (lower-triangular A)
                                  2: contract only k >= column-tile start (A stored [K][M], upper part zero) */
  const void* a_dev;           /* bf16 */
  const void* b_dev;           /* bf16 */
  void* c_dev;                 /* bf16 or fp32 (SIF_EPI_OUT_F32)                                        */
  const void* bias_dev;        /* bf16 [N] or null                                                      */
  const void* res_dev;         /* residual, or null                                                     */
  void* aux_dev;               /* see SIF_EPI_GELU / SIF_EPI_GELU_GRAD                                  */
  uint32_t tile;               /* block tile edge: 0 = chosen from the shape, 128, or 256 (256: k a multiple of 64, no
                                  k_causal, no SIF_EPI_CAUSAL_SKIP).  The result has the same bits whichever is used. */
  uint32_t k_limit;            /* 0, or the whole K of a product that batch_inner cuts into slices of k along K (the
                                  operands' inner batch strides step along K, the results of the slices go to
                                  separate outputs): slice i then contracts only k_limit - i*k (at most k)
                                  elements, so the last slice may be shorter than the others (256-wide tiles: it
                                  too must be a multiple of 64) */
} sif_gemm_args;

/* bf16 matrix product on the MFMA units, fp32 accumulation. */
sif_status sif_k_gemm_bf16(const sif_gemm_args* a, void* stream);

/* Several bf16 products as ONE launch of 128 x 128 tiles (Sec. 2.1: the weight gradients of a transformer layer, each
 * with too few output tiles for the chip by itself).  list[0..n): n <= 16 products, all with A stored [K][M] and B
 * stored [K][N] (a_layout = SIF_A_ROW_M, b_layout = SIF_B_ROW_N), no batches; `tile` is ignored.  records_dev: device
 * memory of at least sif_k_gemm_bf16_group_bytes(n) bytes, 16-byte aligned, owned by the caller; the call copies the
 * products' records there (a synchronous host -> device copy) and launches on `stream`; the memory must stay
 * untouched until the launch has finished.  Every product's result has the bits of sif_k_gemm_bf16 with tile = 128.
 * Errors: SIF_E_INVAL for a null or misaligned pointer, n outside 1..16, other layouts, a batched product or anything
 * sif_k_gemm_bf16 refuses; nothing is launched then. */
uint64_t sif_k_gemm_bf16_group_bytes(uint32_t n);
sif_status sif_k_gemm_bf16_group(const sif_gemm_args* list, uint32_t n, void* records_dev, void* stream);

/* fp32 matrix product C[M,N] = sum_k A(m,k) B(k,n) with arbitrary element strides (Tiny configuration):
 * A(m,k) = a[m*a_sm + k*a_sk], B(k,n) = b[k*b_sk + n*b_sn], C row-major ldc.  epilogue: SIF_EPI_BIAS,
 * SIF_EPI_GELU (aux = pre-activation, fp32), SIF_EPI_GELU_GRAD (aux fp32) as above, all fp32. */
sif_status sif_k_gemm_f32(const float* a_dev, int64_t a_sm, int64_t a_sk, const float* b_dev, int64_t b_sk,
                          int64_t b_sn, float* c_dev, int64_t ldc, uint32_t m, uint32_t n, uint32_t k,
                          uint32_t epilogue, const float* bias_dev, float* aux_dev, void* stream);

/* LayerNorm over the last dimension (biased variance, eps 1e-5), bf16 in/out, fp32 statistics.
 * mean_dev / rstd_dev: fp32 [rows] or null (not saved). */
sif_status sif_k_layernorm_fwd(const void* x_dev, const void* g_dev, const void* b_dev, void* y_dev,
                               float* mean_dev, float* rstd_dev, uint32_t rows, uint32_t d, void* stream);
/* dx = res + LNbwd(dy) (res_dev may be null), dg/db = column sums of dy .* xhat and dy.  dsum_dev (bf16 [d], may
 * be null) receives the column sums of the stored dx: in a transformer block dx is the upstream gradient of the
 * bias added just before the residual sum this LayerNorm reads, so this is that bias's gradient.  part_dev is
 * fp32 scratch of (dsum_dev ? 3 : 2) * sif_colsum_parts(rows) * d floats.  Fixed summation order (no atomics). */
sif_status sif_k_layernorm_bwd(const void* dy_dev, const void* x_dev, const void* g_dev, const float* mean_dev,
                               const float* rstd_dev, const void* res_dev, void* dx_dev, void* dg_dev,
                               void* db_dev, void* dsum_dev, float* part_dev, uint32_t rows, uint32_t d, void* stream);
uint32_t sif_colsum_parts(uint32_t rows);
/* out[n] = sum_m x[m,n]  (bf16 in/out, fp32 fixed-order accumulation); part_dev: sif_colsum_parts(rows)*n floats */
sif_status sif_k_colsum(const void* x_dev, uint32_t ld, void* out_dev, float* part_dev, uint32_t rows, uint32_t n,
                        void* stream);

/* sif_k_colsum for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the partial sums live in a device array inside the library, 4 MiB on every GPU
 * the library runs on, held until the process ends.  Same kernels, same bits as sif_k_colsum.  Calls no hipMalloc,
 * hipFree or other allocating routine.  SIF_E_NOMEM (nothing launched) if sif_colsum_parts(rows) * n exceeds
 * sif_colsum_static_max_floats() (2^20); SIF_E_INVAL as sif_k_colsum.  All calls on one GPU share the one array, which
 * keeps the last call's contents (every element that is read is written first by the same call): two calls that
 * overlap on one GPU (different streams, no ordering between them) race; calls on one stream are safe. */
sif_status sif_k_colsum_static(const void* x_dev, uint32_t ld, void* out_dev, uint32_t rows, uint32_t n, void* stream);
uint64_t sif_colsum_static_max_floats(void);

/* Row softmax of fp32 scores [batch][rows][ld_s] into bf16 probabilities [batch][rows][ld_p]; causal != 0
 * keeps columns j <= i only.  Columns >= cols (up to ld_p) are written as zeros; with causal != 0 the zero fill of
 * row i stops at the end of its 128-column tile, (i/128 + 1)*128, which is as far as a causal product reads. */
sif_status sif_k_softmax_fwd(const float* s_dev, void* p_dev, uint32_t batch, uint32_t rows, uint32_t cols,
                             uint32_t ld_s, uint32_t ld_p, uint32_t causal, void* stream);
/* dS = scale * P .* (dP - rowsum(dP .* P)), dP fp32, P and dS bf16 (causal: columns j > i written as 0, up to the
 * end of the row's 128-column tile) */
sif_status sif_k_softmax_bwd(const float* dp_dev, const void* p_dev, void* ds_dev, uint32_t batch, uint32_t rows,
                             uint32_t cols, uint32_t ld, float scale, uint32_t causal, void* stream);

/* Fused attention forward: o[b,s,h*dh:(h+1)*dh] = softmax(q k^T / sqrt(dh) [+ causal mask]) v per (batch, head),
 * qkv bf16 [batch*seq][ld_qkv] with columns [q | k | v], each heads*d_head wide; o bf16 [batch*seq][ld_o].
 * d_head must be 64 or 128.  Scores never leave the chip.  lse_dev (device, fp32 [batch*heads][seq], may be NULL)
 * receives log(sum_j exp(score_ij)) of the scaled, masked scores, which the backward pass needs. */
sif_status sif_k_attn_fwd(const void* qkv_dev, void* o_dev, float* lse_dev, uint32_t batch, uint32_t seq, uint32_t heads,
                          uint32_t d_head, uint32_t ld_qkv, uint32_t ld_o, uint32_t causal, void* stream);
/* The same for n_seqs sequences of unequal length stored back to back: sequence i occupies rows seq_starts[i] ..
 * seq_starts[i+1] of qkv and o (seq_starts: HOST array of n_seqs + 1 ascending row numbers, read during the call;
 * 1 <= n_seqs <= 64, no empty sequence).  Each sequence's result has the bits it has when run by itself. */
sif_status sif_k_attn_fwd_varlen(const void* qkv_dev, void* o_dev, const uint32_t* seq_starts, uint32_t n_seqs, uint32_t heads,
                                 uint32_t d_head, uint32_t ld_qkv, uint32_t ld_o, uint32_t causal, void* stream);
/* Fused attention backward: dqkv [batch*seq][ld_dqkv] (columns [dq | dk | dv]) from qkv, the forward's o and lse and
 * the upstream gradient d_o [batch*seq][ld_o] (same layout and leading dimension as o).  The probabilities are
 * recomputed as exp(score - lse) and rounded to bf16, dS = P .* (dP - delta) / sqrt(dh) likewise, as the training
 * step of the collocated instance stores them (Sec. 5.1 workloads: transformer training); delta_dev (device, fp32
 * [batch*heads][seq]) is scratch that receives rowsum(d_o .* o).  Two launches on `stream` (dq; dk and dv), no
 * atomics: results do not depend on the launch configuration.  d_head must be 64 or 128. */
sif_status sif_k_attn_bwd(const void* qkv_dev, const void* o_dev, const void* d_o_dev, const float* lse_dev, float* delta_dev,
                          void* dqkv_dev, uint32_t batch, uint32_t seq, uint32_t heads, uint32_t d_head, uint32_t ld_qkv,
                          uint32_t ld_o, uint32_t ld_dqkv, uint32_t causal, void* stream);

/* x[t,:] = wte[ids[t],:] + wpe[t % seq,:]   (bf16).  wte has `vocab` rows; an id outside [0, vocab) is taken as the
 * nearest valid one (here and in every kernel that indexes a table with caller data: embedding backward, the targets
 * of the cross entropy), so that no input can make a kernel touch memory outside the table. */
sif_status sif_k_embed_fwd(const int32_t* ids_dev, const void* wte_dev, const void* wpe_dev, void* x_dev, uint32_t vocab,
                           uint32_t tokens, uint32_t seq, uint32_t d, void* stream);
/* dwte[v,:] += sum over tokens t with ids[t] = v of dx[t,:] in ascending t (bf16, fp32 sum, no atomics);
 * dwpe[s,:] = sum over the batch of dx[b*seq+s,:]. */
sif_status sif_k_embed_bwd(const int32_t* ids_dev, const void* dx_dev, void* dwte_dev, void* dwpe_dev, uint32_t vocab,
                           uint32_t tokens, uint32_t seq, uint32_t d, void* stream);

/* Mean token cross entropy over bf16 logits [tokens][ld] (first `vocab` columns valid): per-token loss into
 * loss_dev[t] (fp32) and, in place, logits <- (softmax - onehot(target)) / tokens with the padding columns
 * vocab..ld-1 set to zero. */
sif_status sif_k_xent_fwd_bwd(void* logits_dev, const int32_t* targets_dev, float* loss_dev, uint32_t tokens,
                              uint32_t vocab, uint32_t ld, void* stream);
/* out[0] = scale * sum x[0..n)  fixed order, one block (fp32) */
sif_status sif_k_reduce_sum(const float* x_dev, float* out_dev, uint32_t n, float scale, void* stream);

/* master <- master - lr * grad (fp32 master, bf16 grad), work <- bf16(master).  lr = 0 makes the working copy. */
sif_status sif_k_sgd_bf16(float* master_dev, const void* grad_dev, void* work_dev, uint64_t n, float lr, void* stream);
/* fp32 everything: p <- p - lr * g */
sif_status sif_k_sgd_f32(float* p_dev, const float* g_dev, uint64_t n, float lr, void* stream);
/* MLP loss: d[i] = (y[i]-t[i])/n, loss_dev[0] = sum (y-t)^2 / (2n)   (fp32, one pass, fixed order) */
sif_status sif_k_mse_fwd_bwd(const float* y_dev, const float* t_dev, float* d_dev, float* loss_dev, uint32_t n,
                             void* stream);
/* fp32 column sum: out[n] = sum_m x[m*ld + n] */
sif_status sif_k_colsum_f32(const float* x_dev, uint32_t ld, float* out_dev, uint32_t rows, uint32_t n, void* stream);

/* ====================================================================================================
 * 3. The collocation runtime.
 * ==================================================================================================== */

typedef struct sif_config {
  uint32_t struct_size;
  uint32_t period_us;        /* Bubble Monitor sampling period P                                       */
  uint32_t window;           /* sliding-window length W (<= 1024)                                      */
  uint32_t count_running;    /* 1: a period in which a training kernel is still running counts >= 1
                                (a launch counter alone reads 0 under one long kernel)                 */
  sif_alg1_params alg1;
  uint32_t kernel_us_max;    /* inference kernels predicted longer than this are split along rows      */
  uint32_t collocate;        /* 0: the barrier never releases anything (solo training / overhead run)  */
  uint32_t device_timed_bubbles; /* 0: bubbles are released by the host clock; 1: timed on the device  */
  uint32_t allow_serial_streams; /* 1: accept a stream pair that does not run concurrently (counter-collecting
                                    profilers serialise all kernels); nothing fills a bubble then            */
  uint64_t device_capacity_bytes; /* Principle-I capacity; 0 = total memory of the current device      */
  uint32_t feedback;         /* 1: concurrent filling with feedback: bubbles are filled as without it; an offline
                                kernel that Algorithm 1's tokens do not cover is forwarded against a time account
                                (sif_concurrent_account) and then starts whatever the training stream does; the share
                                of busy time follows sif_feedback_share after every training iteration during which
                                the barrier forwarded a kernel.  Reference = the shortest iteration seen since the
                                last sif_calibrate, starting from its solo iteration time when it was given training
                                inputs.  An online request is pulled outside a bubble too, as soon as the account
                                is in credit, and its kernels are paid from it one by one (before offline ones);
                                inside a bubble it is handled as without the option.                        */
  uint32_t feedback_eps_ppm; /* an iteration counts as lengthened beyond ref * (1 + eps)                      */
  uint32_t feedback_add_ppm; /* increase of the share after an iteration that did not lengthen               */
  uint32_t feedback_cap_ppm; /* largest share                                                                 */
  uint32_t gate_spin_log2;   /* 0 = default (18).  A block of a speculatively launched inference kernel waits at most
                                2^gate_spin_log2 polls for the decision of the launch's first block, then gives the
                                launch back to the host (it is run again).  Tests set 0 < value <= 30 small to force
                                that path; every kernel still exits normally.                                  */
  uint32_t gate_spin_every;  /* 0 or 1: gate_spin_log2 applies to every launch; n > 1: only to launches whose number on
                                the inference stream is a multiple of n, and not to the run that follows a launch
                                which came back (the others wait the default time), so that such a launch gets
                                through when it is run again                                                    */
} sif_config;

/* Fills *cfg with the defaults (P = 5 us, W = 64, alpha 1, beta 3, gamma 2, m 1, t0 = 200, LL = 400, UL = 800
 * tokens, kernel_us_max 300, collocate 1, feedback 0 with eps 2 %, add 2 %, cap 100 %).  With these constants a
 * period's grant (up to 800 us of predicted kernel time per 5 us period) never limits what is forwarded: the
 * speculation bound, the predicted end of the bubble and the device gate do.  Tokens limit the releases when UL is
 * of the order of the period (e.g. P = 100, t0 = 25, LL = 50, UL = 100). */
sif_status sif_default_config(sif_config* cfg);

/* Bytes of device workspace sif_create needs (activity records, trace rings). */
uint64_t sif_ctx_workspace_bytes(void);

/* Creates a context on the current device.  train_stream / infer_stream: two distinct hipStream_t of default
 * priority.  workspace_dev: caller-owned HBM, >= sif_ctx_workspace_bytes(), 256-byte aligned, zero-filled
 * by this call.  Starts the monitor and barrier threads. */
sif_status sif_create(const sif_config* cfg, void* train_stream, void* infer_stream, void* workspace_dev,
                      uint64_t workspace_bytes, sif_ctx** out);
/* Stops the threads, cancels pending tickets (SIF_E_CANCELLED), synchronises both streams. */
sif_status sif_destroy(sif_ctx* ctx);
/* on = 0: the barrier releases nothing while a training instance is registered (solo training, or the
 * "collocated but no requests served" overhead run of Sec. 5.4); on = 1: normal operation. */
sif_status sif_set_collocate(sif_ctx* ctx, uint32_t on);

enum { SIF_MODEL_MLP = 0, SIF_MODEL_DECODER = 1, SIF_MODEL_ENCODER = 2 };
enum { SIF_PAR_NONE = 0, SIF_PAR_FIXED = 1, SIF_PAR_DP = 2, SIF_PAR_PP = 3, SIF_PAR_TP = 4 };

/* Shape of a model.  MLP: d_in, d_hidden, d_out, batch.  DECODER / ENCODER: n_layers, d_model, n_heads,
 * d_head, d_ffn, vocab, max_pos, batch, seq (vocab = 0: layer stack only, activations in / gradient in).
 * d_model, d_head, d_ffn multiples of 8; batch*seq a multiple of 8 for training. */
typedef struct sif_model_shape {
  uint32_t kind, dtype;
  uint32_t n_layers, d_model, n_heads, d_head, d_ffn, vocab, max_pos;
  uint32_t d_in, d_hidden, d_out;
  uint32_t batch, seq;
} sif_model_shape;

/* Flat parameter layout (element offsets into one array of sif_model_n_params elements), in this order:
 *   MLP     : w1[d_hidden,d_in] b1 w2[d_out,d_hidden] b2
 *   DECODER : (vocab > 0: wte[vocab,d] wpe[max_pos,d]) then per layer ln1_g ln1_b w_qkv[3da,d] b_qkv w_o[d,da]
 *             b_o ln2_g ln2_b w_fc[f,d] b_fc w_proj[d,f] b_proj, then (vocab > 0: lnf_g lnf_b); da = n_heads*d_head
 *   ENCODER : wte wpe emb_ln_g emb_ln_b then per layer w_qkv b_qkv w_o b_o ln1_g ln1_b w_fc b_fc w_proj b_proj
 *             ln2_g ln2_b */
uint64_t sif_model_n_params(const sif_model_shape* s);

typedef struct sif_train_desc {
  uint32_t struct_size;
  uint32_t par_mode;             /* SIF_PAR_*: which bubbles the step contains                          */
  sif_model_shape shape;
  float lr;
  uint32_t pp_stages, pp_micro, pp_stage;
  uint64_t bw_bytes_per_s;       /* DP, TP: modelled collective bandwidth                               */
  uint64_t fixed_bubble_ns;      /* FIXED: one bubble of this length after backward                     */
  uint64_t pp_tf_ns, pp_tb_ns;   /* PP: per-micro-batch forward/backward time (0 = measured by calibration) */
  float* master_dev;             /* fp32 [n_params], caller-initialised, updated in place by each step  */
  void* workspace_dev;           /* >= sif_train_workspace_bytes(), 256-byte aligned                    */
  uint64_t workspace_bytes;
  uint64_t dp_bucket_bytes;      /* DP, decoder: 0 = one exposed all-reduce of all gradients after backward;
                                    > 0 = the gradients are exchanged in buckets of at least this size beside
                                    backward (sif_dp_gradient_buckets over: per layer, last to first, the layer's
                                    gradients (the final LayerNorm's ride with the last layer), then the
                                    embeddings), each as soon as it is final, and only what is left of the
                                    exchange when backward ends is waited for (sif_dp_overlapped_wait)        */
} sif_train_desc;

uint64_t sif_train_workspace_bytes(const sif_train_desc* d);

/* Sec. 3.1 (the training instance whose kernels the monitoring library counts) and Sec. 2.1 (where its idle phases
 * come from).  Registers the training instance (one per context).  Builds the kernel sequence and the bubble sites, makes
 * the working copy of the parameters (one cast kernel per tensor group on the training stream) and returns. */
sif_status sif_register_training_step(sif_ctx* ctx, const sif_train_desc* d, sif_handle* out);

/* Enqueues one training step on the training stream and returns without waiting.
 *   MLP: inputs_dev fp32 [batch,d_in], targets_dev fp32 [batch,d_out].
 *   DECODER with vocab: inputs_dev / targets_dev int32 token ids [batch,seq].
 *   DECODER stack (vocab = 0): inputs_dev bf16 activations [batch,seq,d]; targets_dev the upstream gradient, bf16
 *   [batch,seq,d].  With SIF_PAR_PP both carry pp_micro micro-batches, [pp_micro,batch,seq,d]; the step runs them
 *   in the 1F1B order of stage pp_stage, accumulates the parameter gradients over the micro-batches and updates
 *   once; outputs and input gradients of every micro-batch are kept as the tensors "y_all" and "dx_all".
 * loss_dev: fp32 device scalar written by the step (may be null).  Buffers must stay valid until the step
 * has run (sif_sync_training). */
sif_status sif_run_training_step(sif_ctx* ctx, sif_handle h, const void* inputs_dev, const void* targets_dev,
                                 float* loss_dev);
sif_status sif_sync_training(sif_ctx* ctx);

/* Device address of a named tensor inside the training workspace, for inspection after sif_sync_training:
 * "work" (working copy of all parameters), "grads" (all gradients, parameter layout; bf16 or fp32 as the
 * model), per layer: "ln1" "qkv" "prob" "o" "x_mid" "ln2" "z" "a" "x_out", and "logits", "x0", "dx_in", "y_all",
 * "dx_all".
 * *elems = number of elements. */
sif_status sif_train_tensor(sif_ctx* ctx, sif_handle h, const char* name, int32_t layer, void** ptr_dev,
                            uint64_t* elems);

/* Bucket `index` of the bucketed gradient exchange (dp_bucket_bytes > 0): its gradient bytes and the index, in the
 * step's kernel sequence, of the launch whose end makes it final.  SIF_E_INVAL past the last bucket. */
sif_status sif_train_dp_bucket(sif_ctx* ctx, sif_handle h, uint32_t index, uint64_t* bytes, uint32_t* ready_launch);

/* Name of the index-th launch of the training step's kernel sequence ("qkv", "attn_scores", "bubble", ...), the
 * same index a training-kernel trace record carries in `id`; null past the end. */
const char* sif_train_op_name(sif_ctx* ctx, sif_handle h, uint32_t index);

typedef struct sif_infer_desc {
  uint32_t struct_size;
  uint32_t online;               /* 0 = offline (token mechanism), 1 = online (pull-and-execute)        */
  sif_model_shape shape;         /* batch, seq = the largest batch / sequence a submit may carry        */
  const float* master_dev;       /* fp32 [n_params] weights, caller-owned                               */
  void* workspace_dev;           /* >= sif_infer_workspace_bytes(): working copy + activations          */
  uint64_t workspace_bytes;
  uint64_t peak_bytes;           /* declared peak memory of this instance (Principle-I)                 */
  uint32_t coalesce;             /* encoder models: up to this many queued requests are released as ONE kernel
                                    sequence over their concatenated rows (0 or 1 = each request by itself, at most 32).
                                    Offline: requests of equal batch and seq.  Online: the requests that wait at the
                                    moment one is pulled, whatever their lengths (fewer if the predicted rest of the
                                    bubble does not hold them all); attention is told where each sequence begins.
                                    Every kernel of the forward pass treats rows (or whole sequences) independently,
                                    so each request's output is bit-identical to a run by itself; the workspace is
                                    sized for coalesce * shape.batch * shape.seq rows.  Requests are never held back
                                    to wait for partners.                                                   */
  uint32_t reserved;
} sif_infer_desc;

uint64_t sif_infer_workspace_bytes(const sif_infer_desc* d);

/* Sec. 3.2 (collocation policy).  Registers an inference instance.  SIF_E_NOMEM if the declared peaks of all instances plus the training
 * workspace exceed the device capacity (Principle-I). */
sif_status sif_register_inference_model(sif_ctx* ctx, const sif_infer_desc* d, sif_handle* out);

/* Runs the registered models alone (no collocation, gates open) `iters` times to measure per-kernel costs,
 * the solo step time and the bubble lengths (a pipeline stage registered without pp_tf_ns / pp_tb_ns gets the idle
 * intervals of its schedule re-sized from the measured forward and backward time of a micro-batch, which needs the
 * training inputs here); blocks until done.  Returns SIF_W_SLO_RISK if an online model's
 * batch-1 time exceeds the longest bubble (Principle-II). */
sif_status sif_calibrate(sif_ctx* ctx, uint32_t iters, const void* train_inputs_dev, const void* train_targets_dev);

/* Sec. 3.3 "Kernel Barrier": an offline batch is served by the token mechanism, an online request by
 * pull-and-execute.  Queues one offline batch / one online request (non-blocking, any thread).  in_dev: int32 ids [batch,seq]
 * (ENCODER) or fp32 [batch,d_in] (MLP); out_dev: bf16 [batch,seq,d] or fp32 [batch,d_out]. */
sif_status sif_submit_offline_batch(sif_ctx* ctx, sif_handle model, const void* in_dev, void* out_dev,
                                    uint32_t batch, uint32_t seq, sif_ticket* out);
sif_status sif_submit_online_request(sif_ctx* ctx, sif_handle model, const void* in_dev, void* out_dev,
                                     uint32_t seq, uint64_t t_arrival_ns, sif_ticket* out);
/* Blocks until the ticket completes or timeout_ns passes (SIF_E_TIMEOUT). */
sif_status sif_wait(sif_ctx* ctx, sif_ticket t, uint64_t timeout_ns);
/* Host monotonic clock used for t_arrival_ns and the latency statistics. */
uint64_t sif_now_ns(void);

/* Sec. 5.1 "Metrics" (training and inference throughput, request latency percentiles) and Sec. 5.4 (overhead). */
typedef struct sif_stats {
  uint32_t struct_size;
  uint32_t status_now, zc_now;
  uint32_t concurrent_share_ppm;  /* concurrent filling with feedback: the share of busy time now granted  */
  uint64_t tokens_now;
  uint64_t steps;                 /* training steps completed                                           */
  uint64_t step_ns_sum, step_ns_last, step_solo_ns;
  uint64_t bubble_ns;             /* total modelled idle time of completed bubbles                      */
  uint64_t filled_ns;             /* inference kernel time that fell inside bubbles                     */
  uint64_t infer_busy_ns;         /* all inference kernel time                                          */
  uint64_t offline_samples, offline_batches;
  uint64_t online_done, online_p50_ns, online_p95_ns;
  uint64_t kernels_launched, kernels_skipped, kernels_run;
  uint64_t gate_violations;       /* inference kernels admitted into a bubble whose start stamp lies outside that
                                     bubble's own begin / end stamps (must be 0; Sec. 2.2: training must not be
                                     disturbed).  Checked by the barrier thread for every such kernel that ran.    */
  uint64_t train_kernels;
  uint64_t periods;               /* monitor periods evaluated                                           */
  uint64_t gate_checked;          /* kernel starts that check has judged so far (violations included)    */
  uint64_t gate_unchecked;        /* starts whose stamps did not reach the host within 200 ms            */
  uint64_t gate_timeouts;         /* != 0: a block gave up waiting for its launch's gate decision (the launch was
                                     run again; see sif_config.gate_spin_log2)                           */
} sif_stats;

/* Snapshot of the counters; takes no lock and touches no stream (the counters are atomics, the latency percentiles
 * come from a fixed-bucket histogram: nearest rank, reported as the middle of the bucket, within 1/32 of the value). */
sif_status sif_poll_stats(sif_ctx* ctx, sif_stats* out);
/* Zeroes the accumulating counters (between measurement phases); requires both streams idle. */
sif_status sif_reset_stats(sif_ctx* ctx);

/* Event timing of the bf16 GEMM launches, for roofline reporting.  While on (on = 1: every GEMM launch of both
 * streams; on = 2: only the variant with both operands K-contiguous, a_layout = b_layout = 0, so that a timed region
 * carries fewer event records; on = 3: every third launch of that variant on each stream - an event pair takes about
 * 2 us of its stream's time, and the launches of a layer come in fours, so every shape is sampled alike) a launch is
 * bracketed by two HIP events on its own stream (at most 16384 launches per switch-on).  sif_profile_read (profiling switched off first; synchronises both streams)
 * returns per layout variant v = a_layout*2 + b_layout the number of timed launches, their algorithmic
 * floating-point operations (2mnk per batch; the lower triangle only for causal products) and the sum of their
 * event-to-event times in seconds.  Inference launches that the device gate skipped are left out. */
sif_status sif_profile_gemm(sif_ctx* ctx, uint32_t on);
sif_status sif_profile_read(sif_ctx* ctx, uint64_t launches[4], double flops[4], double seconds[4]);

/* What the Kernel Barrier forwarded while a training instance was registered: one record per launch, in launch order.
 * The newest 65536 are kept. */
typedef struct sif_release_rec {
  uint64_t period;      /* number of the monitor period whose grant was the balance at that moment         */
  uint64_t grant;       /* that grant (tokens per instance)                                                */
  uint32_t model;       /* inference instance                                                              */
  uint32_t charge;      /* tokens taken (sif_kb_charge of the predicted time)                              */
  uint32_t launch;      /* launch number on the inference stream (sif_trace_rec.reserved)                  */
  uint32_t kind;        /* 0 offline, paid with tokens (Sec. 3.3 token mechanism); 1 kernel of a pulled online
                           request (no tokens); 2 beside training, paid from the time account (feedback) */
} sif_release_rec;
/* Copies the newest records to out[0..max), oldest first; pauses the barrier thread meanwhile. */
sif_status sif_read_release_log(sif_ctx* ctx, sif_release_rec* out, uint32_t max, uint32_t* n);
/* Counts of the online latency histogram (buckets as sif_latency_bucket numbers them); takes no lock. */
sif_status sif_read_latency_histogram(sif_ctx* ctx, uint64_t* counts, uint32_t max, uint32_t* n);

/* One record of the device trace ring. */
typedef struct sif_trace_rec {
  uint32_t kind;        /* 1 training kernel, 2 inference kernel, 3 bubble, 4 step                      */
  uint32_t id;          /* kernel sequence number / bubble site / step index                            */
  uint32_t decision;    /* inference kernels: 1 ran, 2 skipped                                          */
  uint32_t reserved;
  uint64_t t0_ns, t1_ns;/* device wall clock                                                            */
} sif_trace_rec;
/* Copies the newest records of a stream's ring (0 = training, 1 = inference) to out[0..max), oldest first;
 * synchronises both streams first.  Returns the count in *n. */
sif_status sif_read_trace(sif_ctx* ctx, uint32_t which, sif_trace_rec* out, uint32_t max, uint32_t* n);

#ifdef __cplusplus
}
#endif
#endif
