// Host-side helpers shared by the launchers: error reporting and the internal launcher prototypes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "monitor.h"
#include "specinf.h"

namespace sif {

sif_status fail(sif_status code, const char* fmt, ...);
sif_status fail_hip(hipError_t e, const char* what);
// Checks hipGetLastError() after a launch.
sif_status check_launch(const char* what);

inline KCtl no_ctl() { KCtl c{}; return c; }

// Internal launchers: same argument checks as the public sif_k_* entry points, plus the monitor control block.
sif_status launch_gemm_bf16(const sif_gemm_args* a, hipStream_t s, const KCtl& c);
// several products of the same operand layouts as one launch of 128x128 tiles: fill the kernel records on the host
// (gemm_group_bytes(n) bytes), copy them to device memory once, launch with that copy
uint64_t gemm_group_bytes(uint32_t n);
sif_status gemm_group_fill(const sif_gemm_args* list, uint32_t n, void* host_records, uint32_t* grid_out);
sif_status launch_gemm_bf16_group(const void* dev_records, uint32_t n, uint32_t grid, uint32_t a_layout, uint32_t b_layout, hipStream_t s, const KCtl& c);
// whether the product may run, and whether it will run, on 256x256 tiles (else 128x128)
bool gemm_can_use_big_tiles(const sif_gemm_args& a);
bool gemm_big_tiles(const sif_gemm_args& a);
sif_status launch_gemm_f32(const float* a, int64_t a_sm, int64_t a_sk, const float* b, int64_t b_sk, int64_t b_sn,
                           float* c, int64_t ldc, uint32_t m, uint32_t n, uint32_t k, uint32_t epi, const float* bias,
                           float* aux, hipStream_t s, const KCtl& ctl);
// segs (optional): the output rows go to the segments' buffers instead of y
struct RowSegs;
sif_status launch_layernorm_fwd(const void* x, const void* g, const void* b, void* y, float* mean, float* rstd,
                                uint32_t rows, uint32_t d, hipStream_t s, const KCtl& c, const RowSegs* segs = nullptr);
sif_status launch_layernorm_bwd_dx(const void* dy, const void* x, const void* g, const float* mean, const float* rstd,
                                   const void* res, void* dx, float* part, uint32_t rows, uint32_t d, uint32_t with_sum, hipStream_t s,
                                   const KCtl& c);
sif_status launch_layernorm_bwd_fin(const float* part, void* dg, void* db, void* dsum, uint32_t rows, uint32_t d, uint32_t acc,
                                    hipStream_t s, const KCtl& c);
sif_status launch_colsum_part(const void* x, uint32_t ld, float* part, uint32_t rows, uint32_t n, hipStream_t s,
                              const KCtl& c);
sif_status launch_colsum_fin(const float* part, void* out, uint32_t rows, uint32_t n, uint32_t acc, hipStream_t s, const KCtl& c);
sif_status launch_softmax_fwd(const float* sc, void* p, uint32_t batch, uint32_t rows, uint32_t cols, uint32_t ld_s,
                              uint32_t ld_p, uint32_t causal, hipStream_t s, const KCtl& c);
sif_status launch_softmax_bwd(const float* dp, const void* p, void* ds, uint32_t batch, uint32_t rows, uint32_t cols,
                              uint32_t ld, float scale, uint32_t causal, hipStream_t s, const KCtl& c);
// Sequences of unequal length in one attention launch: sequence i occupies rows start[i] .. start[i+1] (n = 0:
// equal lengths, see launch_attn_fwd)
constexpr uint32_t kAttnMaxSeqs = 64;
struct AttnSeqs { uint32_t n; uint32_t start[kAttnMaxSeqs + 1]; };

// Rows of several requests laid back to back: segment r is rows row0[r] .. row0[r+1] and has a buffer of its own
// (the token ids an embedding reads, or the place a LayerNorm writes).  n = 0: no segments, one buffer for all rows.
constexpr uint32_t kMaxRowSegs = 32;
struct RowSegs {
  uint32_t n;
  uint32_t row0[kMaxRowSegs + 1];
  uint32_t seq[kMaxRowSegs];         // embedding: the sequence length within the segment (position = row in segment % seq)
  void* ptr[kMaxRowSegs];
};
sif_status launch_attn_fwd_varlen(const void* qkv, void* o, const uint32_t* starts, uint32_t n_seqs, uint32_t heads, uint32_t d_head,
                                  uint32_t ld_qkv, uint32_t ld_o, uint32_t causal, hipStream_t s, const KCtl& c);
sif_status launch_attn_fwd(const void* qkv, void* o, float* lse, uint32_t batch, uint32_t seq, uint32_t heads, uint32_t d_head,
                           uint32_t ld_qkv, uint32_t ld_o, uint32_t causal, hipStream_t s, const KCtl& c);
sif_status launch_attn_bwd_dq(const void* qkv, const void* o, const void* d_o, const float* lse, float* delta, void* dqkv, uint32_t batch,
                              uint32_t seq, uint32_t heads, uint32_t d_head, uint32_t ld_qkv, uint32_t ld_o, uint32_t ld_dqkv, uint32_t causal,
                              hipStream_t s, const KCtl& c);
sif_status launch_attn_bwd_dkv(const void* qkv, const void* d_o, const float* lse, const float* delta, void* dqkv, uint32_t batch, uint32_t seq,
                               uint32_t heads, uint32_t d_head, uint32_t ld_qkv, uint32_t ld_o, uint32_t ld_dqkv, uint32_t causal, hipStream_t s,
                               const KCtl& c);
// token ids per segment (segs.ptr), positions restart with every sequence of a segment
sif_status launch_embed_fwd_segs(const RowSegs& segs, const void* wte, const void* wpe, void* x, uint32_t vocab, uint32_t d, hipStream_t s, const KCtl& c);
sif_status launch_embed_fwd(const int32_t* ids, const void* wte, const void* wpe, void* x, uint32_t vocab, uint32_t tokens,
                            uint32_t seq, uint32_t d, hipStream_t s, const KCtl& c);
sif_status launch_embed_bwd_wte(const int32_t* ids, const void* dx, void* dwte, uint32_t vocab, uint32_t tokens, uint32_t d,
                                hipStream_t s, const KCtl& c);
sif_status launch_embed_bwd_wpe(const void* dx, void* dwpe, uint32_t tokens, uint32_t seq, uint32_t d, hipStream_t s,
                                const KCtl& c);
sif_status launch_xent(void* logits, const int32_t* targets, float* loss, uint32_t tokens, uint32_t vocab, uint32_t ld,
                       hipStream_t s, const KCtl& c);
sif_status launch_reduce_sum(const float* x, float* out, uint32_t n, float scale, hipStream_t s, const KCtl& c);
sif_status launch_sgd_bf16(float* master, const void* grad, void* work, uint64_t n, float lr, hipStream_t s,
                           const KCtl& c);
sif_status launch_sgd_f32(float* p, const float* g, uint64_t n, float lr, hipStream_t s, const KCtl& c);
sif_status launch_mse(const float* y, const float* t, float* d, float* loss, uint32_t n, hipStream_t s, const KCtl& c);
sif_status launch_colsum_f32(const float* x, uint32_t ld, float* out, uint32_t rows, uint32_t n, hipStream_t s,
                             const KCtl& c);
sif_status launch_copy(void* dst, const void* src, uint64_t bytes, hipStream_t s, const KCtl& c);
sif_status launch_fill_u32(uint32_t* p, uint32_t v, uint64_t n, hipStream_t s, const KCtl& c);

uint32_t colsum_parts(uint32_t rows);
// one set of partial column sums awaiting its finalize: part = nsum consecutive blocks of [parts][n] floats, out[s]
// (bf16 [n], may be null) receives the s-th sum
struct FinItem { const float* part; uint16_t* out[3]; uint32_t parts, n, nsum, pad; };
// one split product awaiting the sum of its K slices: part = splits blocks of n floats, out bf16 [n] (n a multiple of 8)
struct RedItem { const float* part; uint16_t* out; uint64_t n; uint32_t splits, pad; };
sif_status launch_reduce_splits_batch(const RedItem* items_dev, uint32_t n_items, uint32_t acc, hipStream_t s, const KCtl& c);
sif_status launch_fin_batch(const FinItem* items_dev, uint32_t n_items, uint32_t max_n, uint32_t acc, hipStream_t s, const KCtl& c);

}  // namespace sif
