// C ABI of the single-kernel launchers (unmonitored launches: no activity record, no gate).
#include <vector>

#include "launch.h"

using namespace sif;
static inline hipStream_t S(void* s) { return reinterpret_cast<hipStream_t>(s); }

extern "C" {

sif_status sif_k_gemm_bf16(const sif_gemm_args* a, void* stream) { return launch_gemm_bf16(a, S(stream), no_ctl()); }

uint64_t sif_k_gemm_bf16_group_bytes(uint32_t n) { return gemm_group_bytes(n); }

sif_status sif_k_gemm_bf16_group(const sif_gemm_args* list, uint32_t n, void* records_dev, void* stream) {
  if (list == nullptr || n == 0 || n > 16 || records_dev == nullptr || (reinterpret_cast<uintptr_t>(records_dev) & 15))
    return fail(SIF_E_INVAL, "gemm group: null or misaligned argument, or n outside 1..16");
  std::vector<unsigned char> host(gemm_group_bytes(n));
  uint32_t grid = 0;
  if (sif_status st = gemm_group_fill(list, n, host.data(), &grid)) return st;
  const hipError_t e = hipMemcpy(records_dev, host.data(), host.size(), hipMemcpyHostToDevice);
  if (e != hipSuccess) return fail_hip(e, "gemm group: copy of the records");
  return launch_gemm_bf16_group(records_dev, n, grid, list[0].a_layout, list[0].b_layout, S(stream), no_ctl());
}

sif_status sif_k_gemm_f32(const float* a_dev, int64_t a_sm, int64_t a_sk, const float* b_dev, int64_t b_sk, int64_t b_sn,
                          float* c_dev, int64_t ldc, uint32_t m, uint32_t n, uint32_t k, uint32_t epilogue,
                          const float* bias_dev, float* aux_dev, void* stream) {
  return launch_gemm_f32(a_dev, a_sm, a_sk, b_dev, b_sk, b_sn, c_dev, ldc, m, n, k, epilogue, bias_dev, aux_dev, S(stream), no_ctl());
}

sif_status sif_k_layernorm_fwd(const void* x, const void* g, const void* b, void* y, float* mean, float* rstd,
                               uint32_t rows, uint32_t d, void* stream) {
  return launch_layernorm_fwd(x, g, b, y, mean, rstd, rows, d, S(stream), no_ctl());
}

sif_status sif_k_layernorm_bwd(const void* dy, const void* x, const void* g, const float* mean, const float* rstd,
                               const void* res, void* dx, void* dg, void* db, void* dsum, float* part, uint32_t rows, uint32_t d,
                               void* stream) {
  if (!dg || !db) return fail(SIF_E_INVAL, "layernorm_bwd: null dg/db");
  sif_status st = launch_layernorm_bwd_dx(dy, x, g, mean, rstd, res, dx, part, rows, d, dsum != nullptr, S(stream), no_ctl());
  if (st != SIF_OK) return st;
  return launch_layernorm_bwd_fin(part, dg, db, dsum, rows, d, 0, S(stream), no_ctl());
}

uint32_t sif_colsum_parts(uint32_t rows) { return colsum_parts(rows); }

sif_status sif_k_colsum(const void* x, uint32_t ld, void* out, float* part, uint32_t rows, uint32_t n, void* stream) {
  if (!out) return fail(SIF_E_INVAL, "colsum: null out");
  sif_status st = launch_colsum_part(x, ld, part, rows, n, S(stream), no_ctl());
  if (st != SIF_OK) return st;
  return launch_colsum_fin(part, out, rows, n, 0, S(stream), no_ctl());
}

sif_status sif_k_softmax_fwd(const float* s, void* p, uint32_t batch, uint32_t rows, uint32_t cols, uint32_t ld_s,
                             uint32_t ld_p, uint32_t causal, void* stream) {
  return launch_softmax_fwd(s, p, batch, rows, cols, ld_s, ld_p, causal, S(stream), no_ctl());
}

sif_status sif_k_softmax_bwd(const float* dp, const void* p, void* ds, uint32_t batch, uint32_t rows, uint32_t cols,
                             uint32_t ld, float scale, uint32_t causal, void* stream) {
  return launch_softmax_bwd(dp, p, ds, batch, rows, cols, ld, scale, causal, S(stream), no_ctl());
}

sif_status sif_k_attn_fwd(const void* qkv, void* o, float* lse, uint32_t batch, uint32_t seq, uint32_t heads, uint32_t d_head,
                          uint32_t ld_qkv, uint32_t ld_o, uint32_t causal, void* stream) {
  return launch_attn_fwd(qkv, o, lse, batch, seq, heads, d_head, ld_qkv, ld_o, causal, S(stream), no_ctl());
}

sif_status sif_k_attn_fwd_varlen(const void* qkv, void* o, const uint32_t* seq_starts, uint32_t n_seqs, uint32_t heads, uint32_t d_head,
                                 uint32_t ld_qkv, uint32_t ld_o, uint32_t causal, void* stream) {
  return launch_attn_fwd_varlen(qkv, o, seq_starts, n_seqs, heads, d_head, ld_qkv, ld_o, causal, S(stream), no_ctl());
}

sif_status sif_k_attn_bwd(const void* qkv, const void* o, const void* d_o, const float* lse, float* delta, void* dqkv, uint32_t batch,
                          uint32_t seq, uint32_t heads, uint32_t d_head, uint32_t ld_qkv, uint32_t ld_o, uint32_t ld_dqkv, uint32_t causal,
                          void* stream) {
  sif_status st = launch_attn_bwd_dq(qkv, o, d_o, lse, delta, dqkv, batch, seq, heads, d_head, ld_qkv, ld_o, ld_dqkv, causal, S(stream), no_ctl());
  if (st != SIF_OK) return st;
  return launch_attn_bwd_dkv(qkv, d_o, lse, delta, dqkv, batch, seq, heads, d_head, ld_qkv, ld_o, ld_dqkv, causal, S(stream), no_ctl());
}

sif_status sif_k_embed_fwd(const int32_t* ids, const void* wte, const void* wpe, void* x, uint32_t vocab, uint32_t tokens, uint32_t seq,
                           uint32_t d, void* stream) {
  return launch_embed_fwd(ids, wte, wpe, x, vocab, tokens, seq, d, S(stream), no_ctl());
}

sif_status sif_k_embed_bwd(const int32_t* ids, const void* dx, void* dwte, void* dwpe, uint32_t vocab, uint32_t tokens, uint32_t seq,
                           uint32_t d, void* stream) {
  sif_status st = launch_embed_bwd_wte(ids, dx, dwte, vocab, tokens, d, S(stream), no_ctl());
  if (st != SIF_OK) return st;
  return launch_embed_bwd_wpe(dx, dwpe, tokens, seq, d, S(stream), no_ctl());
}

sif_status sif_k_xent_fwd_bwd(void* logits, const int32_t* targets, float* loss, uint32_t tokens, uint32_t vocab,
                              uint32_t ld, void* stream) {
  return launch_xent(logits, targets, loss, tokens, vocab, ld, S(stream), no_ctl());
}

sif_status sif_k_reduce_sum(const float* x, float* out, uint32_t n, float scale, void* stream) {
  return launch_reduce_sum(x, out, n, scale, S(stream), no_ctl());
}

sif_status sif_k_sgd_bf16(float* master, const void* grad, void* work, uint64_t n, float lr, void* stream) {
  return launch_sgd_bf16(master, grad, work, n, lr, S(stream), no_ctl());
}

sif_status sif_k_sgd_f32(float* p, const float* g, uint64_t n, float lr, void* stream) {
  return launch_sgd_f32(p, g, n, lr, S(stream), no_ctl());
}

sif_status sif_k_mse_fwd_bwd(const float* y, const float* t, float* d, float* loss, uint32_t n, void* stream) {
  return launch_mse(y, t, d, loss, n, S(stream), no_ctl());
}

sif_status sif_k_colsum_f32(const float* x, uint32_t ld, float* out, uint32_t rows, uint32_t n, void* stream) {
  return launch_colsum_f32(x, ld, out, rows, n, S(stream), no_ctl());
}

}  // extern "C"
