// Kernel plans of the registered models: which kernels one training step (forward, loss, backward, optimizer,
// with the modelled bubbles at their sites) and one inference forward pass consist of, and where their tensors
// live inside the caller's workspace.  The paper schedules the kernels of named transformer models (Sec. 5.1
// "Workloads"); these are the textbook blocks of those models at the benchmark shapes:
//   training  : two-Linear fp32 MLP, or a pre-LN GPT-style decoder (optionally with embedding + tied LM head)
//   inference : the same MLP forward, or a post-LN BERT-shaped encoder forward
// Attention materialises the score matrix per (batch, head) with the batched GEMM; every reduction has a fixed
// order, so a plan gives bit-identical results whenever and next to whatever it runs.
#include <algorithm>
#include <math.h>
#include <string.h>

#include "common.h"
#include "runtime.h"

namespace sif {

// ------------------------------------------------------------------------------------------ parameter layout
struct ParamMap {
  std::unordered_map<std::string, uint64_t> off;
  uint64_t n = 0;
  void add(const std::string& k, uint64_t elems) { off[k] = n; n += elems; }
  uint64_t at(const std::string& k) const { return off.at(k); }
};

static std::string L(uint32_t l, const char* k) { return "L" + std::to_string(l) + "." + k; }

static ParamMap param_map(const sif_model_shape& s) {
  ParamMap m;
  const uint64_t d = s.d_model, da = (uint64_t)s.n_heads * s.d_head, f = s.d_ffn;
  if (s.kind == SIF_MODEL_MLP) {
    m.add("w1", (uint64_t)s.d_hidden * s.d_in); m.add("b1", s.d_hidden);
    m.add("w2", (uint64_t)s.d_out * s.d_hidden); m.add("b2", s.d_out);
  } else if (s.kind == SIF_MODEL_DECODER) {
    if (s.vocab) { m.add("wte", (uint64_t)s.vocab * d); m.add("wpe", (uint64_t)s.max_pos * d); }
    for (uint32_t l = 0; l < s.n_layers; ++l) {
      m.add(L(l, "ln1_g"), d); m.add(L(l, "ln1_b"), d); m.add(L(l, "w_qkv"), 3 * da * d); m.add(L(l, "b_qkv"), 3 * da);
      m.add(L(l, "w_o"), d * da); m.add(L(l, "b_o"), d); m.add(L(l, "ln2_g"), d); m.add(L(l, "ln2_b"), d);
      m.add(L(l, "w_fc"), f * d); m.add(L(l, "b_fc"), f); m.add(L(l, "w_proj"), d * f); m.add(L(l, "b_proj"), d);
    }
    if (s.vocab) { m.add("lnf_g", d); m.add("lnf_b", d); }
  } else if (s.kind == SIF_MODEL_ENCODER) {
    m.add("wte", (uint64_t)s.vocab * d); m.add("wpe", (uint64_t)s.max_pos * d); m.add("emb_ln_g", d); m.add("emb_ln_b", d);
    for (uint32_t l = 0; l < s.n_layers; ++l) {
      m.add(L(l, "w_qkv"), 3 * da * d); m.add(L(l, "b_qkv"), 3 * da); m.add(L(l, "w_o"), d * da); m.add(L(l, "b_o"), d);
      m.add(L(l, "ln1_g"), d); m.add(L(l, "ln1_b"), d); m.add(L(l, "w_fc"), f * d); m.add(L(l, "b_fc"), f);
      m.add(L(l, "w_proj"), d * f); m.add(L(l, "b_proj"), d); m.add(L(l, "ln2_g"), d); m.add(L(l, "ln2_b"), d);
    }
  }
  return m;
}

uint64_t model_n_params(const sif_model_shape& s) { return param_map(s).n; }

static sif_status check_shape(const sif_model_shape& s, bool training) {
  if (s.kind == SIF_MODEL_MLP) {
    if (s.dtype != SIF_F32) return fail(SIF_E_INVAL, "MLP models are fp32");
    if (!s.d_in || !s.d_hidden || !s.d_out || !s.batch) return fail(SIF_E_INVAL, "MLP: empty dimension");
    return SIF_OK;
  }
  if (s.kind != SIF_MODEL_DECODER && s.kind != SIF_MODEL_ENCODER) return fail(SIF_E_INVAL, "unknown model kind");
  if (s.dtype != SIF_BF16) return fail(SIF_E_INVAL, "transformer models are bf16");
  if (!s.n_layers || !s.d_model || !s.n_heads || !s.d_head || !s.d_ffn || !s.batch || !s.seq) return fail(SIF_E_INVAL, "transformer: empty dimension");
  if ((s.d_model | s.d_head | s.d_ffn) & 7) return fail(SIF_E_INVAL, "d_model, d_head and d_ffn must be multiples of 8");
  if (s.d_model > 4096) return fail(SIF_E_INVAL, "d_model must be <= 4096");
  if (s.seq > 2048) return fail(SIF_E_INVAL, "seq must be <= 2048");
  if (s.kind == SIF_MODEL_ENCODER && (!s.vocab || !s.max_pos)) return fail(SIF_E_INVAL, "encoder needs vocab and max_pos");
  if (s.vocab && s.max_pos < s.seq) return fail(SIF_E_INVAL, "max_pos must be >= seq");
  if (training && ((s.batch * s.seq) & 7)) return fail(SIF_E_INVAL, "training needs batch*seq to be a multiple of 8");
  return SIF_OK;
}

// ------------------------------------------------------------------------------------------ op builders
struct G {
  sif_gemm_args a;
  G(const void* A, const void* B, void* C, uint32_t m, uint32_t n, uint32_t k, uint32_t lda, uint32_t ldb, uint32_t ldc) {
    memset(&a, 0, sizeof(a));
    a.struct_size = sizeof(a);
    a.a_dev = A; a.b_dev = B; a.c_dev = C; a.m = m; a.n = n; a.k = k; a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.batch_outer = a.batch_inner = 1; a.alpha = 1.0f;
  }
  G& lay(uint32_t al, uint32_t bl) { a.a_layout = al; a.b_layout = bl; return *this; }
  G& epi(uint32_t e, const void* bias = nullptr, const void* res = nullptr, void* aux = nullptr) {
    a.epilogue = e; a.bias_dev = bias; a.res_dev = res; a.aux_dev = aux; return *this;
  }
  G& batch(uint32_t bo, uint32_t bi, int64_t aso, int64_t asi, int64_t bso, int64_t bsi, int64_t cso, int64_t csi) {
    a.batch_outer = bo; a.batch_inner = bi; a.a_stride_outer = aso; a.a_stride_inner = asi; a.b_stride_outer = bso;
    a.b_stride_inner = bsi; a.c_stride_outer = cso; a.c_stride_inner = csi; return *this;
  }
  G& alpha(float v) { a.alpha = v; return *this; }
  G& causal(uint32_t kc) { a.k_causal = kc; return *this; }
  G& k_limit(uint32_t kl) { a.k_limit = kl; return *this; }
  G& tile(uint32_t t) { a.tile = t; return *this; }
};

// scratch buffers of the backward pass, shared by all layers
struct Scratch { float* scores; bf16_t* ds; float* delta; bf16_t *dx_a, *dx_b, *dln, *dqkv, *d_o, *dz; };

static double gemm_cost_us(const sif_gemm_args& g) {
  double flops = 2.0 * g.m * g.n * g.k * g.batch_outer * g.batch_inner;
  if (g.k_causal || (g.epilogue & SIF_EPI_CAUSAL_SKIP)) flops *= 0.55;
  return 4.0 + flops / 6.0e8;          // 600 TFLOP/s plus launch latency
}
static double bytes_cost_us(double bytes) { return 3.0 + bytes / 2.0e6; }   // 2 TB/s plus launch latency

// Floating-point operations the product needs: 2mnk per batch; a causal product touches only the lower
// triangle of the square score matrix (s(s+1)/2 of its s*s entries).
static double gemm_flops(const sif_gemm_args& g) {
  const double batches = (double)g.batch_outer * g.batch_inner;
  if (g.epilogue & SIF_EPI_CAUSAL_SKIP) return batches * 2.0 * g.k * (0.5 * g.m * (g.m + 1.0));
  if (g.k_causal) return batches * 2.0 * g.n * (0.5 * g.m * (g.m + 1.0));
  if (g.k_limit) return (double)g.batch_outer * 2.0 * g.m * g.n * g.k_limit;       // slices of one long K, the last one shorter
  return batches * 2.0 * g.m * g.n * g.k;
}

static Op make_gemm_op(const char* name, const sif_gemm_args& a) {
  Op op;
  op.name = name;
  op.fn = [a](hipStream_t s, const KCtl& c) { return launch_gemm_bf16(&a, s, c); };
  op.cost_us = gemm_cost_us(a);
  op.prof_class = (int32_t)(a.a_layout * 2 + a.b_layout);
  op.flops = gemm_flops(a);
  op.gemm = a;
  op.row_split = a.a_layout == SIF_A_ROW_K && a.batch_outer * a.batch_inner == 1 && a.k_causal == 0 && !(a.epilogue & SIF_EPI_CAUSAL_SKIP);
  return op;
}

static void emit_gemm(Plan& p, const char* name, const G& g) { p.push_back(make_gemm_op(name, g.a)); }

// rows [r0, r0 + rows) of a product whose rows are independent
static sif_gemm_args gemm_row_range(const sif_gemm_args& g, uint32_t r0, uint32_t rows) {
  sif_gemm_args part = g;
  const size_t csz = (g.epilogue & SIF_EPI_OUT_F32) ? 4 : 2;
  part.m = rows;
  part.a_dev = (const bf16_t*)g.a_dev + (size_t)r0 * g.lda;
  part.c_dev = (unsigned char*)g.c_dev + (size_t)r0 * g.ldc * csz;
  if (g.res_dev) part.res_dev = (const unsigned char*)g.res_dev + (size_t)r0 * g.ldc * csz;
  if (g.aux_dev) part.aux_dev = (bf16_t*)g.aux_dev + (size_t)r0 * g.ldc;
  return part;
}

uint32_t gemm_round_rows(const sif_gemm_args& a) {
  // 256x256 tiles run one per CU, 128x128 tiles two per CU
  if (gemm_big_tiles(a)) return 256 * std::max(1u, 256u / ((a.n + 255) / 256));
  return 128 * std::max(1u, 512u / ((a.n + 127) / 128));
}

void split_gemm_rows(const Op& op, uint32_t rows_first, Op& first, Op& rest) {
  const sif_gemm_args& g = op.gemm;
  first = make_gemm_op(op.name, gemm_row_range(g, 0, rows_first));
  rest = make_gemm_op(op.name, gemm_row_range(g, rows_first, g.m - rows_first));
  const double share = (double)rows_first / (double)g.m;
  // each part pays the fixed part of a launch (prologue, epilogue, a last round that is not full) again, and a part of
  // one or two rounds of tiles runs a little below the rate of the whole
  first.cost_us = std::max(1.0, op.cost_us * share * 1.1) + 6.0;
  rest.cost_us = std::max(1.0, op.cost_us * (1.0 - share)) + 6.0;
}

// A GEMM whose rows are independent (A [M][K] row-major, C [M][N]) split into row ranges of at most
// `rows_per` rows (a multiple of the 128-row tile), so that no single launch exceeds the kernel time limit.
static void emit_gemm_rows(Plan& p, const char* name, const G& g, uint32_t kernel_us_max) {
  const double cost = gemm_cost_us(g.a);
  if (kernel_us_max == 0 || cost <= kernel_us_max || g.a.a_layout != SIF_A_ROW_K || g.a.batch_outer * g.a.batch_inner != 1 || g.a.m <= 128) {
    emit_gemm(p, name, g);
    return;
  }
  uint32_t pieces = (uint32_t)ceil(cost / kernel_us_max);
  uint32_t rows_per = ((g.a.m + pieces - 1) / pieces + 127) / 128 * 128;
  for (uint32_t r0 = 0; r0 < g.a.m; r0 += rows_per) {
    const uint32_t rows = (g.a.m - r0 < rows_per) ? g.a.m - r0 : rows_per;
    p.push_back(make_gemm_op(name, gemm_row_range(g.a, r0, rows)));
  }
}

static void emit(Plan& p, const char* name, double cost_us, std::function<sif_status(hipStream_t, const KCtl&)> fn) {
  Op op;
  op.name = name; op.cost_us = cost_us; op.fn = std::move(fn);
  p.push_back(std::move(op));
}

static void emit_bubble(Plan& p, int32_t site, uint64_t ns) {
  Op op;
  op.name = "bubble"; op.bubble_site = site; op.bubble_ns = ns; op.cost_us = ns / 1000.0;
  p.push_back(std::move(op));
}

// Weight gradient dW[m_out, n_out] = A^T B with A stored [tokens][m_out], B stored [tokens][n_out].
// K slices of a weight-gradient product: few output tiles (d x d .. d x 4d) but a long K (the tokens), so the
// product is cut along K into `splits` launches-in-one (a batch index) with fp32 partial results, summed afterwards.
// As many slices as fill one round of 128x128 tiles at two blocks per CU (at most 8: every slice writes and the sum
// reads m_out x n_out floats); a slice is a whole number of 64-wide K steps, the last one takes what is left
// (768 x 3072 over 8192 tokens: 3 slices of 2752, 2752, 2688 = 432 blocks, 50 us; 2 slices = 288 blocks, 61 us).
static uint32_t wgrad_splits(uint32_t m_out, uint32_t n_out, uint32_t tokens, uint32_t* kper_out = nullptr) {
  const uint32_t tiles = ((m_out + 127) / 128) * ((n_out + 127) / 128);
  const uint32_t want = std::min<uint32_t>(8, 512 / std::max<uint32_t>(1, tiles));
  uint32_t kper = tokens, splits = 1;
  if ((n_out & 7) == 0 && want >= 2 && tokens >= 256) {
    kper = ((tokens + want - 1) / want + 63) / 64 * 64;
    splits = (tokens + kper - 1) / kper;
    if (splits < 2) { kper = tokens; splits = 1; }
  }
  if (kper_out) *kper_out = kper;
  return splits;
}

// The partial results of all split products of a backward pass are summed by ONE launch at its end (RedPlan works
// like FinPlan below: the first pass emitted records the items, later passes reuse the buffers in the same order).
struct RedPlan {
  float* pool = nullptr;
  uint64_t pool_floats = 0, used = 0;
  std::vector<RedItem> items;
  RedItem* dev = nullptr;
  uint32_t max_items = 0;
  size_t cursor = 0;
  bool recorded = false, overflow = false;
  float* take(uint64_t n, uint32_t splits, bf16_t* out) {
    if (recorded) {
      if (cursor >= items.size()) { overflow = true; return pool; }
      return const_cast<float*>(items[cursor++].part);
    }
    if (used + n * splits > pool_floats || items.size() >= max_items) { overflow = true; return pool; }
    RedItem it;
    it.part = pool ? pool + used : nullptr; it.out = out; it.n = n; it.splits = splits; it.pad = 0;
    used += n * splits;
    items.push_back(it);
    return const_cast<float*>(it.part);
  }
};

static void emit_wgrad(Plan& p, const char* name, const bf16_t* a, const bf16_t* b, bf16_t* dw, uint32_t m_out, uint32_t n_out,
                       uint32_t tokens, RedPlan& rp, uint32_t acc) {
  uint32_t kper = tokens;
  const uint32_t splits = wgrad_splits(m_out, n_out, tokens, &kper);
  if (splits == 1) {
    G g(a, b, dw, m_out, n_out, tokens, m_out, n_out, n_out);
    g.lay(SIF_A_ROW_M, SIF_B_ROW_N);
    if (acc) g.epi(SIF_EPI_RESIDUAL, nullptr, dw);      // micro-batch accumulation: add to the stored gradient
    emit_gemm(p, name, g);
    return;
  }
  float* part = rp.take((uint64_t)m_out * n_out, splits, dw);
  emit_gemm(p, name, G(a, b, part, m_out, n_out, kper, m_out, n_out, n_out).lay(SIF_A_ROW_M, SIF_B_ROW_N).epi(SIF_EPI_OUT_F32)
                         .batch(1, splits, 0, (int64_t)kper * m_out, 0, (int64_t)kper * n_out, 0, (int64_t)m_out * n_out).k_limit(tokens));
}

// The four weight gradients of a layer as ONE launch (gemm_group_fill / launch_gemm_bf16_group): each by itself has too
// few 128x128 tiles for the chip and is cut along K above, with fp32 partial results written, read again and summed
// (1.25 GB per step of the 12-layer decoder); together they are 432 tiles over the whole K, no partial results.  The
// products' operands (the incoming gradient, dz, the gradient between the two halves of the layer, dqkv, the saved
// activations) are all still in place when the last of them, dqkv, has been computed.  GroupPlan hands out device
// memory for the launches' kernel records, which are written once, when the plan is built.
// A bias gradient (the column sums of a gradient over the tokens) rides along as one more product of the group: the
// left operand is `ones`, [tokens][8] with 1 in column 0, the result one row; its few tiles take block slots the weight
// gradients leave idle, and the launch that would read the gradient once more for the sums is not needed.
struct GroupPlan {
  unsigned char* pool = nullptr;
  uint64_t pool_bytes = 0, used = 0;
  const bf16_t* ones = nullptr;
  sif_status status = SIF_OK;
};
struct WgradItem { const bf16_t* a; const bf16_t* b; bf16_t* dw; uint32_t m_out, n_out, lda; };

static bool emit_wgrad_group(Plan& p, const char* name, const WgradItem* items, uint32_t n, uint32_t tokens, uint32_t acc, GroupPlan& gp) {
  const uint64_t bytes = gemm_group_bytes(n);
  if (gp.pool == nullptr || gp.used + bytes > gp.pool_bytes || n > 8) return false;
  sif_gemm_args list[8];
  double cost = 0.0, flops = 0.0;
  for (uint32_t i = 0; i < n; ++i) {
    if (items[i].n_out & 7) return false;
    G g(items[i].a, items[i].b, items[i].dw, items[i].m_out, items[i].n_out, tokens, items[i].lda, items[i].n_out, items[i].n_out);
    g.lay(SIF_A_ROW_M, SIF_B_ROW_N);
    if (acc) g.epi(SIF_EPI_RESIDUAL, nullptr, items[i].dw);      // micro-batch accumulation: add to the stored gradient
    list[i] = g.a;
    cost += gemm_cost_us(g.a) - 4.0;
    flops += gemm_flops(g.a);
  }
  std::vector<unsigned char> host(bytes);
  uint32_t grid = 0;
  if (gemm_group_fill(list, n, host.data(), &grid) != SIF_OK) return false;
  unsigned char* dev = gp.pool + gp.used;
  gp.used += (bytes + 255) & ~uint64_t(255);
  const hipError_t e = hipMemcpy(dev, host.data(), bytes, hipMemcpyHostToDevice);
  if (e != hipSuccess) { gp.status = fail_hip(e, "training plan: upload of a weight-gradient group"); return false; }
  Op op;
  op.name = name;
  op.fn = [dev, n, grid](hipStream_t s, const KCtl& c) { return launch_gemm_bf16_group(dev, n, grid, SIF_A_ROW_M, SIF_B_ROW_N, s, c); };
  op.cost_us = cost + 4.0;
  op.prof_class = (int32_t)(SIF_A_ROW_M * 2 + SIF_B_ROW_N);
  op.flops = flops;
  p.push_back(std::move(op));
  return true;
}

// Column sums (bias gradients) and the LayerNorm parameter gradients are computed as per-block partial sums by
// the kernel that reads the rows, and finalized by ONE launch at the end of a backward pass instead of one small
// launch each (49 per step of the 12-layer decoder).  FinPlan hands every producer its own partial buffer and
// collects what the batched finalize has to do.  The first backward pass that is emitted records the items; the
// passes emitted after it (further micro-batches) find the same producers in the same order and reuse the buffers.
struct FinPlan {
  float* pool = nullptr;          // partial sums of one backward pass
  uint64_t pool_floats = 0, used = 0;
  std::vector<FinItem> items;
  FinItem* dev = nullptr;         // the items on the device (uploaded when the plan is complete)
  uint32_t max_items = 0, max_n = 0;
  size_t cursor = 0;
  bool open = false, recorded = false, overflow = false;
  void begin() { open = true; cursor = 0; }
  // partial buffer for a producer of `nsum` sums over `n` columns
  float* take(uint32_t parts, uint32_t n, uint32_t nsum, bf16_t* o0, bf16_t* o1, bf16_t* o2) {
    if (recorded) {
      if (cursor >= items.size()) { overflow = true; return pool; }
      return const_cast<float*>(items[cursor++].part);
    }
    const uint64_t need = (uint64_t)parts * n * nsum;
    if (used + need > pool_floats || items.size() >= max_items) { overflow = true; return pool; }
    FinItem it;
    it.part = pool ? pool + used : nullptr; it.out[0] = o0; it.out[1] = o1; it.out[2] = o2;
    it.parts = parts; it.n = n; it.nsum = nsum; it.pad = 0;
    used += need;
    if (n > max_n) max_n = n;
    items.push_back(it);
    return const_cast<float*>(it.part);
  }
};

static void emit_colsum(Plan& p, const char* name, const void* x, uint32_t ld, void* out, FinPlan& fp, uint32_t rows, uint32_t n) {
  float* part = fp.take(colsum_parts(rows), n, 1, (bf16_t*)out, nullptr, nullptr);
  emit(p, name, bytes_cost_us(2.0 * rows * n), [=](hipStream_t s, const KCtl& c) { return launch_colsum_part(x, ld, part, rows, n, s, c); });
}

// dsum (may be null): gradient of the bias whose upstream gradient is this LayerNorm backward's output dx
static void emit_ln_bwd(Plan& p, const void* dy, const void* x, const void* g, const float* mean, const float* rstd, const void* res,
                        void* dx, void* dg, void* db, void* dsum, FinPlan& fp, uint32_t rows, uint32_t d) {
  const uint32_t ws = dsum != nullptr;
  float* part = fp.take(colsum_parts(rows), d, ws ? 3 : 2, (bf16_t*)dg, (bf16_t*)db, (bf16_t*)dsum);
  emit(p, "ln_bwd", bytes_cost_us(8.0 * rows * d), [=](hipStream_t s, const KCtl& c) { return launch_layernorm_bwd_dx(dy, x, g, mean, rstd, res, dx, part, rows, d, ws, s, c); });
}

// finalize launches for the producers [f0, f1) and the split products [r0, r1); acc: add to the stored gradients
// (micro-batch accumulation)
static void emit_fin_range(Plan& p, const FinPlan& fp, const RedPlan& rp, uint32_t acc, size_t f0, size_t f1, size_t r0, size_t r1) {
  if (f1 > f0) {
    const FinItem* dev = fp.dev + f0;
    const uint32_t n_items = (uint32_t)(f1 - f0), max_n = fp.max_n;
    emit(p, "grad_fin", 10.0, [=](hipStream_t s, const KCtl& c) { return launch_fin_batch(dev, n_items, max_n, acc, s, c); });
  }
  if (r1 > r0) {
    const RedItem* rdev = rp.dev + r0;
    const uint32_t rn = (uint32_t)(r1 - r0);
    double bytes = 0;
    for (size_t i = r0; i < r1; ++i) bytes += 4.0 * rp.items[i].n * rp.items[i].splits + 2.0 * rp.items[i].n;
    emit(p, "wgrad_sum", bytes_cost_us(bytes), [=](hipStream_t s, const KCtl& c) { return launch_reduce_splits_batch(rdev, rn, acc, s, c); });
  }
}

// the finalize launches of a whole backward pass (one of each kind)
static void emit_fin_batch(Plan& p, FinPlan& fp, RedPlan& rp, uint32_t acc) {
  emit_fin_range(p, fp, rp, acc, 0, fp.items.size(), 0, rp.items.size());
  fp.recorded = true;
  fp.open = false;
  rp.recorded = true;
  rp.cursor = 0;
}

// ------------------------------------------------------------------------------------------ transformer block
struct Dims { uint32_t B, S, M, d, H, dh, da, f, Sp; };

static Dims dims_of(const sif_model_shape& s, uint32_t batch, uint32_t seq) {
  Dims q;
  q.B = batch; q.S = seq; q.M = batch * seq; q.d = s.d_model; q.H = s.n_heads; q.dh = s.d_head; q.da = s.n_heads * s.d_head;
  q.f = s.d_ffn; q.Sp = (seq + 7) & ~7u;
  return q;
}

// Attention for all (batch, head) pairs: scores (fp32) = scale q k^T, prob = softmax, o = prob v.
static void emit_attention_fwd(Plan& p, const Dims& q, const bf16_t* qkv, float* scores, bf16_t* prob, bf16_t* o, bool causal) {
  const int64_t ss = (int64_t)q.S * q.Sp;
  const float scale = 1.0f / sqrtf((float)q.dh);
  emit_gemm(p, "attn_scores", G(qkv, qkv + q.da, scores, q.S, q.S, q.dh, 3 * q.da, 3 * q.da, q.Sp)
                                  .epi(SIF_EPI_OUT_F32 | (causal ? SIF_EPI_CAUSAL_SKIP : 0)).alpha(scale)
                                  .batch(q.B, q.H, (int64_t)q.S * 3 * q.da, q.dh, (int64_t)q.S * 3 * q.da, q.dh, q.H * ss, ss));
  const uint32_t bh = q.B * q.H, S = q.S, Sp = q.Sp, c = causal ? 1 : 0;
  emit(p, "attn_softmax", bytes_cost_us(6.0 * bh * S * Sp * (causal ? 0.5 : 1.0)),
       [=](hipStream_t s, const KCtl& k) { return launch_softmax_fwd(scores, prob, bh, S, S, Sp, Sp, c, s, k); });
  emit_gemm(p, "attn_pv", G(prob, qkv + 2 * q.da, o, q.S, q.dh, q.S, q.Sp, 3 * q.da, q.da).lay(SIF_A_ROW_K, SIF_B_ROW_N)
                              .causal(causal ? 1 : 0)
                              .batch(q.B, q.H, q.H * ss, ss, (int64_t)q.S * 3 * q.da, q.dh, (int64_t)q.S * q.da, q.dh));
}

// dqkv from do, the saved probabilities and qkv.  dp (fp32) and ds (bf16) are scratch [B*H][S][Sp].
static void emit_attention_bwd(Plan& p, const Dims& q, const bf16_t* qkv, const bf16_t* prob, const bf16_t* d_o, float* dp, bf16_t* ds,
                               bf16_t* dqkv) {
  const int64_t ss = (int64_t)q.S * q.Sp, row3 = (int64_t)q.S * 3 * q.da, row1 = (int64_t)q.S * q.da;
  const float scale = 1.0f / sqrtf((float)q.dh);
  emit_gemm(p, "attn_dv", G(prob, d_o, dqkv + 2 * q.da, q.S, q.dh, q.S, q.Sp, q.da, 3 * q.da).lay(SIF_A_ROW_M, SIF_B_ROW_N).causal(2)
                              .batch(q.B, q.H, q.H * ss, ss, row1, q.dh, row3, q.dh));
  emit_gemm(p, "attn_dp", G(d_o, qkv + 2 * q.da, dp, q.S, q.S, q.dh, q.da, 3 * q.da, q.Sp).epi(SIF_EPI_OUT_F32 | SIF_EPI_CAUSAL_SKIP)
                              .batch(q.B, q.H, row1, q.dh, row3, q.dh, q.H * ss, ss));
  const uint32_t bh = q.B * q.H, S = q.S, Sp = q.Sp;
  emit(p, "attn_softmax_bwd", bytes_cost_us(4.0 * bh * S * Sp),
       [=](hipStream_t s, const KCtl& k) { return launch_softmax_bwd(dp, prob, ds, bh, S, S, Sp, scale, 1, s, k); });
  emit_gemm(p, "attn_dq", G(ds, qkv + q.da, dqkv, q.S, q.dh, q.S, q.Sp, 3 * q.da, 3 * q.da).lay(SIF_A_ROW_K, SIF_B_ROW_N).causal(1)
                              .batch(q.B, q.H, q.H * ss, ss, row3, q.dh, row3, q.dh));
  emit_gemm(p, "attn_dk", G(ds, qkv, dqkv + q.da, q.S, q.dh, q.S, q.Sp, 3 * q.da, 3 * q.da).lay(SIF_A_ROW_M, SIF_B_ROW_N).causal(2)
                              .batch(q.B, q.H, q.H * ss, ss, row3, q.dh, row3, q.dh));
}

struct LayerActs {       // saved by the forward pass of one decoder layer (prob: unfused attention, lse: fused)
  bf16_t *ln1, *qkv, *prob, *o, *x_mid, *ln2, *z, *a, *x_out;
  float *m1, *r1, *m2, *r2, *lse;
};
// head sizes the fused attention kernels are built for; other sizes take the three-launch path through HBM
static bool fused_attention(uint32_t dh) { return dh == 64 || dh == 128; }
static double attn_fused_cost_us(const Dims& q, double products, bool causal) {
  return 4.0 + products * 2.0 * q.B * q.H * (double)q.S * q.S * q.dh * (causal ? 0.55 : 1.0) / 2.0e8;      // 200 TFLOP/s plus launch latency
}
struct LayerW { const bf16_t *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o, *ln2_g, *ln2_b, *w_fc, *b_fc, *w_proj, *b_proj; };
struct LayerG { bf16_t *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o, *ln2_g, *ln2_b, *w_fc, *b_fc, *w_proj, *b_proj; };

template <typename T, typename P>
static T layer_ptrs(P* base, const ParamMap& pm, uint32_t l) {
  T w;
  w.ln1_g = base + pm.at(L(l, "ln1_g")); w.ln1_b = base + pm.at(L(l, "ln1_b")); w.w_qkv = base + pm.at(L(l, "w_qkv"));
  w.b_qkv = base + pm.at(L(l, "b_qkv")); w.w_o = base + pm.at(L(l, "w_o")); w.b_o = base + pm.at(L(l, "b_o"));
  w.ln2_g = base + pm.at(L(l, "ln2_g")); w.ln2_b = base + pm.at(L(l, "ln2_b")); w.w_fc = base + pm.at(L(l, "w_fc"));
  w.b_fc = base + pm.at(L(l, "b_fc")); w.w_proj = base + pm.at(L(l, "w_proj")); w.b_proj = base + pm.at(L(l, "b_proj"));
  return w;
}

struct TpSites { bool on; uint64_t ns; int32_t* next; };

static void emit_decoder_layer_fwd(Plan& p, const Dims& q, const LayerW& w, const bf16_t* x_in, const LayerActs& a, const Scratch& sc,
                                   const TpSites& tp) {
  const uint32_t M = q.M, d = q.d;
  emit(p, "ln1", bytes_cost_us(4.0 * M * d), [=](hipStream_t s, const KCtl& c) { return launch_layernorm_fwd(x_in, w.ln1_g, w.ln1_b, a.ln1, a.m1, a.r1, M, d, s, c); });
  emit_gemm(p, "qkv", G(a.ln1, w.w_qkv, a.qkv, M, 3 * q.da, d, d, d, 3 * q.da).epi(SIF_EPI_BIAS, w.b_qkv));
  if (fused_attention(q.dh)) {
    const uint32_t B = q.B, S = q.S, H = q.H, dh = q.dh, da = q.da;
    emit(p, "attn_fused", attn_fused_cost_us(q, 2, true),
         [=](hipStream_t s, const KCtl& c) { return launch_attn_fwd(a.qkv, a.o, a.lse, B, S, H, dh, 3 * da, da, 1, s, c); });
  } else {
    emit_attention_fwd(p, q, a.qkv, sc.scores, a.prob, a.o, true);
  }
  emit_gemm(p, "attn_out", G(a.o, w.w_o, a.x_mid, M, d, q.da, q.da, q.da, d).epi(SIF_EPI_BIAS | SIF_EPI_RESIDUAL, w.b_o, x_in));
  if (tp.on) emit_bubble(p, (*tp.next)++, tp.ns);
  emit(p, "ln2", bytes_cost_us(4.0 * M * d), [=](hipStream_t s, const KCtl& c) { return launch_layernorm_fwd(a.x_mid, w.ln2_g, w.ln2_b, a.ln2, a.m2, a.r2, M, d, s, c); });
  emit_gemm(p, "mlp_up", G(a.ln2, w.w_fc, a.a, M, q.f, d, d, d, q.f).epi(SIF_EPI_GELU, w.b_fc, nullptr, a.z));
  emit_gemm(p, "mlp_down", G(a.a, w.w_proj, a.x_out, M, d, q.f, q.f, q.f, d).epi(SIF_EPI_BIAS | SIF_EPI_RESIDUAL, w.b_proj, a.x_mid));
  if (tp.on) emit_bubble(p, (*tp.next)++, tp.ns);
}

// dx_out -> dx_in (both bf16 [M,d]); gradients of the layer's parameters into g.  `tmp` is a second [M,d] buffer.
// The gradients of b_proj and b_o are column sums of dx_out and dx_mid, which LayerNorm backward kernels write:
// they come from those kernels.  have_db_proj: the producer of dx_out has already written g.b_proj;
// db_proj_below: where this layer's last kernel puts the b_proj gradient of the layer below (null: none).
static void emit_decoder_layer_bwd(Plan& p, const Dims& q, const LayerW& w, const LayerG& g, const bf16_t* x_in, const LayerActs& a,
                                   const Scratch& sc, const bf16_t* dx_out, bf16_t* dx_mid, bf16_t* dx_in, const TpSites& tp, uint32_t acc,
                                   bool have_db_proj, bf16_t* db_proj_below, FinPlan& fp, RedPlan& rp, GroupPlan& gp) {
  const uint32_t M = q.M, d = q.d, f = q.f, da = q.da;
  // the layer's weight gradients as one launch where that can be had (below, once dqkv is there), else one by one
  // (with them the gradients of b_fc and b_qkv, where the plan has the operand for that)
  const WgradItem wg[6] = {{dx_out, a.a, g.w_proj, d, f, d}, {sc.dz, a.ln2, g.w_fc, f, d, f}, {dx_mid, a.o, g.w_o, d, da, d},
                           {sc.dqkv, a.ln1, g.w_qkv, 3 * da, d, 3 * da}, {gp.ones, sc.dz, g.b_fc, 1, f, 8}, {gp.ones, sc.dqkv, g.b_qkv, 1, 3 * da, 8}};
  const uint32_t n_group = gp.ones != nullptr ? 6 : 4;
  const bool grouped = gp.pool != nullptr && gp.used + gemm_group_bytes(n_group) <= gp.pool_bytes && !((f | d | da) & 7);
  const bool bias_grouped = grouped && n_group == 6;
  if (!have_db_proj) emit_colsum(p, "db_proj", dx_out, d, g.b_proj, fp, M, d);
  if (!grouped) emit_wgrad(p, "dw_proj", dx_out, a.a, g.w_proj, d, f, M, rp, acc);
  emit_gemm(p, "dz", G(dx_out, w.w_proj, sc.dz, M, f, d, d, f, f).lay(SIF_A_ROW_K, SIF_B_ROW_N).epi(SIF_EPI_GELU_GRAD, nullptr, nullptr, a.z));
  if (!bias_grouped) emit_colsum(p, "db_fc", sc.dz, f, g.b_fc, fp, M, f);
  if (!grouped) emit_wgrad(p, "dw_fc", sc.dz, a.ln2, g.w_fc, f, d, M, rp, acc);
  emit_gemm(p, "dln2", G(sc.dz, w.w_fc, sc.dln, M, d, f, f, d, d).lay(SIF_A_ROW_K, SIF_B_ROW_N));
  if (tp.on) emit_bubble(p, (*tp.next)++, tp.ns);
  emit_ln_bwd(p, sc.dln, a.x_mid, w.ln2_g, a.m2, a.r2, dx_out, dx_mid, g.ln2_g, g.ln2_b, g.b_o, fp, M, d);
  if (!grouped) emit_wgrad(p, "dw_o", dx_mid, a.o, g.w_o, d, da, M, rp, acc);
  emit_gemm(p, "do", G(dx_mid, w.w_o, sc.d_o, M, da, d, d, da, da).lay(SIF_A_ROW_K, SIF_B_ROW_N));
  if (fused_attention(q.dh)) {
    const uint32_t B = q.B, S = q.S, H = q.H, dh = q.dh;
    emit(p, "attn_bwd_dq", attn_fused_cost_us(q, 3, true), [=](hipStream_t s, const KCtl& c) {
      return launch_attn_bwd_dq(a.qkv, a.o, sc.d_o, a.lse, sc.delta, sc.dqkv, B, S, H, dh, 3 * da, da, 3 * da, 1, s, c);
    });
    emit(p, "attn_bwd_dkv", attn_fused_cost_us(q, 4, true), [=](hipStream_t s, const KCtl& c) {
      return launch_attn_bwd_dkv(a.qkv, sc.d_o, a.lse, sc.delta, sc.dqkv, B, S, H, dh, 3 * da, da, 3 * da, 1, s, c);
    });
  } else {
    emit_attention_bwd(p, q, a.qkv, a.prob, sc.d_o, sc.scores, sc.ds, sc.dqkv);
  }
  if (!bias_grouped) emit_colsum(p, "db_qkv", sc.dqkv, 3 * da, g.b_qkv, fp, M, 3 * da);
  if (grouped) {
    if (!emit_wgrad_group(p, "dw_layer", wg, n_group, M, acc, gp) && gp.status == SIF_OK)
      gp.status = fail(SIF_E_INVAL, "training plan: the weight gradients of a layer could not be set up as one launch");
  } else {
    emit_wgrad(p, "dw_qkv", sc.dqkv, a.ln1, g.w_qkv, 3 * da, d, M, rp, acc);
  }
  emit_gemm(p, "dln1", G(sc.dqkv, w.w_qkv, sc.dln, M, d, 3 * da, 3 * da, d, d).lay(SIF_A_ROW_K, SIF_B_ROW_N));
  if (tp.on) emit_bubble(p, (*tp.next)++, tp.ns);
  emit_ln_bwd(p, sc.dln, x_in, w.ln1_g, a.m1, a.r1, dx_mid, dx_in, g.ln1_g, g.ln1_b, db_proj_below, fp, M, d);
}

// ------------------------------------------------------------------------------------------ training models
static void put(TrainModel& tm, const std::string& name, void* p, uint64_t elems) { tm.tensors[name] = NamedTensor{p, elems}; }

static sif_status build_mlp_train(TrainModel& tm, Arena& ar) {
  const sif_model_shape& s = tm.desc.shape;
  const ParamMap pm = param_map(s);
  const uint32_t B = s.batch, di = s.d_in, dh = s.d_hidden, dout = s.d_out;
  float* W = tm.desc.master_dev;
  float* grads = (float*)ar.take(pm.n * 4);
  float* z = (float*)ar.take((uint64_t)B * dh * 4);
  float* h = (float*)ar.take((uint64_t)B * dh * 4);
  float* y = (float*)ar.take((uint64_t)B * dout * 4);
  float* dy = (float*)ar.take((uint64_t)B * dout * 4);
  float* dz = (float*)ar.take((uint64_t)B * dh * 4);
  float* loss = (float*)ar.take(256);
  tm.workspace_bytes = ar.off;
  if (!ar.base) return SIF_OK;
  put(tm, "work", W, pm.n); put(tm, "grads", grads, pm.n); put(tm, "z", z, (uint64_t)B * dh); put(tm, "a", h, (uint64_t)B * dh);
  put(tm, "y", y, (uint64_t)B * dout); put(tm, "loss", loss, 1);
  float *w1 = W + pm.at("w1"), *b1 = W + pm.at("b1"), *w2 = W + pm.at("w2"), *b2 = W + pm.at("b2");
  float *gw1 = grads + pm.at("w1"), *gb1 = grads + pm.at("b1"), *gw2 = grads + pm.at("w2"), *gb2 = grads + pm.at("b2");
  TrainModel* t = &tm;
  Plan& p = tm.plan;
  emit(p, "fc1", 5, [=](hipStream_t st, const KCtl& c) { return launch_gemm_f32((const float*)t->cur_inputs, di, 1, w1, 1, di, h, dh, B, dh, di, SIF_EPI_GELU, b1, z, st, c); });
  emit(p, "fc2", 5, [=](hipStream_t st, const KCtl& c) { return launch_gemm_f32(h, dh, 1, w2, 1, dh, y, dout, B, dout, dh, SIF_EPI_BIAS, b2, nullptr, st, c); });
  emit(p, "mse", 4, [=](hipStream_t st, const KCtl& c) { return launch_mse(y, (const float*)t->cur_targets, dy, t->cur_loss ? t->cur_loss : loss, B * dout, st, c); });
  emit(p, "dw2", 5, [=](hipStream_t st, const KCtl& c) { return launch_gemm_f32(dy, 1, dout, h, dh, 1, gw2, dh, dout, dh, B, 0, nullptr, nullptr, st, c); });
  emit(p, "db2", 4, [=](hipStream_t st, const KCtl& c) { return launch_colsum_f32(dy, dout, gb2, B, dout, st, c); });
  emit(p, "dz", 5, [=](hipStream_t st, const KCtl& c) { return launch_gemm_f32(dy, dout, 1, w2, dh, 1, dz, dh, B, dh, dout, SIF_EPI_GELU_GRAD, nullptr, z, st, c); });
  emit(p, "dw1", 5, [=](hipStream_t st, const KCtl& c) { return launch_gemm_f32(dz, 1, dh, (const float*)t->cur_inputs, di, 1, gw1, di, dh, di, B, 0, nullptr, nullptr, st, c); });
  emit(p, "db1", 4, [=](hipStream_t st, const KCtl& c) { return launch_colsum_f32(dz, dh, gb1, B, dh, st, c); });
  if (tm.desc.par_mode == SIF_PAR_FIXED && tm.desc.fixed_bubble_ns) emit_bubble(p, 0, tm.desc.fixed_bubble_ns);
  const uint64_t n = pm.n;
  const float lr = tm.desc.lr;
  emit(p, "sgd", 4, [=](hipStream_t st, const KCtl& c) { return launch_sgd_f32(W, grads, n, lr, st, c); });
  return SIF_OK;
}

static sif_status build_decoder_train(TrainModel& tm, Arena& ar, hipStream_t stream) {
  const sif_model_shape& s = tm.desc.shape;
  const ParamMap pm = param_map(s);
  const Dims q = dims_of(s, s.batch, s.seq);
  // Row pitch of the logits: the vocabulary rounded up to 8 columns, for a large vocabulary to whole 64-wide K steps, so
  // that the LM head's data gradient, which contracts the logits' columns, can be cut into slices of whole K steps.
  const uint32_t M = q.M, d = q.d, Vp = s.vocab >= 8192 ? (s.vocab + 63) & ~63u : (s.vocab + 7) & ~7u;
  const uint64_t ssz = (uint64_t)q.B * q.H * q.S * q.Sp;
  const bool fused = fused_attention(q.dh);
  const bool pp = tm.desc.par_mode == SIF_PAR_PP;
  // pipeline stage: n_micro micro-batches per step; a 1F1B stage holds the activations of at most
  // (stages - stage) micro-batches at a time, so that many activation slots are enough
  const uint32_t n_micro = pp ? tm.desc.pp_micro : 1;
  const uint32_t n_slots = pp ? std::min(n_micro, tm.desc.pp_stages - tm.desc.pp_stage) : 1;
  bf16_t* work = (bf16_t*)ar.take(pm.n * 2);
  bf16_t* grads = (bf16_t*)ar.take(pm.n * 2);
  std::vector<std::vector<LayerActs>> acts(n_slots, std::vector<LayerActs>(s.n_layers));
  std::vector<bf16_t*> x0(n_slots);
  for (uint32_t sl = 0; sl < n_slots; ++sl) {
    x0[sl] = (bf16_t*)ar.take((uint64_t)M * d * 2);
    for (auto& a : acts[sl]) {
      a.ln1 = (bf16_t*)ar.take((uint64_t)M * d * 2); a.qkv = (bf16_t*)ar.take((uint64_t)M * 3 * q.da * 2);
      a.prob = fused ? nullptr : (bf16_t*)ar.take(ssz * 2);
      a.lse = fused ? (float*)ar.take((uint64_t)q.B * q.H * q.S * 4) : nullptr;
      a.o = (bf16_t*)ar.take((uint64_t)M * q.da * 2);
      a.x_mid = (bf16_t*)ar.take((uint64_t)M * d * 2); a.ln2 = (bf16_t*)ar.take((uint64_t)M * d * 2);
      a.z = (bf16_t*)ar.take((uint64_t)M * q.f * 2); a.a = (bf16_t*)ar.take((uint64_t)M * q.f * 2);
      a.x_out = (bf16_t*)ar.take((uint64_t)M * d * 2);
      a.m1 = (float*)ar.take((uint64_t)M * 4); a.r1 = (float*)ar.take((uint64_t)M * 4);
      a.m2 = (float*)ar.take((uint64_t)M * 4); a.r2 = (float*)ar.take((uint64_t)M * 4);
    }
  }
  Scratch sc;
  sc.scores = fused ? nullptr : (float*)ar.take(ssz * 4);
  sc.ds = fused ? nullptr : (bf16_t*)ar.take(ssz * 2);
  sc.delta = fused ? (float*)ar.take((uint64_t)q.B * q.H * q.S * 4) : nullptr;
  sc.dx_a = (bf16_t*)ar.take((uint64_t)M * d * 2); sc.dx_b = (bf16_t*)ar.take((uint64_t)M * d * 2);
  sc.dln = (bf16_t*)ar.take((uint64_t)M * d * 2); sc.dqkv = (bf16_t*)ar.take((uint64_t)M * 3 * q.da * 2);
  sc.d_o = (bf16_t*)ar.take((uint64_t)M * q.da * 2); sc.dz = (bf16_t*)ar.take((uint64_t)M * q.f * 2);
  // partial sums of one backward pass: per layer two LayerNorm backwards (three sums over d each), the fc and qkv
  // bias gradients, and one more LayerNorm backward (final LayerNorm) or column sum (top of a stack)
  FinPlan fp;
  fp.max_items = 4 * s.n_layers + 2;
  fp.pool_floats = (uint64_t)colsum_parts(M) * ((uint64_t)s.n_layers * (6 * d + q.f + 3 * q.da) + 3 * d);
  fp.pool = (float*)ar.take(fp.pool_floats * 4);
  fp.dev = (FinItem*)ar.take((uint64_t)fp.max_items * sizeof(FinItem));
  // the weight gradients: one launch per layer and backward pass where the widths allow it (then there are no K slices
  // to sum, and no buffer for them), else each product by itself, cut along K
  GroupPlan gp;
  const bool group_wgrads = !((q.f | d | q.da) & 7);
  if (group_wgrads) {
    // (a pipeline stage emits one backward pass per micro-batch and one more to estimate its duration)
    gp.pool_bytes = (uint64_t)s.n_layers * (pp ? tm.desc.pp_micro + 1 : 1) * ((gemm_group_bytes(6) + 255) & ~uint64_t(255));
    gp.pool = (unsigned char*)ar.take(gp.pool_bytes);
    bf16_t* ones = (bf16_t*)ar.take((uint64_t)M * 8 * 2);
    if (ones != nullptr) {
      std::vector<uint16_t> h((size_t)M * 8, 0);
      for (uint32_t t = 0; t < M; ++t) h[(size_t)t * 8] = 0x3F80;      // bf16 1.0
      const hipError_t e = hipMemcpy(ones, h.data(), h.size() * 2, hipMemcpyHostToDevice);
      if (e != hipSuccess) return fail_hip(e, "training plan: upload of the bias-gradient operand");
      gp.ones = ones;
    }
  }
  RedPlan rp;
  rp.max_items = 4 * s.n_layers;
  if (!group_wgrads) {
    const uint32_t da = q.da, f = q.f;
    const uint64_t per_layer = (uint64_t)d * f * wgrad_splits(d, f, M) + (uint64_t)f * d * wgrad_splits(f, d, M) +
                               (uint64_t)d * da * wgrad_splits(d, da, M) + (uint64_t)3 * da * d * wgrad_splits(3 * da, d, M);
    rp.pool_floats = per_layer * s.n_layers;
  }
  rp.pool = (float*)ar.take(rp.pool_floats * 4);
  rp.dev = (RedItem*)ar.take((uint64_t)rp.max_items * sizeof(RedItem));
  bf16_t *lnf = nullptr, *logits = nullptr, *y_all = nullptr, *dx_all = nullptr;
  float *mf = nullptr, *rf = nullptr, *loss_tok = nullptr, *loss = nullptr;
  // The LM head's data gradient [M][d] contracts the whole vocabulary: few output tiles and a very long K.  It is cut
  // along K into slices whose tiles fill whole rounds of block slots, summed by one small launch right behind it.
  // Where the padded vocabulary can be contracted as a whole (its padding columns are zero in the loss gradient and
  // the rows of the working copy behind wte stand in for the padding rows, as for the forward product), the slices can
  // be whole numbers of K steps and the product can take the 256x256 tiles, one block per CU: as many slices as fill
  // whole rounds of 256 blocks (8192 x 768 over 50304: 96 tiles x 8 slices of 99, ..., 93 steps = three rounds).
  uint32_t head_splits = 1, head_kper = 0, head_k = s.vocab;
  float* head_part = nullptr;
  RedItem* head_item = nullptr;
  if (s.vocab) {
    const uint32_t tiles = ((M + 127) / 128) * ((d + 127) / 128);
    double best = 0.0;
    for (uint32_t k = 1; k <= 8 && tiles < 512 && s.vocab >= 8192; ++k) {
      const double fill = (double)tiles * k / (512.0 * ((tiles * k + 511) / 512));      // share of the rounds' slots in use
      if (fill > best * 1.02) { best = fill; head_splits = k; }
    }
    if (head_splits > 1) {
      head_kper = ((s.vocab + head_splits - 1) / head_splits + 63) / 64 * 64;
      if ((uint64_t)(head_splits - 1) * head_kper >= s.vocab) head_splits = 1;
    }
    const uint32_t tiles_big = ((M + 255) / 256) * ((d + 255) / 256), steps = Vp / 64;
    if (head_splits > 1 && Vp - s.vocab <= s.max_pos && (Vp % 64) == 0 && (d % 8) == 0 && tiles_big < 256) {
      uint32_t k_big = 1;
      double best_big = 0.0;
      for (uint32_t k = 1; k <= 16 && k <= steps; ++k) {
        const double fill = (double)tiles_big * k / (256.0 * ((tiles_big * k + 255) / 256));
        if (fill > best_big * 1.02) { best_big = fill; k_big = k; }
      }
      const uint32_t kper_big = (steps + k_big - 1) / k_big * 64;
      // the launcher's timing model for the two configurations, plus what the sum of the slices reads
      const double t_small = (1.0 + 1.19 * (head_kper / 64.0)) * std::max(0.85, (double)tiles * head_splits / 512.0) + bytes_cost_us(4.0 * M * d * head_splits);
      const double t_big = (4.0 + 1.75 * (kper_big / 64.0)) * (double)((tiles_big * k_big + 255) / 256) + bytes_cost_us(4.0 * M * d * k_big);
      if (k_big > 1 && (uint64_t)(k_big - 1) * kper_big < Vp && t_big < t_small) { head_splits = k_big; head_kper = kper_big; head_k = Vp; }
    }
    if (head_splits > 1) {
      head_part = (float*)ar.take((uint64_t)head_splits * M * d * 4);
      head_item = (RedItem*)ar.take(sizeof(RedItem));
    }
  }
  // The LM head's weight gradient [V][d] over K = the tokens, on 256x256 tiles with one block per CU: a last round
  // that few of the CUs take part in costs as much as a full one (50257 x 768: 591 tiles = 2.3 rounds, paid as three).
  // The tile rows of the whole rounds are then one launch and the rest a second one, cut along K into as many slices
  // as still fit one round, with fp32 partial results that a small launch sums (510 tiles, then 81 tiles x 3 slices).
  uint32_t wte_tail_row0 = 0, wte_tail_rows = 0, wte_tail_splits = 1, wte_tail_kper = 0;
  float* wte_tail_part = nullptr;
  RedItem* wte_tail_item = nullptr;
  if (s.vocab && (M % 64) == 0 && (d % 8) == 0) {
    const uint32_t tm_all = (s.vocab + 255) / 256, tn_all = (d + 255) / 256, tiles_all = tm_all * tn_all, steps = M / 64;
    const uint32_t main_tm = tiles_all / 256 * 256 / tn_all, tail_tm = tm_all - main_tm;
    if (tiles_all > 256 && main_tm > 0 && tail_tm > 0 && tail_tm * tn_all <= 128) {
      uint32_t k = std::min<uint32_t>(std::min<uint32_t>(8u, 256u / (tail_tm * tn_all)), steps);
      const uint32_t kper = (steps + k - 1) / k * 64;
      while (k > 1 && (uint64_t)(k - 1) * kper >= M) --k;
      const uint32_t rows = s.vocab - main_tm * 256;
      // the launcher's timing model: one more whole round against a round of K / k steps and the sum of the slices
      const double t_whole = 4.0 + 1.75 * steps, t_cut = 4.0 + 1.75 * (kper / 64.0) + bytes_cost_us(4.0 * rows * d * k) + 8.0;
      if (k > 1 && t_cut < 0.8 * t_whole) {
        wte_tail_row0 = main_tm * 256; wte_tail_rows = rows; wte_tail_splits = k; wte_tail_kper = kper;
        wte_tail_part = (float*)ar.take((uint64_t)k * rows * d * 4);
        wte_tail_item = (RedItem*)ar.take(sizeof(RedItem));
      }
    }
  }
  if (s.vocab) {
    lnf = (bf16_t*)ar.take((uint64_t)M * d * 2);
    logits = (bf16_t*)ar.take((uint64_t)M * Vp * 2);
    mf = (float*)ar.take((uint64_t)M * 4); rf = (float*)ar.take((uint64_t)M * 4);
    loss_tok = (float*)ar.take((uint64_t)M * 4); loss = (float*)ar.take(256);
  }
  if (pp) {
    y_all = (bf16_t*)ar.take((uint64_t)n_micro * M * d * 2);
    dx_all = (bf16_t*)ar.take((uint64_t)n_micro * M * d * 2);
  }
  tm.workspace_bytes = ar.off;
  if (!ar.base) return SIF_OK;

  put(tm, "work", work, pm.n); put(tm, "grads", grads, pm.n);
  for (uint32_t l = 0; l < s.n_layers; ++l) {      // named tensors refer to activation slot 0
    const LayerActs& a = acts[0][l];
    const std::string sfx = "." + std::to_string(l);
    put(tm, "ln1" + sfx, a.ln1, (uint64_t)M * d); put(tm, "qkv" + sfx, a.qkv, (uint64_t)M * 3 * q.da); if (fused) put(tm, "lse" + sfx, a.lse, (uint64_t)q.B * q.H * q.S); else put(tm, "prob" + sfx, a.prob, ssz);
    put(tm, "o" + sfx, a.o, (uint64_t)M * q.da); put(tm, "x_mid" + sfx, a.x_mid, (uint64_t)M * d); put(tm, "ln2" + sfx, a.ln2, (uint64_t)M * d);
    put(tm, "z" + sfx, a.z, (uint64_t)M * q.f); put(tm, "a" + sfx, a.a, (uint64_t)M * q.f); put(tm, "x_out" + sfx, a.x_out, (uint64_t)M * d);
  }
  put(tm, "x0", x0[0], (uint64_t)M * d);
  put(tm, "dx_in", sc.dx_a, (uint64_t)M * d);
  if (s.vocab) { put(tm, "logits", logits, (uint64_t)M * Vp); put(tm, "lnf", lnf, (uint64_t)M * d); put(tm, "loss", loss, 1); }
  if (pp) { put(tm, "y_all", y_all, (uint64_t)n_micro * M * d); put(tm, "dx_all", dx_all, (uint64_t)n_micro * M * d); }

  // gradients of position rows beyond seq are never written: clear the gradient buffer once
  hipError_t e = hipMemsetAsync(grads, 0, pm.n * 2, stream);
  if (e != hipSuccess) return fail_hip(e, "register: clear gradients");
  sif_status st = launch_sgd_bf16(tm.desc.master_dev, nullptr, work, pm.n, 0.f, stream, no_ctl());
  if (st != SIF_OK) return st;

  int32_t next_site = 0;
  TpSites tp{false, 0, &next_site};
  if (tm.desc.par_mode == SIF_PAR_TP) {
    tp.on = true;
    tp.ns = sif_collective_ns((uint64_t)M * d * 2, tm.desc.bw_bytes_per_s);
    tm.max_bubble_ns = tp.ns;
  }
  TrainModel* t = &tm;
  const uint32_t seq = q.S, V = s.vocab;
  const uint64_t mb_bytes = (uint64_t)M * d * 2;

  // Bucketed gradient exchange beside backward: the gradient groups in the order they become final (the layers from
  // the last to the first, the final LayerNorm with the last layer; then the embeddings), their buckets, and per
  // bucket the op that finalizes it (filled in while the plan is emitted).
  const bool overlap = tm.desc.par_mode == SIF_PAR_DP && tm.desc.dp_bucket_bytes > 0;
  std::vector<uint64_t> group_bytes;
  std::vector<uint32_t> bucket_of;
  uint32_t n_buckets = 0;
  tm.dp_buckets.clear();
  if (overlap) {
    const uint64_t emb = s.vocab ? ((uint64_t)s.vocab + s.max_pos) * d : 0, lnf_n = s.vocab ? 2ull * d : 0;
    const uint64_t per_layer = (pm.n - emb - lnf_n) / s.n_layers;
    for (uint32_t l = 0; l < s.n_layers; ++l) group_bytes.push_back(2 * (per_layer + (l == 0 ? lnf_n : 0)));
    if (s.vocab) group_bytes.push_back(2 * emb);
    bucket_of.resize(group_bytes.size());
    const int32_t nb = sif_dp_gradient_buckets(group_bytes.data(), (uint32_t)group_bytes.size(), tm.desc.dp_bucket_bytes, bucket_of.data());
    if (nb < 0) return (sif_status)nb;
    if ((uint32_t)nb > kMaxDpBuckets) return fail(SIF_E_INVAL, "dp_bucket_bytes gives %d buckets, at most %u are supported", nb, kMaxDpBuckets);
    n_buckets = (uint32_t)nb;
    tm.dp_buckets.assign(n_buckets, TrainModel::DpBucket{0, 0, 0});
    for (size_t g = 0; g < group_bytes.size(); ++g) tm.dp_buckets[bucket_of[g]].bytes += group_bytes[g];
    for (auto& b : tm.dp_buckets) b.dur_ns = sif_collective_ns(b.bytes, tm.desc.bw_bytes_per_s);
  }
  auto closes_bucket = [&](size_t g) { return g + 1 == group_bytes.size() || bucket_of[g + 1] != bucket_of[g]; };

  // forward pass of micro-batch k into activation slot k % n_slots
  auto emit_forward = [&](Plan& p, uint32_t k) {
    const uint32_t sl = k % n_slots;
    bf16_t* xin0 = x0[sl];
    if (s.vocab) {
      const bf16_t *wte = work + pm.at("wte"), *wpe = work + pm.at("wpe");
      emit(p, "embed", bytes_cost_us(6.0 * M * d), [=](hipStream_t s2, const KCtl& c) { return launch_embed_fwd((const int32_t*)t->cur_inputs, wte, wpe, xin0, V, M, seq, d, s2, c); });
    } else {
      // layer stack: the caller's activations become the input of the first layer
      emit(p, "stage_x", bytes_cost_us(2.0 * mb_bytes), [=](hipStream_t s2, const KCtl& c) {
        return launch_copy(xin0, (const unsigned char*)t->cur_inputs + (size_t)k * mb_bytes, mb_bytes, s2, c); });
    }
    const bf16_t* x_in = xin0;
    for (uint32_t l = 0; l < s.n_layers; ++l) {
      const LayerW w = layer_ptrs<LayerW, const bf16_t>(work, pm, l);
      emit_decoder_layer_fwd(p, q, w, x_in, acts[sl][l], sc, tp);
      x_in = acts[sl][l].x_out;
    }
    if (pp) {
      bf16_t* dst = y_all + (size_t)k * M * d;
      emit(p, "save_y", bytes_cost_us(2.0 * mb_bytes), [=](hipStream_t s2, const KCtl& c) { return launch_copy(dst, x_in, mb_bytes, s2, c); });
    }
    return x_in;
  };
  // backward pass of micro-batch k; acc != 0 adds the parameter gradients to the stored ones
  auto emit_backward = [&](Plan& p, uint32_t k, uint32_t acc, const bf16_t* dx_top) {
    const uint32_t sl = k % n_slots;
    if (!fp.open) fp.begin();
    rp.cursor = 0;
    size_t fin_done = 0, red_done = 0;
    const bf16_t* dx = dx_top;
    if (!s.vocab) {
      // top of a stack: the upstream gradient comes from the caller
      bf16_t* dst = sc.dx_a;
      emit(p, "stage_dy", bytes_cost_us(2.0 * mb_bytes), [=](hipStream_t s2, const KCtl& c) {
        return launch_copy(dst, (const unsigned char*)t->cur_targets + (size_t)k * mb_bytes, mb_bytes, s2, c); });
      dx = sc.dx_a;
    }
    for (int32_t l = (int32_t)s.n_layers - 1; l >= 0; --l) {
      const LayerW w = layer_ptrs<LayerW, const bf16_t>(work, pm, l);
      const LayerG g = layer_ptrs<LayerG, bf16_t>(grads, pm, l);
      const bf16_t* xin_l = (l == 0) ? x0[sl] : acts[sl][l - 1].x_out;
      const bool have_db_proj = s.vocab != 0 || l + 1 < (int32_t)s.n_layers;     // the final LayerNorm or the layer above wrote it
      bf16_t* below = l > 0 ? grads + pm.at(L((uint32_t)l - 1, "b_proj")) : nullptr;
      emit_decoder_layer_bwd(p, q, w, g, xin_l, acts[sl][l], sc, dx, sc.dx_b, sc.dx_a, tp, acc, have_db_proj, below, fp, rp, gp);
      dx = sc.dx_a;
      const size_t grp = s.n_layers - 1 - (size_t)l;
      if (overlap && closes_bucket(grp)) {       // the bucket is complete: finalize what it holds, its exchange can start
        emit_fin_range(p, fp, rp, acc, fin_done, fp.items.size(), red_done, rp.items.size());
        fin_done = fp.items.size(); red_done = rp.items.size();
        tm.dp_buckets[bucket_of[grp]].ready_op = (uint32_t)p.size() - 1;
      }
    }
    if (overlap) {
      emit_fin_range(p, fp, rp, acc, fin_done, fp.items.size(), red_done, rp.items.size());
      fp.recorded = true; fp.open = false; rp.recorded = true; rp.cursor = 0;
    } else {
      emit_fin_batch(p, fp, rp, acc);
    }
    if (pp) {
      bf16_t* dst = dx_all + (size_t)k * M * d;
      const bf16_t* src = sc.dx_a;
      emit(p, "save_dx", bytes_cost_us(2.0 * mb_bytes), [=](hipStream_t s2, const KCtl& c) { return launch_copy(dst, src, mb_bytes, s2, c); });
    }
  };

  Plan& p = tm.plan;
  if (!pp) {
    const bf16_t* x_last = emit_forward(p, 0);
    const bf16_t* dx = nullptr;
    if (s.vocab) {
      const bf16_t *wte = work + pm.at("wte"), *lnf_g = work + pm.at("lnf_g"), *lnf_b = work + pm.at("lnf_b");
      emit(p, "lnf", bytes_cost_us(4.0 * M * d), [=](hipStream_t s2, const KCtl& c) { return launch_layernorm_fwd(x_last, lnf_g, lnf_b, lnf, mf, rf, M, d, s2, c); });
      // The product is taken over the padded vocabulary when the rows after wte (the position table follows it in the
      // working copy) can stand in for the padding rows: the epilogue then stores whole 16-byte vectors.  The padding
      // columns of the logits are never read by the loss and are zeroed when it writes the gradient in place.
      const uint32_t n_head = (Vp - V <= s.max_pos) ? Vp : V;
      emit_gemm(p, "lm_head", G(lnf, wte, logits, M, n_head, d, d, d, Vp));
      emit(p, "xent", bytes_cost_us(4.0 * M * Vp), [=](hipStream_t s2, const KCtl& c) { return launch_xent(logits, (const int32_t*)t->cur_targets, loss_tok, M, V, Vp, s2, c); });
      emit(p, "loss", 4.0, [=](hipStream_t s2, const KCtl& c) { return launch_reduce_sum(loss_tok, t->cur_loss ? t->cur_loss : loss, M, 1.0f / (float)M, s2, c); });
      if (wte_tail_splits > 1) {
        bf16_t* dwte = grads + pm.at("wte");
        const uint32_t r0 = wte_tail_row0, rows = wte_tail_rows, kper = wte_tail_kper, ks = wte_tail_splits;
        emit_gemm(p, "dwte_head", G(logits, lnf, dwte, r0, d, M, Vp, d, d).lay(SIF_A_ROW_M, SIF_B_ROW_N).tile(256));
        emit_gemm(p, "dwte_head_tail", G(logits + r0, lnf, wte_tail_part, rows, d, kper, Vp, d, d).lay(SIF_A_ROW_M, SIF_B_ROW_N).epi(SIF_EPI_OUT_F32).tile(256)
                                           .batch(1, ks, 0, (int64_t)kper * Vp, 0, (int64_t)kper * d, 0, (int64_t)rows * d).k_limit(M));
        RedItem it;
        it.part = wte_tail_part; it.out = dwte + (size_t)r0 * d; it.n = (uint64_t)rows * d; it.splits = ks; it.pad = 0;
        hipError_t e2 = hipMemcpy(wte_tail_item, &it, sizeof(it), hipMemcpyHostToDevice);
        if (e2 != hipSuccess) return fail_hip(e2, "training plan: upload of the LM-head weight gradient's slice table");
        const RedItem* ti = wte_tail_item;
        emit(p, "dwte_head_sum", bytes_cost_us(4.0 * rows * d * ks + 2.0 * rows * d), [=](hipStream_t s2, const KCtl& c) { return launch_reduce_splits_batch(ti, 1, 0, s2, c); });
      } else {
        emit_gemm(p, "dwte_head", G(logits, lnf, grads + pm.at("wte"), V, d, M, Vp, d, d).lay(SIF_A_ROW_M, SIF_B_ROW_N));
      }
      if (head_splits > 1) {
        emit_gemm(p, "dlnf", G(logits, wte, head_part, M, d, head_kper, Vp, d, d).lay(SIF_A_ROW_K, SIF_B_ROW_N).epi(SIF_EPI_OUT_F32)
                                 .batch(1, head_splits, 0, head_kper, 0, (int64_t)head_kper * d, 0, (int64_t)M * d).k_limit(head_k));
        RedItem it;
        it.part = head_part; it.out = sc.dln; it.n = (uint64_t)M * d; it.splits = head_splits; it.pad = 0;
        hipError_t e2 = hipMemcpy(head_item, &it, sizeof(it), hipMemcpyHostToDevice);
        if (e2 != hipSuccess) return fail_hip(e2, "training plan: upload of the LM-head slice table");
        const RedItem* hi = head_item;
        emit(p, "dlnf_sum", bytes_cost_us(4.0 * M * d * head_splits + 2.0 * M * d), [=](hipStream_t s2, const KCtl& c) { return launch_reduce_splits_batch(hi, 1, 0, s2, c); });
      } else {
        emit_gemm(p, "dlnf", G(logits, wte, sc.dln, M, d, V, Vp, d, d).lay(SIF_A_ROW_K, SIF_B_ROW_N));
      }
      fp.begin();                  // the final LayerNorm's gradients are finalized with the layers'
      emit_ln_bwd(p, sc.dln, x_last, lnf_g, mf, rf, nullptr, sc.dx_a, grads + pm.at("lnf_g"), grads + pm.at("lnf_b"),
                  grads + pm.at(L(s.n_layers - 1, "b_proj")), fp, M, d);
      dx = sc.dx_a;
    }
    emit_backward(p, 0, 0, dx);
    if (s.vocab) {
      bf16_t *gwte = grads + pm.at("wte"), *gwpe = grads + pm.at("wpe");
      const bf16_t* dx0 = sc.dx_a;
      emit(p, "dwte_scatter", bytes_cost_us(4.0 * M * d) + 10.0, [=](hipStream_t s2, const KCtl& c) { return launch_embed_bwd_wte((const int32_t*)t->cur_inputs, dx0, gwte, V, M, d, s2, c); });
      emit(p, "dwpe", bytes_cost_us(2.0 * M * d), [=](hipStream_t s2, const KCtl& c) { return launch_embed_bwd_wpe(dx0, gwpe, M, seq, d, s2, c); });
    }
    if (overlap) {
      // The embeddings' gradients are final with the last launch of backward.  The bubble's length is decided on the
      // device; what is stored here is the cost model's estimate of it (calibration replaces it by a measured one).
      if (s.vocab) tm.dp_buckets[bucket_of.back()].ready_op = (uint32_t)p.size() - 1;
      std::vector<uint64_t> ready(n_buckets), dur(n_buckets);
      std::vector<double> until(p.size());
      double acc_us = 0;
      for (size_t i = 0; i < p.size(); ++i) { acc_us += p[i].cost_us; until[i] = acc_us; }
      for (uint32_t b = 0; b < n_buckets; ++b) { ready[b] = (uint64_t)(until[tm.dp_buckets[b].ready_op] * 1000.0); dur[b] = tm.dp_buckets[b].dur_ns; }
      const uint64_t ns = sif_dp_overlapped_wait(ready.data(), dur.data(), n_buckets, (uint64_t)(acc_us * 1000.0));
      emit_bubble(p, next_site++, ns);
      p.back().dp_overlap = true;
      tm.max_bubble_ns = ns;
    } else if (tm.desc.par_mode == SIF_PAR_DP) {
      const uint64_t ns = sif_collective_ns(pm.n * 2, tm.desc.bw_bytes_per_s);
      emit_bubble(p, next_site++, ns);
      tm.max_bubble_ns = ns;
    } else if (tm.desc.par_mode == SIF_PAR_FIXED && tm.desc.fixed_bubble_ns) {
      emit_bubble(p, next_site++, tm.desc.fixed_bubble_ns);
      tm.max_bubble_ns = tm.desc.fixed_bubble_ns;
    }
  } else {
    // 1F1B order of this stage: (stages-1-stage) warm-up forwards, then one forward / one backward alternating,
    // then the remaining backwards; idle intervals from the closed form of the schedule
    Plan fwd_probe, bwd_probe;
    emit_forward(fwd_probe, 0);
    emit_backward(bwd_probe, 0, 0, nullptr);
    double tf_us = 0, tb_us = 0;
    for (const Op& o : fwd_probe) tf_us += o.cost_us;
    for (const Op& o : bwd_probe) tb_us += o.cost_us;
    const uint64_t tf = tm.desc.pp_tf_ns ? tm.desc.pp_tf_ns : (uint64_t)(tf_us * 1000.0);
    const uint64_t tb = tm.desc.pp_tb_ns ? tm.desc.pp_tb_ns : (uint64_t)(tb_us * 1000.0);
    int32_t kind[64], index[64];
    uint64_t gap[64];
    const int32_t ng = sif_pp_1f1b_bubbles(tm.desc.pp_stage, tm.desc.pp_stages, n_micro, tf, tb, kind, index, gap, 64);
    if (ng < 0) return (sif_status)ng;
    if (ng > 64) return fail(SIF_E_INVAL, "pipeline schedule has too many idle intervals");
    auto gap_before = [&](int32_t kd, int32_t idx) {
      for (int32_t i = 0; i < ng; ++i)
        if (kind[i] == kd && (kd == 2 || index[i] == idx)) {
          emit_bubble(p, next_site++, gap[i]);
          p.back().pp_kind = kind[i]; p.back().pp_index = index[i];
          if (gap[i] > tm.max_bubble_ns) tm.max_bubble_ns = gap[i];
        }
    };
    const uint32_t warm = std::min(n_micro, tm.desc.pp_stages - 1 - tm.desc.pp_stage);
    uint32_t f = 0, b = 0;
    auto mark = [&](size_t from, int32_t pass) { for (size_t i = from; i < p.size(); ++i) p[i].pp_pass = pass; };
    auto fwd = [&](uint32_t k) { gap_before(0, (int32_t)k); const size_t at = p.size(); emit_forward(p, k); mark(at, 2 * (int32_t)k); };
    auto bwd = [&](uint32_t k) { gap_before(1, (int32_t)k); const size_t at = p.size(); emit_backward(p, k, k > 0, nullptr); mark(at, 2 * (int32_t)k + 1); };
    for (; f < warm; ++f) fwd(f);
    while (f < n_micro) { fwd(f); ++f; bwd(b); ++b; }
    for (; b < n_micro; ++b) bwd(b);
    gap_before(2, -1);
    tm.pp_times_estimated = tm.desc.pp_tf_ns == 0 || tm.desc.pp_tb_ns == 0;
  }
  if (fp.overflow || rp.overflow) return fail(SIF_E_INVAL, "training plan: a partial-result pool does not match the plan");
  if (gp.status != SIF_OK) return gp.status;
  if (!rp.items.empty()) {
    hipError_t e = hipMemcpy(rp.dev, rp.items.data(), rp.items.size() * sizeof(RedItem), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail_hip(e, "training plan: upload of the split-product table");
  }
  if (!fp.items.empty()) {
    hipError_t e = hipMemcpy(fp.dev, fp.items.data(), fp.items.size() * sizeof(FinItem), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail_hip(e, "training plan: upload of the finalize table");
  }
  const uint64_t n = pm.n;
  const float lr = tm.desc.lr;
  float* master = tm.desc.master_dev;
  emit(p, "sgd", bytes_cost_us(12.0 * n), [=](hipStream_t s2, const KCtl& c) { return launch_sgd_bf16(master, grads, work, n, lr, s2, c); });
  return SIF_OK;
}

sif_status build_train_model(TrainModel& tm, hipStream_t stream) {
  sif_status st = check_shape(tm.desc.shape, true);
  if (st != SIF_OK) return st;
  if (tm.desc.par_mode > SIF_PAR_TP) return fail(SIF_E_INVAL, "unknown par_mode");
  if (tm.desc.par_mode == SIF_PAR_PP) {
    if (tm.desc.shape.kind != SIF_MODEL_DECODER || tm.desc.shape.vocab) return fail(SIF_E_INVAL, "a pipeline stage is a decoder layer stack (vocab = 0)");
    if (tm.desc.pp_stages == 0 || tm.desc.pp_stage >= tm.desc.pp_stages || tm.desc.pp_micro < tm.desc.pp_stages || tm.desc.pp_micro > 32)
      return fail(SIF_E_INVAL, "pipeline: need stage < stages <= micro-batches <= 32");
  }
  if ((tm.desc.par_mode == SIF_PAR_DP || tm.desc.par_mode == SIF_PAR_TP) && tm.desc.bw_bytes_per_s == 0) return fail(SIF_E_INVAL, "bw_bytes_per_s must be positive");
  tm.n_params = model_n_params(tm.desc.shape);
  Arena ar;
  ar.base = (unsigned char*)tm.desc.workspace_dev;
  tm.plan.clear();
  tm.tensors.clear();
  if (tm.desc.shape.kind == SIF_MODEL_MLP) {
    if (tm.desc.par_mode == SIF_PAR_FIXED) tm.max_bubble_ns = tm.desc.fixed_bubble_ns;
    return build_mlp_train(tm, ar);
  }
  if (tm.desc.shape.kind == SIF_MODEL_DECODER) return build_decoder_train(tm, ar, stream);
  return fail(SIF_E_INVAL, "training model must be MLP or DECODER");
}

// ------------------------------------------------------------------------------------------ inference models
static uint64_t layout_infer(InferModel& im, Arena& ar) {
  const sif_model_shape& s = im.desc.shape;
  if (s.kind == SIF_MODEL_MLP) {
    im.bufs["h"] = ar.take((uint64_t)s.batch * s.d_hidden * 4);
    im.calib_in = ar.take((uint64_t)s.batch * s.d_in * 4);
    im.calib_out = ar.take((uint64_t)s.batch * s.d_out * 4);
    return ar.off;
  }
  const Dims q = dims_of(s, s.batch * infer_coalesce(im.desc), s.seq);
  const uint64_t ssz = fused_attention(q.dh) ? 8 : (uint64_t)q.B * q.H * q.S * q.Sp, M = q.M;      // scores: unfused attention only
  im.work = ar.take(im.n_params * 2);
  im.bufs["x"] = ar.take(M * q.d * 2); im.bufs["t"] = ar.take(M * q.d * 2); im.bufs["x1"] = ar.take(M * q.d * 2);
  im.bufs["qkv"] = ar.take(M * 3 * q.da * 2); im.bufs["scores"] = ar.take(ssz * 4); im.bufs["prob"] = ar.take(ssz * 2);
  im.bufs["o"] = ar.take(M * q.da * 2); im.bufs["a"] = ar.take(M * q.f * 2);
  im.calib_in = ar.take(M * 4);
  im.calib_out = ar.take(M * q.d * 2);
  return ar.off;
}

uint32_t infer_coalesce(const sif_infer_desc& d) {
  if (d.shape.kind != SIF_MODEL_ENCODER || d.coalesce < 2) return 1;
  return d.coalesce;
}

uint64_t infer_workspace_bytes(const sif_infer_desc& d) {
  InferModel im;
  im.desc = d;
  im.n_params = model_n_params(d.shape);
  Arena ar;
  return layout_infer(im, ar);
}

sif_status build_infer_model(InferModel& im, hipStream_t stream) {
  sif_status st = check_shape(im.desc.shape, false);
  if (st != SIF_OK) return st;
  if (im.desc.shape.kind == SIF_MODEL_DECODER) return fail(SIF_E_INVAL, "inference model must be MLP or ENCODER");
  if (im.desc.coalesce > kMaxCoalesce) return fail(SIF_E_INVAL, "inference model: coalesce must be at most %u", kMaxCoalesce);
  im.n_params = model_n_params(im.desc.shape);
  Arena ar;
  ar.base = (unsigned char*)im.desc.workspace_dev;
  const uint64_t need = layout_infer(im, ar);
  if (need > im.desc.workspace_bytes) return fail(SIF_E_NOMEM, "inference workspace too small: need %llu bytes", (unsigned long long)need);
  const sif_model_shape& s = im.desc.shape;
  const uint64_t in_bytes = s.kind == SIF_MODEL_MLP ? (uint64_t)s.batch * s.d_in * 4 : (uint64_t)s.batch * s.seq * 4;
  hipError_t e = hipMemsetAsync(im.calib_in, 0, in_bytes, stream);
  if (e != hipSuccess) return fail_hip(e, "register: clear calibration input");
  if (s.kind == SIF_MODEL_ENCODER) return launch_sgd_bf16(const_cast<float*>(im.desc.master_dev), nullptr, im.work, im.n_params, 0.f, stream, no_ctl());
  return SIF_OK;
}

sif_status build_infer_plan(const InferModel& im, const InferIO* io, uint32_t n_io, uint32_t batch, uint32_t seq,
                            uint32_t kernel_us_max, Plan& p) {
  const sif_model_shape& s = im.desc.shape;
  if (!io || n_io == 0 || n_io > infer_coalesce(im.desc)) return fail(SIF_E_INVAL, "submit: bad request count");
  for (uint32_t i = 0; i < n_io; ++i) if (!io[i].in_dev || !io[i].out_dev) return fail(SIF_E_INVAL, "submit: null buffer");
  const void* in_dev = io[0].in_dev;
  void* out_dev = io[0].out_dev;
  (void)out_dev;
  if (batch == 0 || batch > s.batch) return fail(SIF_E_INVAL, "submit: batch must be in 1..%u", s.batch);
  const ParamMap pm = param_map(s);
  if (s.kind == SIF_MODEL_MLP) {
    const float* W = im.desc.master_dev;
    const float *w1 = W + pm.at("w1"), *b1 = W + pm.at("b1"), *w2 = W + pm.at("w2"), *b2 = W + pm.at("b2");
    float* h = (float*)im.bufs.at("h");
    const uint32_t di = s.d_in, dh = s.d_hidden, dout = s.d_out;
    const float* x = (const float*)in_dev;
    float* y = (float*)out_dev;
    emit(p, "fc1", 5, [=](hipStream_t st, const KCtl& c) { return launch_gemm_f32(x, di, 1, w1, 1, di, h, dh, batch, dh, di, SIF_EPI_GELU, b1, nullptr, st, c); });
    emit(p, "fc2", 5, [=](hipStream_t st, const KCtl& c) { return launch_gemm_f32(h, dh, 1, w2, 1, dh, y, dout, batch, dout, dh, SIF_EPI_BIAS, b2, nullptr, st, c); });
    return SIF_OK;
  }
  if (n_io != 1 && s.kind != SIF_MODEL_ENCODER) return fail(SIF_E_INVAL, "submit: only encoder requests can be coalesced");
  if (seq == 0 || seq > s.seq) return fail(SIF_E_INVAL, "submit: seq must be in 1..%u", s.seq);
  // n_io requests of batch x seq rows each run as one sequence over their concatenated rows: every kernel below treats
  // rows (LayerNorm, GEMM) or whole sequences (attention) independently, so a request's result does not depend on
  // what it is concatenated with.  Only the first and the last kernel touch the requests' own buffers.
  // Requests of one sequence each may differ in length: their rows still lie back to back, and attention is told where
  // each sequence begins.
  Dims q = dims_of(s, batch * n_io, seq);
  std::vector<uint32_t> rows_of(n_io), row0(n_io + 1, 0);
  bool ragged = false;
  for (uint32_t r = 0; r < n_io; ++r) {
    const uint32_t sr = io[r].seq ? io[r].seq : seq;
    if (sr == 0 || sr > seq) return fail(SIF_E_INVAL, "submit: a request's seq must be in 1..%u", seq);
    ragged = ragged || sr != seq;
    rows_of[r] = batch * sr;
    row0[r + 1] = row0[r] + rows_of[r];
  }
  if (ragged && (batch != 1 || !(q.dh == 64 || q.dh == 128) || n_io > kAttnMaxSeqs))
    return fail(SIF_E_INVAL, "submit: requests of different lengths need batch 1 and d_head 64 or 128");
  q.M = row0[n_io];
  const uint32_t M = q.M, d = q.d;
  const bf16_t* W = (const bf16_t*)im.work;
  bf16_t *x = (bf16_t*)im.bufs.at("x"), *t = (bf16_t*)im.bufs.at("t"), *x1 = (bf16_t*)im.bufs.at("x1"), *qkv = (bf16_t*)im.bufs.at("qkv");
  bf16_t *prob = (bf16_t*)im.bufs.at("prob"), *o = (bf16_t*)im.bufs.at("o"), *a = (bf16_t*)im.bufs.at("a");
  float* scores = (float*)im.bufs.at("scores");
  const bf16_t *wte = W + pm.at("wte"), *wpe = W + pm.at("wpe"), *eg = W + pm.at("emb_ln_g"), *eb = W + pm.at("emb_ln_b");
  const uint32_t vocab = s.vocab;
  // the first and the last kernel serve all requests of the sequence at once: a table says which rows are whose
  static_assert(kMaxRowSegs >= kMaxCoalesce, "one row segment per coalesced request");
  RowSegs in_segs, out_segs;
  in_segs.n = out_segs.n = n_io;
  for (uint32_t r = 0; r <= n_io; ++r) in_segs.row0[r] = out_segs.row0[r] = row0[r];
  for (uint32_t r = 0; r < n_io; ++r) {
    in_segs.ptr[r] = const_cast<void*>(io[r].in_dev); out_segs.ptr[r] = io[r].out_dev;
    in_segs.seq[r] = out_segs.seq[r] = rows_of[r] / batch;
  }
  emit(p, "embed", bytes_cost_us(6.0 * M * d), [=](hipStream_t st, const KCtl& c) { return launch_embed_fwd_segs(in_segs, wte, wpe, t, vocab, d, st, c); });
  emit(p, "emb_ln", bytes_cost_us(4.0 * M * d), [=](hipStream_t st, const KCtl& c) { return launch_layernorm_fwd(t, eg, eb, x, nullptr, nullptr, M, d, st, c); });
  for (uint32_t l = 0; l < s.n_layers; ++l) {
    const bf16_t *w_qkv = W + pm.at(L(l, "w_qkv")), *b_qkv = W + pm.at(L(l, "b_qkv")), *w_o = W + pm.at(L(l, "w_o")), *b_o = W + pm.at(L(l, "b_o"));
    const bf16_t *g1 = W + pm.at(L(l, "ln1_g")), *be1 = W + pm.at(L(l, "ln1_b")), *w_fc = W + pm.at(L(l, "w_fc")), *b_fc = W + pm.at(L(l, "b_fc"));
    const bf16_t *w_pr = W + pm.at(L(l, "w_proj")), *b_pr = W + pm.at(L(l, "b_proj")), *g2 = W + pm.at(L(l, "ln2_g")), *be2 = W + pm.at(L(l, "ln2_b"));
    const bool last = l + 1 == s.n_layers;
    emit_gemm_rows(p, "qkv", G(x, w_qkv, qkv, M, 3 * q.da, d, d, d, 3 * q.da).epi(SIF_EPI_BIAS, b_qkv), kernel_us_max);
    if (q.dh == 64 || q.dh == 128) {
      // one fused kernel: scores stay on chip, two launches fewer per layer
      const uint32_t B = q.B, S = q.S, H = q.H, dh = q.dh, da = q.da;
      const double cost = 4.0 + 4.0 * B * H * (double)S * S * dh / 3.0e8 + bytes_cost_us(8.0 * M * da);
      if (ragged) {
        const std::vector<uint32_t> starts = row0;
        emit(p, "attn_fused", cost, [=](hipStream_t st, const KCtl& c) { return launch_attn_fwd_varlen(qkv, o, starts.data(), n_io, H, dh, 3 * da, da, 0, st, c); });
      } else {
        emit(p, "attn_fused", cost, [=](hipStream_t st, const KCtl& c) { return launch_attn_fwd(qkv, o, nullptr, B, S, H, dh, 3 * da, da, 0, st, c); });
      }
    } else {
      emit_attention_fwd(p, q, qkv, scores, prob, o, false);
    }
    emit_gemm_rows(p, "attn_out", G(o, w_o, t, M, d, q.da, q.da, q.da, d).epi(SIF_EPI_BIAS | SIF_EPI_RESIDUAL, b_o, x), kernel_us_max);
    emit(p, "ln1", bytes_cost_us(4.0 * M * d), [=](hipStream_t st, const KCtl& c) { return launch_layernorm_fwd(t, g1, be1, x1, nullptr, nullptr, M, d, st, c); });
    emit_gemm_rows(p, "mlp_up", G(x1, w_fc, a, M, q.f, d, d, d, q.f).epi(SIF_EPI_GELU, b_fc), kernel_us_max);
    emit_gemm_rows(p, "mlp_down", G(a, w_pr, t, M, d, q.f, q.f, q.f, d).epi(SIF_EPI_BIAS | SIF_EPI_RESIDUAL, b_pr, x1), kernel_us_max);
    if (!last) {
      emit(p, "ln2", bytes_cost_us(4.0 * M * d), [=](hipStream_t st, const KCtl& c) { return launch_layernorm_fwd(t, g2, be2, x, nullptr, nullptr, M, d, st, c); });
    } else {
      emit(p, "ln2", bytes_cost_us(4.0 * M * d), [=](hipStream_t st, const KCtl& c) { return launch_layernorm_fwd(t, g2, be2, nullptr, nullptr, nullptr, M, d, st, c, &out_segs); });
    }
  }
  return SIF_OK;
}

}  // namespace sif
