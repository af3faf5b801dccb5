// Fused attention, forward and backward, without materialising the score matrix in HBM (the unfused path writes
// and re-reads 4 + 2 bytes per score and costs three launches per layer forward, five backward; an inference
// forward is a chain of short, launch-bound kernels, Sec. 3.3 "Kernel Barrier", and the training instance's step
// time is what Principle II of Sec. 3.2 protects).
//
//   forward    o = softmax(scale q k^T [+ causal mask]) v,  lse = log sum exp of the scaled, masked scores (optional)
//   backward   delta = rowsum(do .* o),  P = exp(scale q k^T - lse),  dS = scale P .* (do v^T - delta)
//              dq = dS k   (one kernel, a block per 128 query rows, keys streamed)
//              dk = dS^T q,  dv = P^T do   (a second kernel, a block per 128 key rows, queries streamed)
// Both backward kernels recompute P from q, k and lse; no atomics, each output element is reduced in one fixed order.
//
// Every product is arranged so that the operand produced on chip (P, dS) goes from the accumulator registers of
// one MFMA straight into the B operand of the next: an accumulator tile holds column (lane % 32) and the rows
// 8*(r/4) + 4*(lane/32) + r%4, so as a B operand [k][col] its k index is a permutation of the row index, which is
// applied to the reads of the matching A operand (fetched with the transposing LDS read) instead.  In the forward and the dq
// kernel the products are taken transposed (S^T = K Q^T, O^T = V^T P^T, dQ^T = K^T dS^T): a query row then lives
// in one lane and its partner 32 further, and the softmax statistics are per-lane scalars.  bf16 operands, fp32
// accumulation and softmax; P and dS are rounded to bf16 where the unfused path stores them.
#include <math.h>
#include <algorithm>

#include "common.h"
#include "launch.h"

namespace sif {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int AT_Q = 128, AT_KV = 128, AT_THREADS = 256;
constexpr int AT_QB = 64;                                    // query rows per step of the dk/dv kernel

__device__ __forceinline__ uint32_t at_key(uint32_t row) { return (row & 7u) ^ ((row >> 3) & 1u); }

// ROWS x DH tile of a row-major bf16 matrix (rows row0.., 16-byte aligned, ld elements apart) into LDS as
// [row][d] with the 16-byte chunks of a row XOR-swizzled; rows >= limit read as zero.
template <int DH, int ROWS>
__device__ __forceinline__ void at_load_rows(bf16_t* dst, const bf16_t* src, size_t ld, uint32_t row0, uint32_t limit) {
  constexpr int CH = DH / 8;
  for (uint32_t v = threadIdx.x; v < ROWS * CH; v += AT_THREADS) {
    const uint32_t row = v / CH, c = v % CH;
    uint4 x = make_uint4(0, 0, 0, 0);
    if (row0 + row < limit) x = *reinterpret_cast<const uint4*>(src + (size_t)(row0 + row) * ld + c * 8);
    *reinterpret_cast<uint4*>(dst + row * DH + ((c ^ (at_key(row) % CH)) << 3)) = x;
  }
}
// The same tile fetched from global memory straight into LDS (global_load_lds_dwordx4: no staging registers, the
// fetch of the next tile runs while the current one is used).  One instruction writes the 64 lanes' 16 bytes to
// consecutive LDS addresses, so a lane's place in the tile is fixed and the swizzle is applied to what it fetches.
// Rows >= limit cannot be zero-filled: they fetch row limit - 1 instead (finite data), and every use of such a row is
// either masked (scores) or multiplied by a probability of zero.
template <int DH, int ROWS>
__device__ __forceinline__ void at_dma_rows(bf16_t* dst, const bf16_t* src, size_t ld, uint32_t row0, uint32_t limit) {
  typedef __attribute__((address_space(3))) void* lds_void_ptr;
  typedef __attribute__((address_space(1))) const void* global_void_ptr;
  constexpr int CH = DH / 8, RPI = 64 / CH;                  // chunks per row, rows per instruction and wavefront
  const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
  for (int i = 0; i < ROWS / (RPI * (AT_THREADS / 64)); ++i) {
    const uint32_t first = (i * (AT_THREADS / 64) + wave) * RPI, row = first + lane / CH, c = (lane % CH) ^ (at_key(row) % CH);
    const uint32_t r = row0 + row < limit ? row0 + row : limit - 1;
    __builtin_amdgcn_global_load_lds((global_void_ptr)(src + (size_t)r * ld + c * 8), (lds_void_ptr)(dst + first * DH), 16, 0, 0);
  }
}
// 32 rows fetched the same way by ONE wavefront into 32*DH elements of LDS of its own (rows swizzled by their number
// within the 32): whole 128-byte rows per fetch, where a lane that reads its own row from global memory fetches 16
// bytes of it per instruction.
template <int DH>
__device__ __forceinline__ void at_dma_rows_wave(bf16_t* dst, const bf16_t* src, size_t ld, uint32_t row0, uint32_t limit) {
  typedef __attribute__((address_space(3))) void* lds_void_ptr;
  typedef __attribute__((address_space(1))) const void* global_void_ptr;
  constexpr int CH = DH / 8, RPI = 64 / CH;
  const uint32_t lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < 32 / RPI; ++i) {
    const uint32_t first = i * RPI, row = first + lane / CH, c = (lane % CH) ^ (at_key(row) % CH);
    const uint32_t r = row0 + row < limit ? row0 + row : limit - 1;
    __builtin_amdgcn_global_load_lds((global_void_ptr)(src + (size_t)r * ld + c * 8), (lds_void_ptr)(dst + first * DH), 16, 0, 0);
  }
}
// A wavefront's 32 x DH results, held transposed in MFMA accumulators (element r of tile d in lane (qi, h) is column
// d*32 + (r/4)*8 + h*4 + r%4 of row qi), times mul, to global memory as whole rows.  Stored straight from the
// accumulators a lane would write 8 bytes at a time and every 128-byte line of the output would be touched by eight
// store instructions, 16 bytes each.  So the tile passes through 32*DH elements of LDS that belong to this wavefront
// alone (16-byte chunks of a row swizzled with the row) and leaves as 16-byte vectors, a row of 128 bytes per eight
// lanes.  dst = row 0, column 0 of the tile; only the first `rows` rows exist.
template <int DH>
__device__ __forceinline__ void at_store_tile(bf16_t* stage, const floatx16 (&acc)[DH / 32], float mul, bf16_t* dst, size_t ld, uint32_t rows) {
  constexpr int CH = DH / 8;
  const uint32_t lane = threadIdx.x & 63, qi = lane & 31, h = lane >> 5;
#pragma unroll
  for (int d = 0; d < DH / 32; ++d)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<uint2*>(stage + qi * DH + (((d * 4 + g) ^ (qi & 7u)) << 3) + h * 4) =
          make_uint2(pack_bf2(acc[d][4 * g] * mul, acc[d][4 * g + 1] * mul), pack_bf2(acc[d][4 * g + 2] * mul, acc[d][4 * g + 3] * mul));
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int it = 0; it < 32 * CH / 64; ++it) {
    const uint32_t idx = lane + it * 64, row = idx / CH, c = idx % CH;
    const uint4 v = *reinterpret_cast<const uint4*>(stage + row * DH + ((c ^ (row & 7u)) << 3));
    if (row < rows) *reinterpret_cast<uint4*>(dst + (size_t)row * ld + c * 8) = v;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}
// A operand (row, k = 8 consecutive d) from a swizzled [row][d] tile; chunk = k / 8.
template <int DH>
__device__ __forceinline__ bf16x8 at_frag(const bf16_t* tile, uint32_t row, uint32_t chunk) {
  return *reinterpret_cast<const bf16x8*>(tile + row * DH + ((chunk ^ (at_key(row) % (DH / 8))) << 3));
}
// A operand of a product that contracts over the tile's rows: operand row d (32 of them from dbase32, one per lane
// and lane + 32), k = the tile rows kb..kb+3 and kb+8..kb+11 (kb already holds the lane half's offset of 4).  The
// tile stays [row][d]; the transposing LDS read of gfx950 (ds_read_b64_tr_b16) does the rest: within a group of
// 16 lanes, source lane s supplies the address of four consecutive d at tile row kb + s/4, d = d0 + 4*(s%4).., and
// lane i receives d0 + i at the four tile rows.
template <int DH>
__device__ __forceinline__ bf16x8 at_frag_tr(const bf16_t* tile, uint32_t dbase32, uint32_t kb) {
  typedef short short4_lds __attribute__((ext_vector_type(4)));
  typedef short short8_v __attribute__((ext_vector_type(8)));
  typedef __attribute__((address_space(3))) short4_lds* lds_ptr;
  const uint32_t lane = threadIdx.x & 63, s = lane & 15;
  const uint32_t row = kb + (s >> 2), d = dbase32 + ((lane >> 4) & 1u) * 16 + 4 * (s & 3u);
  const bf16_t* p0 = tile + row * DH + ((((d >> 3) ^ (at_key(row) % (DH / 8))) << 3) | (d & 7u));
  const bf16_t* p1 = tile + (row + 8) * DH + ((((d >> 3) ^ (at_key(row + 8) % (DH / 8))) << 3) | (d & 7u));
  const short4_lds lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p0);
  const short4_lds hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p1);
  const short8_v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}
// eight accumulator values r0..r0+7 as a B operand
__device__ __forceinline__ bf16x8 at_pack8(const float (&v)[16], int r0) {
  uint4 pv = make_uint4(pack_bf2(v[r0], v[r0 + 1]), pack_bf2(v[r0 + 2], v[r0 + 3]), pack_bf2(v[r0 + 4], v[r0 + 5]), pack_bf2(v[r0 + 6], v[r0 + 7]));
  return *reinterpret_cast<bf16x8*>(&pv);
}
__device__ __forceinline__ float at_round(float x) { return bf2f(f2bf(x)); }

// Forward.  One block = 128 query rows of one (batch, head), 4 wavefronts x 32 rows; keys/values streamed in tiles
// of 128 through LDS (K and V as [kv][d]); running maximum / sum / rescale per lane.
template <int DH, int CAUSAL>
__global__ __launch_bounds__(AT_THREADS, 2) void attn_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o, float* __restrict__ lse,
                                                              uint32_t S, uint32_t H, uint32_t ld_qkv, uint32_t ld_o, float scale, AttnSeqs seqs,
                                                              KCtl ctl) {
  constexpr int KS = DH / 16, DT = DH / 32;                   // k steps of q k^T, 32-wide d tiles
  // d_head 64: two K and two V tile buffers (as four objects, so that the compiler can tell the one being filled from
  // the one being read), the next tile is fetched while the current one is used; d_head 128: LDS holds one of each
  constexpr bool DB = DH == 64;
  __shared__ __align__(1024) bf16_t sK0[AT_KV * DH];
  __shared__ __align__(1024) bf16_t sV0[AT_KV * DH];
  __shared__ __align__(1024) bf16_t sK1[DB ? AT_KV * DH : 8];
  __shared__ __align__(1024) bf16_t sV1[DB ? AT_KV * DH : 8];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, qi = lane & 31, h = lane >> 5;
  const uint32_t bh = blockIdx.x, b = bh / H, head = bh % H, da = H * DH;
  // sequences of equal length S back to back, or (seqs.n > 0) sequence b in rows seqs.start[b] .. seqs.start[b+1]
  size_t row0 = (size_t)b * S;
  if (seqs.n != 0) { row0 = seqs.start[b]; S = seqs.start[b + 1] - seqs.start[b]; }
  const bf16_t* base = qkv + row0 * ld_qkv + head * DH;
  // with a causal mask the last query block has the most keys: the grid's slow index is the query block, reversed,
  // so that the long blocks of every (batch, head) start first
  const uint32_t q_blk = (CAUSAL ? gridDim.y - 1 - blockIdx.y : blockIdx.y) * AT_Q, qw = q_blk + wave * 32, q = qw + qi;
  const float c2 = scale * 1.44269504088896f;
  if (q_blk >= S) { kernel_end(ctl, true); return; }       // the grid is sized for the longest sequence

  bf16x8 fq[KS];
  if constexpr (!DB) {
    const bf16_t* qp = base + (size_t)(q < S ? q : 0) * ld_qkv;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 v = *reinterpret_cast<const uint4*>(qp + ks * 16 + h * 8);
      if (q >= S) v = make_uint4(0, 0, 0, 0);
      fq[ks] = *reinterpret_cast<bf16x8*>(&v);
    }
  }
  floatx16 oacc[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[d][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f, l_true = 0.f;

  const uint32_t kv_end = CAUSAL ? min(S, q_blk + AT_Q) : S;
  auto tile = [&](const bf16_t* sK, const bf16_t* sV, const uint32_t kv0) {
    // S^T tiles: rows = kv (32 per tile), columns = the wavefront's 32 query rows (straight-line code: the four
    // accumulator chains interleave; skipping the tiles above the diagonal would cost more than it saves)
    const bool need_mask = kv0 + AT_KV > S || (CAUSAL && kv0 + AT_KV - 1 > qw);
    floatx16 sacc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[t][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at_frag<DH>(sK, t * 32 + qi, ks * 2 + h), fq[ks], sacc[t], 0, 0, 0);
    }
    // mask (only tiles that meet the diagonal or the end of the sequence), running maximum of the raw scores
    float mx = -INFINITY;
    if (need_mask) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
  #pragma unroll
        for (int r = 0; r < 16; ++r) {
          const uint32_t kv = kv0 + t * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
          const bool ok = kv < S && (!CAUSAL || kv <= q);
          sacc[t][r] = ok ? sacc[t][r] : -INFINITY;
        }
      }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[t][r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c2;                       // base-2 exponent units: c2 = scale * log2(e) > 0
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;          // a fully masked row keeps everything at zero
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);        // 2^(-inf) = 0 on the first tile
    float rs = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[t][r] = __builtin_amdgcn_exp2f(fmaf(sacc[t][r], c2, -m_use)); rs += sacc[t][r]; }
    }
    rs += __shfl_xor(rs, 32, 64);
    l_run = l_run * alpha + rs;
    l_true = l_run;
    m_run = m_new;
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[d][r] *= alpha;
    // a single tile covers all keys: normalise before rounding, as the unfused path does
    const bool single = kv_end <= AT_KV;
    const float pn = single ? 1.0f / l_run : 1.0f;

    // O^T += V^T P^T.  Element e of step s2 in tile t is key  t*32 + 16*s2 + 8*(e/4) + 4*h + e%4.
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      float pt[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) pt[r] = sacc[t][r] * pn;
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8 fp = at_pack8(pt, 8 * s2);
#pragma unroll
        for (int d = 0; d < DT; ++d)
          oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at_frag_tr<DH>(sV, d * 32, t * 32 + 16 * s2 + 4 * h), fp, oacc[d], 0, 0, 0);
      }
    }
    if (single) l_run = 1.0f;
  };
  if constexpr (DB) {
    // The wavefront's 32 query rows pass through its own quarter of buffer 1, which nobody fetches into before the
    // first barrier of the loop; by then the fragments are in registers.  (Rows past the end of the sequence hold a
    // copy of its last row: their results are not stored.)
    bf16_t* sQ = sK1 + __builtin_amdgcn_readfirstlane(wave) * (32 * DH);
    at_dma_rows_wave<DH>(sQ, base, ld_qkv, qw, S);
    at_dma_rows<DH, AT_KV>(sK0, base + da, ld_qkv, 0, S);
    at_dma_rows<DH, AT_KV>(sV0, base + 2 * da, ld_qkv, 0, S);
    wait_fetches();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fq[ks] = at_frag<DH>(sQ, qi, ks * 2 + h);
    for (uint32_t kv0 = 0; kv0 < kv_end; kv0 += 2 * AT_KV) {
      wait_fetches();
      __syncthreads();                                   // tile kv0 has landed, nobody reads buffer 1 any more
      const bool more = kv0 + AT_KV < kv_end;
      if (more) {
        at_dma_rows<DH, AT_KV>(sK1, base + da, ld_qkv, kv0 + AT_KV, S);
        at_dma_rows<DH, AT_KV>(sV1, base + 2 * da, ld_qkv, kv0 + AT_KV, S);
      }
      tile(sK0, sV0, kv0);
      if (more) {
        wait_fetches();
        __syncthreads();                                 // tile kv0 + 128 has landed, nobody reads buffer 0 any more
        if (kv0 + 2 * AT_KV < kv_end) {
          at_dma_rows<DH, AT_KV>(sK0, base + da, ld_qkv, kv0 + 2 * AT_KV, S);
          at_dma_rows<DH, AT_KV>(sV0, base + 2 * da, ld_qkv, kv0 + 2 * AT_KV, S);
        }
        tile(sK1, sV1, kv0 + AT_KV);
      }
    }
  } else {
    for (uint32_t kv0 = 0; kv0 < kv_end; kv0 += AT_KV) {
      __syncthreads();
      at_load_rows<DH, AT_KV>(sK0, base + da, ld_qkv, kv0, S);
      at_load_rows<DH, AT_KV>(sV0, base + 2 * da, ld_qkv, kv0, S);
      __syncthreads();
      tile(sK0, sV0, kv0);
    }
  }

  __syncthreads();                                         // nobody reads the last K/V tile any more: sK0 stages the output
  at_store_tile<DH>(sK0 + wave * (32 * DH), oacc, l_run > 0.f ? 1.0f / l_run : 0.f, o + (row0 + qw) * ld_o + head * DH, ld_o,
                    qw < S ? S - qw : 0u);
  if (q < S && lse != nullptr && h == 0) lse[(size_t)bh * S + q] = (m_run + __log2f(l_true)) * 0.693147180559945f;
  kernel_end(ctl, true);
}

// Backward, dq.  One block = 128 query rows of one (batch, head), a query row per lane pair as in the forward;
// keys/values streamed in tiles of 128, K and V as [kv][d].  Also writes delta = rowsum(do .* o)
// for the dk/dv kernel.
template <int DH, int CAUSAL>
__global__ __launch_bounds__(AT_THREADS, 2) void attn_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ o,
                                                                 const bf16_t* __restrict__ d_o, const float* __restrict__ lse,
                                                                 float* __restrict__ delta, bf16_t* __restrict__ dqkv, uint32_t S, uint32_t H,
                                                                 uint32_t ld_qkv, uint32_t ld_o, uint32_t ld_dqkv, float scale, KCtl ctl) {
  constexpr int KS = DH / 16, DT = DH / 32;
  constexpr bool DB = DH == 64;                               // two tile buffers each, as in the forward kernel
  __shared__ __align__(1024) bf16_t sK0[AT_KV * DH];
  __shared__ __align__(1024) bf16_t sV0[AT_KV * DH];
  __shared__ __align__(1024) bf16_t sK1[DB ? AT_KV * DH : 8];
  __shared__ __align__(1024) bf16_t sV1[DB ? AT_KV * DH : 8];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, qi = lane & 31, h = lane >> 5;
  const uint32_t bh = blockIdx.x, b = bh / H, head = bh % H, da = H * DH;
  const bf16_t* base = qkv + (size_t)b * S * ld_qkv + head * DH;
  const uint32_t q_blk = (CAUSAL ? gridDim.y - 1 - blockIdx.y : blockIdx.y) * AT_Q, qw = q_blk + wave * 32, q = qw + qi;
  const bool q_ok = q < S;
  const float c2 = scale * 1.44269504088896f;

  bf16x8 fq[KS], fdo[KS];
  float dsum = 0.f;
  {
    const size_t row = (size_t)b * S + (q_ok ? q : 0);
    const bf16_t* qp = base + (size_t)(q_ok ? q : 0) * ld_qkv;
    const bf16_t* dop = d_o + row * ld_o + head * DH;
    const bf16_t* op = o + row * ld_o + head * DH;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 vq = *reinterpret_cast<const uint4*>(qp + ks * 16 + h * 8);
      uint4 vd = *reinterpret_cast<const uint4*>(dop + ks * 16 + h * 8);
      const uint4 vo = *reinterpret_cast<const uint4*>(op + ks * 16 + h * 8);
      if (!q_ok) { vq = make_uint4(0, 0, 0, 0); vd = make_uint4(0, 0, 0, 0); }
      fq[ks] = *reinterpret_cast<bf16x8*>(&vq);
      fdo[ks] = *reinterpret_cast<bf16x8*>(&vd);
      dsum += bflo(vd.x) * bflo(vo.x) + bfhi(vd.x) * bfhi(vo.x) + bflo(vd.y) * bflo(vo.y) + bfhi(vd.y) * bfhi(vo.y) +
              bflo(vd.z) * bflo(vo.z) + bfhi(vd.z) * bfhi(vo.z) + bflo(vd.w) * bflo(vo.w) + bfhi(vd.w) * bfhi(vo.w);
    }
  }
  dsum += __shfl_xor(dsum, 32, 64);
  const float lq2 = q_ok ? lse[(size_t)bh * S + q] * 1.44269504088896f : INFINITY;     // base-2 units
  if (q_ok && h == 0) delta[(size_t)bh * S + q] = dsum;

  floatx16 dqacc[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqacc[d][r] = 0.f;

  const uint32_t kv_end = CAUSAL ? min(S, q_blk + AT_Q) : S;
  auto tile = [&](const bf16_t* sK, const bf16_t* sV, const uint32_t kv0) {
    const bool need_mask = kv0 + AT_KV > S || (CAUSAL && kv0 + AT_KV - 1 > qw);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      floatx16 sacc, pacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; pacc[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at_frag<DH>(sK, t * 32 + qi, ks * 2 + h), fq[ks], sacc, 0, 0, 0);     // S^T
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at_frag<DH>(sV, t * 32 + qi, ks * 2 + h), fdo[ks], pacc, 0, 0, 0);    // dP^T
      }
      float ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = at_round(__builtin_amdgcn_exp2f(fmaf(sacc[r], c2, -lq2)));
        if (need_mask) {
          const uint32_t kv = kv0 + t * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
          p = (kv < S && (!CAUSAL || kv <= q)) ? p : 0.f;
        }
        ds[r] = p * scale * (pacc[r] - dsum);
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8 fds = at_pack8(ds, 8 * s2);
#pragma unroll
        for (int d = 0; d < DT; ++d)
          dqacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at_frag_tr<DH>(sK, d * 32, t * 32 + 16 * s2 + 4 * h), fds, dqacc[d], 0, 0, 0);
      }
    }
  };
  if constexpr (DB) {
    at_dma_rows<DH, AT_KV>(sK0, base + da, ld_qkv, 0, S);
    at_dma_rows<DH, AT_KV>(sV0, base + 2 * da, ld_qkv, 0, S);
    for (uint32_t kv0 = 0; kv0 < kv_end; kv0 += 2 * AT_KV) {
      wait_fetches();
      __syncthreads();                                   // tile kv0 has landed, nobody reads buffer 1 any more
      const bool more = kv0 + AT_KV < kv_end;
      if (more) {
        at_dma_rows<DH, AT_KV>(sK1, base + da, ld_qkv, kv0 + AT_KV, S);
        at_dma_rows<DH, AT_KV>(sV1, base + 2 * da, ld_qkv, kv0 + AT_KV, S);
      }
      tile(sK0, sV0, kv0);
      if (more) {
        wait_fetches();
        __syncthreads();
        if (kv0 + 2 * AT_KV < kv_end) {
          at_dma_rows<DH, AT_KV>(sK0, base + da, ld_qkv, kv0 + 2 * AT_KV, S);
          at_dma_rows<DH, AT_KV>(sV0, base + 2 * da, ld_qkv, kv0 + 2 * AT_KV, S);
        }
        tile(sK1, sV1, kv0 + AT_KV);
      }
    }
  } else {
    for (uint32_t kv0 = 0; kv0 < kv_end; kv0 += AT_KV) {
      __syncthreads();
      at_load_rows<DH, AT_KV>(sK0, base + da, ld_qkv, kv0, S);
      at_load_rows<DH, AT_KV>(sV0, base + 2 * da, ld_qkv, kv0, S);
      __syncthreads();
      tile(sK0, sV0, kv0);
    }
  }
  __syncthreads();                                         // nobody reads the last K/V tile any more: sK0 stages dq
  at_store_tile<DH>(sK0 + wave * (32 * DH), dqacc, 1.0f, dqkv + ((size_t)b * S + qw) * ld_dqkv + head * DH, ld_dqkv, qw < S ? S - qw : 0u);
  kernel_end(ctl, true);
}

// Backward, dk and dv.  One block = 128 key rows of one (batch, head), a key row per lane pair (its K and V rows stay
// in registers); queries streamed in steps of 64 rows: q and do as [q][d], lse and delta beside them.
template <int DH, int CAUSAL>
__global__ __launch_bounds__(AT_THREADS, DH == 64 ? 2 : 1) void attn_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ d_o,
                                                                  const float* __restrict__ lse, const float* __restrict__ delta,
                                                                  bf16_t* __restrict__ dqkv, uint32_t S, uint32_t H, uint32_t ld_qkv,
                                                                  uint32_t ld_o, uint32_t ld_dqkv, float scale, KCtl ctl) {
  constexpr int KS = DH / 16, DT = DH / 32;
  constexpr bool DB = DH == 64;                               // two buffers of everything that is streamed, as in the forward kernel
  __shared__ __align__(1024) bf16_t sQ0[AT_QB * DH];
  __shared__ __align__(1024) bf16_t sDo0[AT_QB * DH];
  __shared__ __align__(1024) bf16_t sQ1[DB ? AT_QB * DH : 8];
  __shared__ __align__(1024) bf16_t sDo1[DB ? AT_QB * DH : 8];
  __shared__ __align__(16) float sL0[AT_QB];
  __shared__ __align__(16) float sD0[AT_QB];
  __shared__ __align__(16) float sL1[AT_QB];
  __shared__ __align__(16) float sD1[AT_QB];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, ki = lane & 31, h = lane >> 5;
  const uint32_t bh = blockIdx.x, b = bh / H, head = bh % H, da = H * DH;
  const bf16_t* base = qkv + (size_t)b * S * ld_qkv + head * DH;
  const bf16_t* dobase = d_o + (size_t)b * S * ld_o + head * DH;
  const float* lrow = lse + (size_t)bh * S;
  const float* drow = delta + (size_t)bh * S;
  const uint32_t kv_blk = blockIdx.y * AT_KV, kw = kv_blk + wave * 32, kv = kw + ki;   // the first key block meets the most queries
  const bool kv_ok = kv < S;
  const float c2 = scale * 1.44269504088896f;

  bf16x8 fk[KS], fv[KS];
  {
    const bf16_t* kp = base + da + (size_t)(kv_ok ? kv : 0) * ld_qkv;
    const bf16_t* vp = kp + da;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 a = *reinterpret_cast<const uint4*>(kp + ks * 16 + h * 8), c = *reinterpret_cast<const uint4*>(vp + ks * 16 + h * 8);
      if (!kv_ok) { a = make_uint4(0, 0, 0, 0); c = make_uint4(0, 0, 0, 0); }
      fk[ks] = *reinterpret_cast<bf16x8*>(&a);
      fv[ks] = *reinterpret_cast<bf16x8*>(&c);
    }
  }
  floatx16 dkacc[DT], dvacc[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkacc[d][r] = 0.f; dvacc[d][r] = 0.f; }

  // lse (base-2 units; a row past the end gets P = 2^(-inf) = 0) and delta of the 64 queries from q0 on
  auto load_vectors = [&](float* sL, float* sD, const uint32_t q0) {
    if (threadIdx.x < AT_QB) {
      const uint32_t qq = q0 + threadIdx.x;
      sL[threadIdx.x] = qq < S ? lrow[qq] * 1.44269504088896f : INFINITY;
      sD[threadIdx.x] = qq < S ? drow[qq] : 0.f;
    }
  };
  auto tile = [&](const bf16_t* sQ, const bf16_t* sDo, const float* sL, const float* sD, const uint32_t q0) {
    // a wavefront whose 32 keys all lie after the 64 queries of this step has nothing to add
    if (CAUSAL && kw > q0 + AT_QB - 1) return;
#pragma unroll
    for (int u = 0; u < AT_QB / 32; ++u) {
      if (CAUSAL && kw > q0 + u * 32 + 31) continue;            // these 32 queries all precede the wavefront's keys (next u)
      const bool need_mask = CAUSAL && kw + 31 > q0 + u * 32;
      floatx16 sacc, pacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; pacc[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at_frag<DH>(sQ, u * 32 + ki, ks * 2 + h), fk[ks], sacc, 0, 0, 0);     // S  [q][kv]
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at_frag<DH>(sDo, u * 32 + ki, ks * 2 + h), fv[ks], pacc, 0, 0, 0);    // dP [q][kv]
      }
      float pr[16], ds[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 l4 = *reinterpret_cast<const float4*>(sL + u * 32 + g * 8 + h * 4);
        const float4 d4 = *reinterpret_cast<const float4*>(sD + u * 32 + g * 8 + h * 4);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = g * 4 + e;
          float p = at_round(__builtin_amdgcn_exp2f(fmaf(sacc[r], c2, -lv[e])));
          if (need_mask) p = kv <= q0 + u * 32 + g * 8 + h * 4 + e ? p : 0.f;
          pr[r] = p;
          ds[r] = p * scale * (pacc[r] - dv[e]);
        }
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8 fp = at_pack8(pr, 8 * s2), fds = at_pack8(ds, 8 * s2);
        const uint32_t qb = u * 32 + 16 * s2 + 4 * h;
#pragma unroll
        for (int d = 0; d < DT; ++d) {
          dvacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at_frag_tr<DH>(sDo, d * 32, qb), fp, dvacc[d], 0, 0, 0);     // dV^T
          dkacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at_frag_tr<DH>(sQ, d * 32, qb), fds, dkacc[d], 0, 0, 0);     // dK^T
        }
      }
    }
  };
  const uint32_t q_first = CAUSAL ? (kv_blk / AT_QB) * AT_QB : 0;
  if constexpr (DB) {
    if (q_first < S) {
      at_dma_rows<DH, AT_QB>(sQ0, base, ld_qkv, q_first, S);
      at_dma_rows<DH, AT_QB>(sDo0, dobase, ld_o, q_first, S);
      load_vectors(sL0, sD0, q_first);
    }
    for (uint32_t q0 = q_first; q0 < S; q0 += 2 * AT_QB) {
      wait_fetches();
      __syncthreads();                                   // step q0 has landed, nobody reads buffer 1 any more
      const bool more = q0 + AT_QB < S;
      if (more) {
        at_dma_rows<DH, AT_QB>(sQ1, base, ld_qkv, q0 + AT_QB, S);
        at_dma_rows<DH, AT_QB>(sDo1, dobase, ld_o, q0 + AT_QB, S);
        load_vectors(sL1, sD1, q0 + AT_QB);
      }
      tile(sQ0, sDo0, sL0, sD0, q0);
      if (more) {
        wait_fetches();
        __syncthreads();
        if (q0 + 2 * AT_QB < S) {
          at_dma_rows<DH, AT_QB>(sQ0, base, ld_qkv, q0 + 2 * AT_QB, S);
          at_dma_rows<DH, AT_QB>(sDo0, dobase, ld_o, q0 + 2 * AT_QB, S);
          load_vectors(sL0, sD0, q0 + 2 * AT_QB);
        }
        tile(sQ1, sDo1, sL1, sD1, q0 + AT_QB);
      }
    }
  } else {
    for (uint32_t q0 = q_first; q0 < S; q0 += AT_QB) {
      __syncthreads();
      at_load_rows<DH, AT_QB>(sQ0, base, ld_qkv, q0, S);
      at_load_rows<DH, AT_QB>(sDo0, dobase, ld_o, q0, S);
      load_vectors(sL0, sD0, q0);
      __syncthreads();
      tile(sQ0, sDo0, sL0, sD0, q0);
    }
  }
  __syncthreads();                                         // nobody reads the last Q/dO step any more: its buffers stage dk, then dv
  {
    bf16_t* stage = (wave < 2 ? sQ0 : sDo0) + (wave & 1) * (32 * DH);
    bf16_t* kp = dqkv + ((size_t)b * S + kw) * ld_dqkv + da + head * DH;
    const uint32_t rows = kw < S ? S - kw : 0u;
    at_store_tile<DH>(stage, dkacc, 1.0f, kp, ld_dqkv, rows);
    at_store_tile<DH>(stage, dvacc, 1.0f, kp + da, ld_dqkv, rows);
  }
  kernel_end(ctl, true);
}

static sif_status attn_check(const char* who, uint32_t batch, uint32_t seq, uint32_t heads, uint32_t d_head) {
  if (!batch || !seq || !heads) return fail(SIF_E_INVAL, "%s: empty extent", who);
  if (d_head != 64 && d_head != 128) return fail(SIF_E_INVAL, "%s: d_head must be 64 or 128", who);
  if ((seq + AT_Q - 1) / AT_Q > 65535) return fail(SIF_E_INVAL, "%s: sequence too long", who);
  return SIF_OK;
}
static bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

sif_status launch_attn_fwd(const void* qkv, void* o, float* lse, uint32_t batch, uint32_t seq, uint32_t heads, uint32_t d_head, uint32_t ld_qkv,
                           uint32_t ld_o, uint32_t causal, hipStream_t s, const KCtl& c) {
  if (!qkv || !o) return fail(SIF_E_INVAL, "attn_fwd: null operand");
  if (sif_status st = attn_check("attn_fwd", batch, seq, heads, d_head)) return st;
  if ((ld_qkv & 7) || (ld_o & 7) || ld_qkv < 3 * heads * d_head || ld_o < heads * d_head) return fail(SIF_E_INVAL, "attn_fwd: bad leading dimensions");
  if (!al16(qkv) || !al16(o)) return fail(SIF_E_INVAL, "attn_fwd: pointers must be 16-byte aligned");
  const float scale = 1.0f / sqrtf((float)d_head);
  dim3 grid(batch * heads, (seq + AT_Q - 1) / AT_Q);
  AttnSeqs seqs;
  seqs.n = 0;
#define AT_LAUNCH(DH, C) hipLaunchKernelGGL((attn_fwd_kernel<DH, C>), grid, dim3(AT_THREADS), 0, s, (const bf16_t*)qkv, (bf16_t*)o, lse, seq, heads, ld_qkv, ld_o, scale, seqs, c)
  if (d_head == 64) { if (causal) AT_LAUNCH(64, 1); else AT_LAUNCH(64, 0); }
  else { if (causal) AT_LAUNCH(128, 1); else AT_LAUNCH(128, 0); }
  return check_launch("attn_fwd");
}

sif_status launch_attn_fwd_varlen(const void* qkv, void* o, const uint32_t* starts, uint32_t n_seqs, uint32_t heads, uint32_t d_head,
                                  uint32_t ld_qkv, uint32_t ld_o, uint32_t causal, hipStream_t s, const KCtl& c) {
  if (!qkv || !o || !starts) return fail(SIF_E_INVAL, "attn_fwd_varlen: null operand");
  if (n_seqs == 0 || n_seqs > kAttnMaxSeqs) return fail(SIF_E_INVAL, "attn_fwd_varlen: 1 to %u sequences", kAttnMaxSeqs);
  AttnSeqs seqs;
  seqs.n = n_seqs;
  uint32_t longest = 0;
  for (uint32_t i = 0; i <= n_seqs; ++i) {
    seqs.start[i] = starts[i];
    if (i > 0) {
      if (starts[i] <= starts[i - 1]) return fail(SIF_E_INVAL, "attn_fwd_varlen: sequence starts must ascend (no empty sequence)");
      longest = std::max(longest, starts[i] - starts[i - 1]);
    }
  }
  for (uint32_t i = n_seqs + 1; i <= kAttnMaxSeqs; ++i) seqs.start[i] = starts[n_seqs];
  if (sif_status st = attn_check("attn_fwd_varlen", n_seqs, longest, heads, d_head)) return st;
  if ((ld_qkv & 7) || (ld_o & 7) || ld_qkv < 3 * heads * d_head || ld_o < heads * d_head) return fail(SIF_E_INVAL, "attn_fwd_varlen: bad leading dimensions");
  if (!al16(qkv) || !al16(o)) return fail(SIF_E_INVAL, "attn_fwd_varlen: pointers must be 16-byte aligned");
  const float scale = 1.0f / sqrtf((float)d_head);
  float* lse = nullptr;
  const uint32_t seq = longest;
  dim3 grid(n_seqs * heads, (longest + AT_Q - 1) / AT_Q);
  if (d_head == 64) { if (causal) AT_LAUNCH(64, 1); else AT_LAUNCH(64, 0); }
  else { if (causal) AT_LAUNCH(128, 1); else AT_LAUNCH(128, 0); }
#undef AT_LAUNCH
  return check_launch("attn_fwd_varlen");
}

static sif_status attn_bwd_check(const char* who, const void* qkv, const void* o, const void* d_o, const float* lse, const float* delta,
                                 const void* dqkv, uint32_t batch, uint32_t seq, uint32_t heads, uint32_t d_head, uint32_t ld_qkv,
                                 uint32_t ld_o, uint32_t ld_dqkv) {
  if (!qkv || !o || !d_o || !lse || !delta || !dqkv) return fail(SIF_E_INVAL, "%s: null operand", who);
  if (sif_status st = attn_check(who, batch, seq, heads, d_head)) return st;
  if ((ld_qkv & 7) || (ld_o & 7) || (ld_dqkv & 7) || ld_qkv < 3 * heads * d_head || ld_dqkv < 3 * heads * d_head || ld_o < heads * d_head)
    return fail(SIF_E_INVAL, "%s: bad leading dimensions", who);
  if (!al16(qkv) || !al16(o) || !al16(d_o) || !al16(dqkv)) return fail(SIF_E_INVAL, "%s: pointers must be 16-byte aligned", who);
  return SIF_OK;
}

sif_status launch_attn_bwd_dq(const void* qkv, const void* o, const void* d_o, const float* lse, float* delta, void* dqkv, uint32_t batch,
                              uint32_t seq, uint32_t heads, uint32_t d_head, uint32_t ld_qkv, uint32_t ld_o, uint32_t ld_dqkv, uint32_t causal,
                              hipStream_t s, const KCtl& c) {
  if (sif_status st = attn_bwd_check("attn_bwd_dq", qkv, o, d_o, lse, delta, dqkv, batch, seq, heads, d_head, ld_qkv, ld_o, ld_dqkv)) return st;
  const float scale = 1.0f / sqrtf((float)d_head);
  dim3 grid(batch * heads, (seq + AT_Q - 1) / AT_Q);
#define AT_LAUNCH(DH, C) hipLaunchKernelGGL((attn_bwd_dq_kernel<DH, C>), grid, dim3(AT_THREADS), 0, s, (const bf16_t*)qkv, (const bf16_t*)o, \
                                            (const bf16_t*)d_o, lse, delta, (bf16_t*)dqkv, seq, heads, ld_qkv, ld_o, ld_dqkv, scale, c)
  if (d_head == 64) { if (causal) AT_LAUNCH(64, 1); else AT_LAUNCH(64, 0); }
  else { if (causal) AT_LAUNCH(128, 1); else AT_LAUNCH(128, 0); }
#undef AT_LAUNCH
  return check_launch("attn_bwd_dq");
}

sif_status launch_attn_bwd_dkv(const void* qkv, const void* d_o, const float* lse, const float* delta, void* dqkv, uint32_t batch, uint32_t seq,
                               uint32_t heads, uint32_t d_head, uint32_t ld_qkv, uint32_t ld_o, uint32_t ld_dqkv, uint32_t causal, hipStream_t s,
                               const KCtl& c) {
  if (sif_status st = attn_bwd_check("attn_bwd_dkv", qkv, d_o, d_o, lse, delta, dqkv, batch, seq, heads, d_head, ld_qkv, ld_o, ld_dqkv)) return st;
  const float scale = 1.0f / sqrtf((float)d_head);
  dim3 grid(batch * heads, (seq + AT_KV - 1) / AT_KV);
#define AT_LAUNCH(DH, C) hipLaunchKernelGGL((attn_bwd_dkv_kernel<DH, C>), grid, dim3(AT_THREADS), 0, s, (const bf16_t*)qkv, (const bf16_t*)d_o, lse, \
                                            delta, (bf16_t*)dqkv, seq, heads, ld_qkv, ld_o, ld_dqkv, scale, c)
  if (d_head == 64) { if (causal) AT_LAUNCH(64, 1); else AT_LAUNCH(64, 0); }
  else { if (causal) AT_LAUNCH(128, 1); else AT_LAUNCH(128, 0); }
#undef AT_LAUNCH
  return check_launch("attn_bwd_dkv");
}

}  // namespace sif
