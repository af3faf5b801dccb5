// Fused attention forward for the inference instance: o = softmax(scale q k^T [+ causal mask]) v per (batch, head),
// without materialising the score matrix in HBM (the unfused path writes and re-reads 4 + 2 bytes per score and
// costs three launches per layer; an inference forward is a chain of short, launch-bound kernels, Sec. 3.3
// "Kernel Barrier": "most kernel execution times under 1 ms").
//
// One block = 128 query rows of one (batch, head), 4 wavefronts x 32 rows.  Keys/values are streamed in tiles of
// 128 through LDS: K as [kv][d] (16-byte chunks XOR-swizzled), V transposed to [d][kv] on the way in.  Both
// products are computed transposed, S^T = K Q^T and O^T = V^T P^T, so that a query row lives in one lane (and its
// partner lane 32 further): the softmax reductions are in-register plus one cross-lane exchange, the running
// maximum / sum / rescale of the streaming softmax are per-lane scalars, and the probabilities go from the
// accumulator registers of the first product straight into the operand registers of the second (the k-index
// permutation this implies is applied to the V^T operand reads).  bf16 operands, fp32 accumulation and softmax.
#include <math.h>

#include "common.h"
#include "launch.h"

namespace sif {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int AT_Q = 128, AT_KV = 128, AT_THREADS = 256, AT_VLD = AT_KV + 4;   // V^T rows padded by 8 bytes

__device__ __forceinline__ uint32_t at_key(uint32_t row) { return (row & 7u) ^ ((row >> 3) & 1u); }

template <int DH, int CAUSAL>
__global__ __launch_bounds__(AT_THREADS) void attn_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o, uint32_t S,
                                                              uint32_t H, uint32_t ld_qkv, uint32_t ld_o, float scale, KCtl ctl) {
  constexpr int KS = DH / 16, DT = DH / 32, CH = DH / 8;      // k steps of q k^T, 32-wide d tiles, 16-byte chunks per K row
  __shared__ __align__(16) bf16_t sK[AT_KV * DH];
  __shared__ __align__(16) bf16_t sVt[DH * AT_VLD];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, qi = lane & 31, h = lane >> 5;
  const uint32_t b = blockIdx.y / H, head = blockIdx.y % H, da = H * DH;
  const bf16_t* base = qkv + (size_t)b * S * ld_qkv + head * DH;
  const uint32_t q_blk = blockIdx.x * AT_Q, q = q_blk + wave * 32 + qi;

  bf16x8 fq[KS];
  {
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
  float m_run = -INFINITY, l_run = 0.f;

  const uint32_t kv_end = CAUSAL ? min(S, q_blk + AT_Q) : S;
  for (uint32_t kv0 = 0; kv0 < kv_end; kv0 += AT_KV) {
    __syncthreads();
    // K tile: 128 rows x CH chunks
    for (uint32_t v = threadIdx.x; v < AT_KV * CH; v += AT_THREADS) {
      const uint32_t row = v / CH, c = v % CH, kv = kv0 + row;
      uint4 x = make_uint4(0, 0, 0, 0);
      if (kv < S) x = *reinterpret_cast<const uint4*>(base + da + (size_t)kv * ld_qkv + c * 8);
      *reinterpret_cast<uint4*>(sK + row * DH + ((c ^ (at_key(row) % CH)) << 3)) = x;
    }
    // V tile transposed: each thread takes 4 kv rows x 8 d columns and writes eight 4-long kv runs
    for (uint32_t sb = threadIdx.x; sb < (AT_KV / 4) * CH; sb += AT_THREADS) {
      const uint32_t kvq = (sb / CH) * 4, d0 = (sb % CH) * 8;
      uint32_t w[4][4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint4 x = make_uint4(0, 0, 0, 0);
        if (kv0 + kvq + i < S) x = *reinterpret_cast<const uint4*>(base + 2 * da + (size_t)(kv0 + kvq + i) * ld_qkv + d0);
        w[i][0] = x.x; w[i][1] = x.y; w[i][2] = x.z; w[i][3] = x.w;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint2 even, odd;
        even.x = (w[0][j] & 0xFFFFu) | (w[1][j] << 16);  even.y = (w[2][j] & 0xFFFFu) | (w[3][j] << 16);
        odd.x = (w[0][j] >> 16) | (w[1][j] & 0xFFFF0000u);  odd.y = (w[2][j] >> 16) | (w[3][j] & 0xFFFF0000u);
        *reinterpret_cast<uint2*>(sVt + (d0 + 2 * j) * AT_VLD + kvq) = even;
        *reinterpret_cast<uint2*>(sVt + (d0 + 2 * j + 1) * AT_VLD + kvq) = odd;
      }
    }
    __syncthreads();

    // S^T tiles: rows = kv (32 per tile), columns = the wavefront's 32 query rows
    floatx16 sacc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[t][r] = 0.f;
      const uint32_t row = t * 32 + qi;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 fk = *reinterpret_cast<const bf16x8*>(sK + row * DH + ((((uint32_t)ks * 2 + h) ^ (at_key(row) % CH)) << 3));
        sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk, fq[ks], sacc[t], 0, 0, 0);
      }
    }
    // mask, running maximum
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t kv = kv0 + t * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
        const bool ok = kv < S && (!CAUSAL || kv <= q);
        sacc[t][r] = ok ? sacc[t][r] * scale : -INFINITY;
        mx = fmaxf(mx, sacc[t][r]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;          // a fully masked row keeps everything at zero
    const float alpha = __expf(m_run - m_use);                         // exp(-inf) = 0 on the first tile
    float rs = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[t][r] = __expf(sacc[t][r] - m_use); rs += sacc[t][r]; }
    rs += __shfl_xor(rs, 32, 64);
    l_run = l_run * alpha + rs;
    m_run = m_new;
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[d][r] *= alpha;
    // a single tile covers all keys: normalise before rounding, as the unfused path (and the oracle) do
    const bool single = kv_end <= AT_KV;
    const float pn = single ? 1.0f / l_run : 1.0f;

    // O^T += V^T P^T.  Element e of step s2 in tile t is key  t*32 + 16*s2 + 8*(e/4) + 4*h + e%4.
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        uint32_t pw[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) pw[e] = pack_bf2(sacc[t][8 * s2 + 2 * e] * pn, sacc[t][8 * s2 + 2 * e + 1] * pn);
        uint4 pv = make_uint4(pw[0], pw[1], pw[2], pw[3]);
        const bf16x8 fp = *reinterpret_cast<bf16x8*>(&pv);
        const uint32_t kvb = t * 32 + 16 * s2 + 4 * h;
#pragma unroll
        for (int d = 0; d < DT; ++d) {
          const bf16_t* vr = sVt + (d * 32 + qi) * AT_VLD + kvb;
          const uint2 lo = *reinterpret_cast<const uint2*>(vr), hi = *reinterpret_cast<const uint2*>(vr + 8);
          uint4 vv = make_uint4(lo.x, lo.y, hi.x, hi.y);
          const bf16x8 fv = *reinterpret_cast<bf16x8*>(&vv);
          oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv, fp, oacc[d], 0, 0, 0);
        }
      }
    if (single) l_run = 1.0f;
  }

  if (q < S) {
    const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
    bf16_t* op = o + ((size_t)b * S + q) * ld_o + head * DH;
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint32_t dd = d * 32 + g * 8 + h * 4;
        *reinterpret_cast<uint2*>(op + dd) = make_uint2(pack_bf2(oacc[d][4 * g] * inv, oacc[d][4 * g + 1] * inv),
                                                        pack_bf2(oacc[d][4 * g + 2] * inv, oacc[d][4 * g + 3] * inv));
      }
  }
  kernel_end(ctl, true);
}

sif_status launch_attn_fwd(const void* qkv, void* o, uint32_t batch, uint32_t seq, uint32_t heads, uint32_t d_head, uint32_t ld_qkv,
                           uint32_t ld_o, uint32_t causal, hipStream_t s, const KCtl& c) {
  if (!qkv || !o || !batch || !seq || !heads) return fail(SIF_E_INVAL, "attn_fwd: null or empty");
  if (d_head != 64 && d_head != 128) return fail(SIF_E_INVAL, "attn_fwd: d_head must be 64 or 128");
  if ((ld_qkv & 7) || (ld_o & 7) || ld_qkv < 3 * heads * d_head || ld_o < heads * d_head) return fail(SIF_E_INVAL, "attn_fwd: bad leading dimensions");
  if (((uintptr_t)qkv & 15) || ((uintptr_t)o & 15)) return fail(SIF_E_INVAL, "attn_fwd: pointers must be 16-byte aligned");
  if (batch * heads > 65535) return fail(SIF_E_INVAL, "attn_fwd: batch*heads too large");
  const float scale = 1.0f / sqrtf((float)d_head);
  dim3 grid((seq + AT_Q - 1) / AT_Q, batch * heads);
#define AT_LAUNCH(DH, C) hipLaunchKernelGGL((attn_fwd_kernel<DH, C>), grid, dim3(AT_THREADS), 0, s, (const bf16_t*)qkv, (bf16_t*)o, seq, heads, ld_qkv, ld_o, scale, c)
  if (d_head == 64) { if (causal) AT_LAUNCH(64, 1); else AT_LAUNCH(64, 0); }
  else { if (causal) AT_LAUNCH(128, 1); else AT_LAUNCH(128, 0); }
#undef AT_LAUNCH
  return check_launch("attn_fwd");
}

}  // namespace sif
