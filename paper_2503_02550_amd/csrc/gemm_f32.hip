// fp32 matrix product with arbitrary element strides and fused bias / GELU / GELU' epilogues, for the Tiny
// configuration (two 256x256 Linear layers, batch 32 / 8).  At that size a product is a few MFLOP and bound by
// launch latency, so this is a plain LDS-tiled FMA kernel: 32x32 tile per block, 256 threads, 2x2 outputs per
// thread, K reduced in ascending order (grid-independent results).
#include "common.h"
#include "launch.h"

namespace sif {

__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ a, long long a_sm, long long a_sk,
                                                       const float* __restrict__ b, long long b_sk, long long b_sn,
                                                       float* __restrict__ c, long long ldc, uint32_t m, uint32_t n, uint32_t k,
                                                       uint32_t epi, const float* __restrict__ bias, float* __restrict__ aux, KCtl ctl) {
  __shared__ float sa[32][33], sb[32][33];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const uint32_t m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  float acc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
  for (uint32_t k0 = 0; k0 < k; k0 += 32) {
    for (uint32_t e = threadIdx.x; e < 1024; e += 256) {
      const uint32_t r = e >> 5, kk = e & 31;
      sa[r][kk] = (m0 + r < m && k0 + kk < k) ? a[(long long)(m0 + r) * a_sm + (long long)(k0 + kk) * a_sk] : 0.f;
      sb[kk][r] = (n0 + r < n && k0 + kk < k) ? b[(long long)(k0 + kk) * b_sk + (long long)(n0 + r) * b_sn] : 0.f;
    }
    __syncthreads();
#pragma unroll 8
    for (uint32_t kk = 0; kk < 32; ++kk) {
      const float a0 = sa[ty][kk], a1 = sa[ty + 16][kk], b0 = sb[kk][tx], b1 = sb[kk][tx + 16];
      acc[0][0] = fmaf(a0, b0, acc[0][0]); acc[0][1] = fmaf(a0, b1, acc[0][1]);
      acc[1][0] = fmaf(a1, b0, acc[1][0]); acc[1][1] = fmaf(a1, b1, acc[1][1]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 2; ++i)
    for (int j = 0; j < 2; ++j) {
      const uint32_t mm = m0 + ty + 16 * i, nn = n0 + tx + 16 * j;
      if (mm < m && nn < n) {
        const long long idx = (long long)mm * ldc + nn;
        float v = acc[i][j] + (bias != nullptr ? bias[nn] : 0.f);
        if (epi & SIF_EPI_GELU) { if (aux != nullptr) aux[idx] = v; v = gelu_f(v); }
        if (epi & SIF_EPI_GELU_GRAD) v *= gelu_grad_f(aux[idx]);
        c[idx] = v;
      }
    }
  kernel_end(ctl, true);
}

sif_status launch_gemm_f32(const float* a, int64_t a_sm, int64_t a_sk, const float* b, int64_t b_sk, int64_t b_sn,
                           float* c, int64_t ldc, uint32_t m, uint32_t n, uint32_t k, uint32_t epi, const float* bias,
                           float* aux, hipStream_t s, const KCtl& ctl) {
  if (!a || !b || !c) return fail(SIF_E_INVAL, "gemm_f32: null operand");
  if (m == 0 || n == 0 || k == 0) return fail(SIF_E_INVAL, "gemm_f32: empty extent");
  if (ldc < (int64_t)n) return fail(SIF_E_INVAL, "gemm_f32: ldc too small");
  if ((epi & SIF_EPI_GELU_GRAD) && !aux) return fail(SIF_E_INVAL, "gemm_f32: GELU_GRAD needs aux");
  if (epi & ~(uint32_t)(SIF_EPI_BIAS | SIF_EPI_GELU | SIF_EPI_GELU_GRAD)) return fail(SIF_E_INVAL, "gemm_f32: unsupported epilogue");
  dim3 grid((n + 31) / 32, (m + 31) / 32);
  if (grid.y > 65535) return fail(SIF_E_INVAL, "gemm_f32: grid too large");
  hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, s, a, (long long)a_sm, (long long)a_sk, b, (long long)b_sk,
                     (long long)b_sn, c, (long long)ldc, m, n, k, epi, (epi & (SIF_EPI_BIAS | SIF_EPI_GELU)) ? bias : nullptr, aux, ctl);
  return check_launch("gemm_f32");
}

}  // namespace sif
