// Shared device helpers: bfloat16 conversion (upper 16 bits of binary32, round to nearest even), exact-erf GELU,
// block reductions with a fixed order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "monitor.h"

namespace sif {

typedef uint16_t bf16_t;

__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
// float -> bfloat16, round to nearest even, by the gfx950 conversion instruction (v_cvt_pk_bf16_f32 takes two values)
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
typedef float floatx2_hw __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
__device__ __forceinline__ float bflo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bfhi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t pack_bf2(float lo, float hi) {
  const floatx2_hw v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_hw));
}

// erf by the rational approximation 7.1.26 of Abramowitz & Stegun (|error| <= 1.5e-7), a dozen instructions
// instead of the library routine's fifty: the GELU epilogue runs on every element of the widest activations.
__device__ __forceinline__ float erf_fast(float x) {
  const float ax = fabsf(x);
  const float t = __frcp_rn(1.0f + 0.3275911f * ax);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float r = 1.0f - poly * __expf(-ax * ax);
  return copysignf(r, x);
}
__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.0f + erf_fast(x * 0.70710678118654752f)); }

// GELU(x) = x Phi(x) for the bf16 epilogues, where it runs on every element of the widest activations: with
// t = |x|, 1 - Phi(t) = 2^p(t) / 2 and p(t) = log2 erfc(t / sqrt 2) ~ t (c0 + c1 t + c2 t^2 + c3 t^3 + c4 t^4), a
// fit of this build (gelu_fit.py beside this file derives the constants; largest absolute error of GELU 9.1e-7, of
// GELU' 7.8e-7 in float arithmetic, far below a bf16 rounding).  One exponential and no division per value.
__device__ __forceinline__ float upper_tail_fast(float t) {       // 1 - Phi(t) for t >= 0
  const float r = fmaf(fmaf(fmaf(fmaf(-0.000502793584f, t, 0.00730014686f), t, -0.0523868538f), t, -0.459369212f), t, -1.15106988f);
  return 0.5f * __builtin_amdgcn_exp2f(t * r);
}
// GELU(x) = max(x, 0) - |x| (1 - Phi(|x|)): for x < 0 that is x (1 - Phi(-x)) = x Phi(x), for x >= 0 x - x (1 - Phi(x)).
// The factor 1/2 goes into the exponent: eleven issue slots per value (five fused multiply-adds, the exponential
// counting four, one maximum, one more fused multiply-add), no comparison and no select.
__device__ __forceinline__ float gelu_fast(float x) {
  const float t = fabsf(x);
  const float r = fmaf(fmaf(fmaf(fmaf(-0.000502793584f, t, 0.00730014686f), t, -0.0523868538f), t, -0.459369212f), t, -1.15106988f);
  const float h = __builtin_amdgcn_exp2f(fmaf(t, r, -1.0f));
  return fmaf(-t, h, fmaxf(x, 0.f));
}
__device__ __forceinline__ float gelu_grad_fast(float x) {
  const float h = upper_tail_fast(fabsf(x));
  const float pdf = 0.3989422804f * __builtin_amdgcn_exp2f(-0.72134752f * x * x);
  return fmaf(x, pdf, x < 0.f ? h : 1.0f - h);
}
__device__ __forceinline__ float gelu_grad_f(float x) {
  float cdf = 0.5f * (1.0f + erf_fast(x * 0.70710678118654752f));
  float pdf = 0.3989422804014327f * __expf(-0.5f * x * x);
  return cdf + x * pdf;
}

// Sum over a wavefront (64 lanes) with a fixed butterfly order; every lane gets the result.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// Block-wide sum for blocks of up to 1024 threads (blockDim.x a multiple of 64); `sm` holds >= 16 floats.
__device__ __forceinline__ float block_sum(float v, float* sm) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += sm[i];
  return t;
}
__device__ __forceinline__ float block_max(float v, float* sm) {
  v = wave_max(v);
  int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[w] = v;
  __syncthreads();
  float t = sm[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, sm[i]);
  return t;
}

// Waits until every global -> LDS fetch (and every other vector memory operation) this wavefront has issued is
// complete: s_waitcnt vmcnt(0), the other counters left alone.  A barrier that hands fetched tiles to the other
// wavefronts of the block needs it in front: __syncthreads() by itself orders LDS accesses, but the compiler waits for
// a wavefront's own fetches only where that wavefront reads the buffer, which may be after the barrier, and then
// another wavefront's part of the tile need not have landed.
__device__ __forceinline__ void wait_fetches() { __builtin_amdgcn_s_waitcnt(0x0F70); }

}  // namespace sif
