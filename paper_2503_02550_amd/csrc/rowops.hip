// Memory-bound kernels of the training step and the inference forward pass: LayerNorm, softmax, embedding,
// cross entropy, column sums, SGD.  They are bound by HBM traffic, so each reads its operands once with 16-byte
// accesses, keeps fp32 statistics in registers / LDS, and uses fixed-order reductions (no float atomics) so
// that results are bit-identical from run to run and independent of what else shares the GPU.
#include <algorithm>

#include "common.h"
#include "launch.h"

namespace sif {

constexpr float kLnEps = 1e-5f;

// compute units of the current device (256 on MI355X), looked up once
static uint32_t n_cus() {
  static const uint32_t n = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    return (uint32_t)v;
  }();
  return n;
}

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
  f[0] = bflo(v.x); f[1] = bfhi(v.x); f[2] = bflo(v.y); f[3] = bfhi(v.y);
  f[4] = bflo(v.z); f[5] = bfhi(v.z); f[6] = bflo(v.w); f[7] = bfhi(v.w);
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  return make_uint4(pack_bf2(f[0], f[1]), pack_bf2(f[2], f[3]), pack_bf2(f[4], f[5]), pack_bf2(f[6], f[7]));
}

// ---------------------------------------------------------------------------------------------- LayerNorm
// One wavefront per row at a time, 4 wavefronts per block; a wavefront works through every (number of wavefronts)-th
// row.  MAXV > 0: the row (at most MAXV vectors of 8 columns per lane) is read once and kept in registers for the
// three passes (mean, variance, output), the next row's loads are issued before the current row is reduced so that
// they travel meanwhile, and the gains and offsets are read once per wavefront; MAXV = 0: any width, three reads per
// row.  Both variants add in the same order, so they give the same bits.
template <int MAXV>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ g,
                                                            const bf16_t* __restrict__ b, bf16_t* __restrict__ y,
                                                            float* __restrict__ mean_out, float* __restrict__ rstd_out,
                                                            uint32_t rows, uint32_t d, RowSegs segs, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  // the row is the same for the whole wavefront: as a scalar it can index the segment table in the kernel arguments
  const uint32_t lane = threadIdx.x & 63, nv = d >> 3, n_waves = gridDim.x * 4;
  uint32_t row = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
  auto out_row = [&](uint32_t r_) -> uint4* {
    if (segs.n != 0) {
      uint32_t r = 0;
      while (r + 1 < segs.n && r_ >= segs.row0[r + 1]) ++r;
      return reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(segs.ptr[r]) + (size_t)(r_ - segs.row0[r]) * d);
    }
    return reinterpret_cast<uint4*>(y + (size_t)r_ * d);
  };
  if constexpr (MAXV > 0) {
    uint4 cx[MAXV], nx[MAXV], cg[MAXV], cb[MAXV];
    auto fetch = [&](uint4 (&dst)[MAXV], uint32_t r_) {
      const uint4* xr = reinterpret_cast<const uint4*>(x + (size_t)r_ * d);
#pragma unroll
      for (int t = 0; t < MAXV; ++t) dst[t] = (lane + 64 * t < nv) ? xr[lane + 64 * t] : make_uint4(0, 0, 0, 0);
    };
    if (row < rows) {
      fetch(cx, row);
#pragma unroll
      for (int t = 0; t < MAXV; ++t) {
        const uint32_t v = lane + 64 * t;
        cg[t] = v < nv ? reinterpret_cast<const uint4*>(g)[v] : make_uint4(0, 0, 0, 0);
        cb[t] = v < nv ? reinterpret_cast<const uint4*>(b)[v] : make_uint4(0, 0, 0, 0);
      }
    }
    while (row < rows) {
      const uint32_t next = __builtin_amdgcn_readfirstlane(row + n_waves);
      if (next < rows) fetch(nx, next);
      uint4* yr = out_row(row);
      float s = 0.f, f[8];
#pragma unroll
      for (int t = 0; t < MAXV; ++t)
        if (lane + 64 * t < nv) { unpack8(cx[t], f); for (int i = 0; i < 8; ++i) s += f[i]; }
      const float mean = wave_sum(s) / (float)d;
      float q = 0.f;
#pragma unroll
      for (int t = 0; t < MAXV; ++t)
        if (lane + 64 * t < nv) { unpack8(cx[t], f); for (int i = 0; i < 8; ++i) { float u = f[i] - mean; q += u * u; } }
      const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + kLnEps);
#pragma unroll
      for (int t = 0; t < MAXV; ++t)
        if (lane + 64 * t < nv) {
          float fg[8], fb[8], o[8];
          unpack8(cx[t], f); unpack8(cg[t], fg); unpack8(cb[t], fb);
          for (int i = 0; i < 8; ++i) o[i] = (f[i] - mean) * rstd * fg[i] + fb[i];
          yr[lane + 64 * t] = pack8(o);
        }
      if (lane == 0 && mean_out != nullptr) { mean_out[row] = mean; rstd_out[row] = rstd; }
#pragma unroll
      for (int t = 0; t < MAXV; ++t) cx[t] = nx[t];
      row = next;
    }
  } else {
    for (; row < rows; row = __builtin_amdgcn_readfirstlane(row + n_waves)) {
      const uint4* xr = reinterpret_cast<const uint4*>(x + (size_t)row * d);
      uint4* yr = out_row(row);
      float s = 0.f, f[8];
      for (uint32_t v = lane; v < nv; v += 64) { unpack8(xr[v], f); for (int i = 0; i < 8; ++i) s += f[i]; }
      const float mean = wave_sum(s) / (float)d;
      float q = 0.f;
      for (uint32_t v = lane; v < nv; v += 64) { unpack8(xr[v], f); for (int i = 0; i < 8; ++i) { float t = f[i] - mean; q += t * t; } }
      const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + kLnEps);
      for (uint32_t v = lane; v < nv; v += 64) {
        float fg[8], fb[8], o[8];
        unpack8(xr[v], f); unpack8(reinterpret_cast<const uint4*>(g)[v], fg); unpack8(reinterpret_cast<const uint4*>(b)[v], fb);
        for (int i = 0; i < 8; ++i) o[i] = (f[i] - mean) * rstd * fg[i] + fb[i];
        yr[v] = pack8(o);
      }
      if (lane == 0 && mean_out != nullptr) { mean_out[row] = mean; rstd_out[row] = rstd; }
    }
  }
  kernel_end(ctl, true);
}

constexpr int LN_MAXV = 8;   // vectors of 8 columns per lane: d <= 4096
uint32_t colsum_parts(uint32_t rows) { uint32_t p = (rows + 15) / 16; return p < 1 ? 1 : (p > 512 ? 512 : p); }

// dx = res + rstd * (dy*g - mean(dy*g) - xhat * mean(dy*g*xhat)); per-block partial column sums of dy*xhat and
// dy are written to part[blk][d] and part[parts+blk][d], and with WITH_SUM those of the rounded dx to
// part[2*parts+blk][d] (dx is the upstream gradient of the bias that was added just before this LayerNorm's input
// went into a residual sum: its column sums are that bias's gradient, and come for free here).  Block b handles
// rows b*rows_per.., its wavefronts interleaved.  MAXV = vectors of 8 columns per lane; up to 4 the row stays in
// registers between the two passes.
template <int MAXV, bool WITH_SUM>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x,
                                                            const bf16_t* __restrict__ g, const float* __restrict__ mean,
                                                            const float* __restrict__ rstd, const bf16_t* __restrict__ res,
                                                            bf16_t* __restrict__ dx, float* __restrict__ part,
                                                            uint32_t rows, uint32_t d, uint32_t parts, KCtl ctl) {
  constexpr bool CACHE = MAXV <= 4;
  constexpr int NSUM = WITH_SUM ? 3 : 2;
  __shared__ float sred[4 * 512];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nv = d >> 3;
  const uint32_t rows_per = (rows + parts - 1) / parts;
  const uint32_t r_begin = blockIdx.x * rows_per, r_end = min(rows, r_begin + rows_per);
  float acc[NSUM][MAXV][8];
#pragma unroll
  for (int w = 0; w < NSUM; ++w)
#pragma unroll
    for (int t = 0; t < MAXV; ++t)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[w][t][i] = 0.f;
  uint4 cg[CACHE ? MAXV : 1];
  if (CACHE) {
#pragma unroll
    for (int t = 0; t < MAXV; ++t) cg[t] = (lane + 64 * t < nv) ? reinterpret_cast<const uint4*>(g)[lane + 64 * t] : make_uint4(0, 0, 0, 0);
  }
  // (CACHE) the wavefront's next row is requested before the current one is worked on
  uint4 cdy[CACHE ? MAXV : 1], cx[CACHE ? MAXV : 1], cres[CACHE ? MAXV : 1];
  uint4 ndy[CACHE ? MAXV : 1], nx[CACHE ? MAXV : 1], nres[CACHE ? MAXV : 1];
  float mu = 0.f, rs = 0.f, nmu = 0.f, nrs = 0.f;
  auto fetch_row = [&](uint32_t r_, uint4 (&qdy)[CACHE ? MAXV : 1], uint4 (&qx)[CACHE ? MAXV : 1], uint4 (&qres)[CACHE ? MAXV : 1], float& qmu, float& qrs) {
    const uint4* dyr = reinterpret_cast<const uint4*>(dy + (size_t)r_ * d);
    const uint4* xr = reinterpret_cast<const uint4*>(x + (size_t)r_ * d);
#pragma unroll
    for (int t = 0; t < (CACHE ? MAXV : 1); ++t) {
      const uint32_t v = lane + 64 * t;
      qdy[t] = v < nv ? dyr[v] : make_uint4(0, 0, 0, 0);
      qx[t] = v < nv ? xr[v] : make_uint4(0, 0, 0, 0);
      qres[t] = (res != nullptr && v < nv) ? reinterpret_cast<const uint4*>(res + (size_t)r_ * d)[v] : make_uint4(0, 0, 0, 0);
    }
    qmu = mean[r_]; qrs = rstd[r_];
  };
  if (CACHE && r_begin + wave < r_end) fetch_row(r_begin + wave, ndy, nx, nres, nmu, nrs);
  for (uint32_t row = r_begin + wave; row < r_end; row += 4) {
    const uint4* dyr = reinterpret_cast<const uint4*>(dy + (size_t)row * d);
    const uint4* xr = reinterpret_cast<const uint4*>(x + (size_t)row * d);
    if (CACHE) {
#pragma unroll
      for (int t = 0; t < MAXV; ++t) { cdy[t] = ndy[t]; cx[t] = nx[t]; cres[t] = nres[t]; }
      mu = nmu; rs = nrs;
      if (row + 4 < r_end) fetch_row(row + 4, ndy, nx, nres, nmu, nrs);
    } else {
      mu = mean[row]; rs = rstd[row];
    }
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int t = 0; t < MAXV; ++t) {
      const uint32_t v = lane + 64 * t;
      if (v < nv) {
        float fdy[8], fx[8], fg[8];
        unpack8(CACHE ? cdy[t] : dyr[v], fdy); unpack8(CACHE ? cx[t] : xr[v], fx);
        unpack8(CACHE ? cg[t] : reinterpret_cast<const uint4*>(g)[v], fg);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float xh = (fx[i] - mu) * rs, dxh = fdy[i] * fg[i];
          s1 += dxh; s2 += dxh * xh;
          acc[0][t][i] += fdy[i] * xh; acc[1][t][i] += fdy[i];
        }
      }
    }
    const float m1 = wave_sum(s1) / (float)d, m2 = wave_sum(s2) / (float)d;
#pragma unroll
    for (int t = 0; t < MAXV; ++t) {
      const uint32_t v = lane + 64 * t;
      if (v < nv) {
        float fdy[8], fx[8], fg[8], fr[8], o[8];
        unpack8(CACHE ? cdy[t] : dyr[v], fdy); unpack8(CACHE ? cx[t] : xr[v], fx);
        unpack8(CACHE ? cg[t] : reinterpret_cast<const uint4*>(g)[v], fg);
        if (res != nullptr) unpack8(CACHE ? cres[t] : reinterpret_cast<const uint4*>(res + (size_t)row * d)[v], fr);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float xh = (fx[i] - mu) * rs;
          o[i] = rs * (fdy[i] * fg[i] - m1 - xh * m2);
          if (res != nullptr) o[i] += fr[i];
        }
        const uint4 packed = pack8(o);
        reinterpret_cast<uint4*>(dx + (size_t)row * d)[v] = packed;
        if (WITH_SUM) {
          unpack8(packed, o);                  // the column sums are those of the stored (rounded) values
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[NSUM - 1][t][i] += o[i];
        }
      }
    }
  }
  // combine the four wavefronts in order 0,1,2,3, 512 columns at a time
#pragma unroll
  for (int t = 0; t < MAXV; ++t) {
    if ((uint32_t)(64 * t) >= nv) break;
#pragma unroll
    for (int which = 0; which < NSUM; ++which) {
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 8; ++i) sred[wave * 512 + lane * 8 + i] = acc[which][t][i];
      __syncthreads();
      for (uint32_t cidx = threadIdx.x; cidx < 512; cidx += 256) {
        const uint32_t col = 512 * t + cidx;
        if (col < d) {
          const float s = ((sred[cidx] + sred[512 + cidx]) + sred[1024 + cidx]) + sred[1536 + cidx];
          part[(size_t)(which * parts + blockIdx.x) * d + col] = s;
        }
      }
    }
  }
  kernel_end(ctl, true);
}

// Sum of `parts` rows of partial sums per column, in a fixed order: 1024 threads = 16 wavefronts x 64 columns;
// wavefront w adds rows w, w+16, ... in ascending order, then the 16 partial sums are added in ascending w.
__device__ __forceinline__ float fin_column(const float* __restrict__ part, uint32_t parts, uint32_t n, uint32_t col, float* sm) {
  const uint32_t w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float s = 0.f;
  if (col < n) {
    // eight loads in flight, added in ascending row order
    for (uint32_t p = w; p < parts; p += 16 * 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = (p + 16 * u < parts) ? part[(size_t)(p + 16 * u) * n + col] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
  }
  __syncthreads();
  sm[w * 64 + lane] = s;
  __syncthreads();
  float t = 0.f;
  if (w == 0)
    for (int i = 0; i < 16; ++i) t += sm[i * 64 + lane];
  return t;
}

// out[c] = bf16(sum_p part[p][c]) for dg (first `parts` rows), db (next `parts` rows) and, if dsum != null, the
// column sums of dx (third `parts` rows).
__global__ __launch_bounds__(1024) void layernorm_bwd_fin_kernel(const float* __restrict__ part, bf16_t* __restrict__ dg,
                                                                 bf16_t* __restrict__ db, bf16_t* __restrict__ dsum, uint32_t parts,
                                                                 uint32_t d, uint32_t acc, KCtl ctl) {
  __shared__ float sm[1024];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t c = blockIdx.x * 64 + (threadIdx.x & 63);
  const float sg = fin_column(part, parts, d, c, sm);
  const float sb = fin_column(part + (size_t)parts * d, parts, d, c, sm);
  const float ss = dsum != nullptr ? fin_column(part + (size_t)2 * parts * d, parts, d, c, sm) : 0.f;
  if (threadIdx.x < 64 && c < d) {
    dg[c] = f2bf(acc ? bf2f(dg[c]) + sg : sg);
    db[c] = f2bf(acc ? bf2f(db[c]) + sb : sb);
    if (dsum != nullptr) dsum[c] = f2bf(acc ? bf2f(dsum[c]) + ss : ss);
  }
  kernel_end(ctl, true);
}

// ---------------------------------------------------------------------------------------------- column sums
// grid (ceil(n/512), parts): lane owns 8 columns, wave w takes rows r_begin+w, +4, ...
__global__ __launch_bounds__(256) void colsum_part_kernel(const bf16_t* __restrict__ x, uint32_t ld, float* __restrict__ part,
                                                          uint32_t rows, uint32_t n, uint32_t parts, KCtl ctl) {
  __shared__ float sred[4 * 512];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t c0 = blockIdx.x * 512 + lane * 8;
  const uint32_t rows_per = (rows + parts - 1) / parts;
  const uint32_t r_begin = blockIdx.y * rows_per, r_end = min(rows, r_begin + rows_per);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (c0 < n) {
    // four rows in flight per wavefront; the additions keep ascending row order
    uint32_t row = r_begin + wave;
    for (; row + 12 < r_end; row += 16) {
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const uint4*>(x + (size_t)(row + 4 * u) * ld + c0);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float f[8];
        unpack8(v[u], f);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] += f[i];
      }
    }
    for (; row < r_end; row += 4) {
      float f[8];
      unpack8(*reinterpret_cast<const uint4*>(x + (size_t)row * ld + c0), f);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += f[i];
    }
  }
  for (int i = 0; i < 8; ++i) sred[wave * 512 + lane * 8 + i] = acc[i];
  __syncthreads();
  for (uint32_t cidx = threadIdx.x; cidx < 512; cidx += 256) {
    const uint32_t col = blockIdx.x * 512 + cidx;
    if (col < n) part[(size_t)blockIdx.y * n + col] = ((sred[cidx] + sred[512 + cidx]) + sred[1024 + cidx]) + sred[1536 + cidx];
  }
  kernel_end(ctl, true);
}

__global__ __launch_bounds__(1024) void colsum_fin_kernel(const float* __restrict__ part, bf16_t* __restrict__ out,
                                                          uint32_t parts, uint32_t n, uint32_t acc, KCtl ctl) {
  __shared__ float sm[1024];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t c = blockIdx.x * 64 + (threadIdx.x & 63);
  const float t = fin_column(part, parts, n, c, sm);
  if (threadIdx.x < 64 && c < n) out[c] = f2bf(acc ? bf2f(out[c]) + t : t);
  kernel_end(ctl, true);
}

// Finalize of many partial-sum sets in one launch (all the bias and LayerNorm parameter gradients of a backward
// pass): grid (column blocks of 64, items); item i sums its `parts` partial rows per column for each of its nsum
// outputs, in the same fixed order as the single kernels above.
__global__ __launch_bounds__(1024) void fin_batch_kernel(const FinItem* __restrict__ items, uint32_t acc, KCtl ctl) {
  __shared__ float sm[1024];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const FinItem it = items[blockIdx.y];
  if (blockIdx.x * 64 < it.n) {                       // uniform over the block
    const uint32_t c = blockIdx.x * 64 + (threadIdx.x & 63);
    for (uint32_t s = 0; s < it.nsum; ++s) {
      const float t = fin_column(it.part + (size_t)s * it.parts * it.n, it.parts, it.n, c, sm);
      bf16_t* out = it.out[s];
      if (threadIdx.x < 64 && c < it.n && out != nullptr) out[c] = f2bf(acc ? bf2f(out[c]) + t : t);
    }
  }
  kernel_end(ctl, true);
}

__global__ __launch_bounds__(256) void colsum_f32_kernel(const float* __restrict__ x, uint32_t ld, float* __restrict__ out,
                                                         uint32_t rows, uint32_t n, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t c = blockIdx.x * 256 + threadIdx.x;
  if (c < n) {
    float s = 0.f;
    for (uint32_t r = 0; r < rows; ++r) s += x[(size_t)r * ld + c];
    out[c] = s;
  }
  kernel_end(ctl, true);
}

// ---------------------------------------------------------------------------------------------- softmax
constexpr int SM_MAXT = 8;   // 4 columns per lane per step: cols <= 2048

// One wavefront per row; the row lives in registers.
__global__ __launch_bounds__(256) void softmax_fwd_kernel(const float* __restrict__ s, bf16_t* __restrict__ p, uint32_t rows,
                                                          uint32_t cols, uint32_t ld_s, uint32_t ld_p, uint32_t causal, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row < rows) {
    const size_t r = (size_t)blockIdx.y * rows + row;
    const uint32_t valid = causal ? min(cols, row + 1) : cols;
    const float* sr = s + r * ld_s;
    float v[SM_MAXT][4];
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < SM_MAXT; ++t) {
      const uint32_t c = (t * 64 + lane) * 4;
      if (c < valid) {
        const float4 q = *reinterpret_cast<const float4*>(sr + c);
        v[t][0] = q.x; v[t][1] = (c + 1 < valid) ? q.y : -INFINITY; v[t][2] = (c + 2 < valid) ? q.z : -INFINITY;
        v[t][3] = (c + 3 < valid) ? q.w : -INFINITY;
      } else { v[t][0] = v[t][1] = v[t][2] = v[t][3] = -INFINITY; }
#pragma unroll
      for (int i = 0; i < 4; ++i) mx = fmaxf(mx, v[t][i]);
    }
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < SM_MAXT; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) { v[t][i] = __expf(v[t][i] - mx); sum += v[t][i]; }
    const float inv = 1.0f / wave_sum(sum);
    bf16_t* pr = p + r * ld_p;
    // a causal row is only ever read up to the end of its 128-column tile (the products that consume it stop at the
    // diagonal tile), so the zero fill stops there too
    const uint32_t w_end = causal ? min(ld_p, (row / 128 + 1) * 128) : ld_p;
#pragma unroll
    for (int t = 0; t < SM_MAXT; ++t) {
      const uint32_t c = (t * 64 + lane) * 4;
      if (c < w_end) *reinterpret_cast<uint2*>(pr + c) = make_uint2(pack_bf2(v[t][0] * inv, v[t][1] * inv), pack_bf2(v[t][2] * inv, v[t][3] * inv));
    }
  }
  kernel_end(ctl, true);
}

__global__ __launch_bounds__(256) void softmax_bwd_kernel(const float* __restrict__ dp, const bf16_t* __restrict__ p,
                                                          bf16_t* __restrict__ ds, uint32_t rows, uint32_t cols, uint32_t ld,
                                                          float scale, uint32_t causal, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row < rows) {
    const size_t r = (size_t)blockIdx.y * rows + row;
    const uint32_t valid = causal ? min(cols, row + 1) : cols;
    float a[SM_MAXT][4], q[SM_MAXT][4];
    float dot = 0.f;
#pragma unroll
    for (int t = 0; t < SM_MAXT; ++t) {
      const uint32_t c = (t * 64 + lane) * 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[t][i] = 0.f; q[t][i] = 0.f; }
      if (c < valid) {
        const float4 g = *reinterpret_cast<const float4*>(dp + r * ld + c);
        const uint2 w = *reinterpret_cast<const uint2*>(p + r * ld + c);
        a[t][0] = g.x; a[t][1] = g.y; a[t][2] = g.z; a[t][3] = g.w;
        q[t][0] = bflo(w.x); q[t][1] = bfhi(w.x); q[t][2] = bflo(w.y); q[t][3] = bfhi(w.y);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (c + i >= valid) { a[t][i] = 0.f; q[t][i] = 0.f; }
          dot += a[t][i] * q[t][i];
        }
      }
    }
    dot = wave_sum(dot);
    const uint32_t w_end = causal ? min(ld, (row / 128 + 1) * 128) : ld;
#pragma unroll
    for (int t = 0; t < SM_MAXT; ++t) {
      const uint32_t c = (t * 64 + lane) * 4;
      if (c < w_end) {
        float o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = scale * q[t][i] * (a[t][i] - dot);
        *reinterpret_cast<uint2*>(ds + r * ld + c) = make_uint2(pack_bf2(o[0], o[1]), pack_bf2(o[2], o[3]));
      }
    }
  }
  kernel_end(ctl, true);
}

// ---------------------------------------------------------------------------------------------- embedding
// A token id (or a target) outside [0, vocab) is taken as the nearest valid one, so that no caller's data can make a
// kernel read or write outside the table.
__device__ __forceinline__ uint32_t clamp_id(int32_t id, uint32_t vocab) { return id < 0 ? 0u : ((uint32_t)id < vocab ? (uint32_t)id : vocab - 1u); }

__global__ __launch_bounds__(256) void embed_fwd_kernel(const int32_t* __restrict__ ids, const bf16_t* __restrict__ wte,
                                                        const bf16_t* __restrict__ wpe, bf16_t* __restrict__ x,
                                                        uint32_t tokens, uint32_t seq, uint32_t d, uint32_t vocab, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63, nv = d >> 3;
  if (t < tokens) {
    const uint4* a = reinterpret_cast<const uint4*>(wte + (size_t)clamp_id(ids[t], vocab) * d);
    const uint4* b = reinterpret_cast<const uint4*>(wpe + (size_t)(t % seq) * d);
    uint4* o = reinterpret_cast<uint4*>(x + (size_t)t * d);
    for (uint32_t v = lane; v < nv; v += 64) {
      float fa[8], fb[8], r[8];
      unpack8(a[v], fa); unpack8(b[v], fb);
      for (int i = 0; i < 8; ++i) r[i] = fa[i] + fb[i];
      o[v] = pack8(r);
    }
  }
  kernel_end(ctl, true);
}

// The same for several requests whose rows lie back to back in x: segment r reads its own token ids, positions
// restart with every sequence of seq[r] tokens.
__global__ __launch_bounds__(256) void embed_fwd_segs_kernel(RowSegs segs, const bf16_t* __restrict__ wte, const bf16_t* __restrict__ wpe,
                                                             bf16_t* __restrict__ x, uint32_t tokens, uint32_t d, uint32_t vocab, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t t = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6)), lane = threadIdx.x & 63, nv = d >> 3;
  if (t < tokens) {
    uint32_t r = 0;
    while (r + 1 < segs.n && t >= segs.row0[r + 1]) ++r;
    const uint32_t local = t - segs.row0[r];
    const uint32_t id = clamp_id(reinterpret_cast<const int32_t*>(segs.ptr[r])[local], vocab);
    const uint4* a = reinterpret_cast<const uint4*>(wte + (size_t)id * d);
    const uint4* b = reinterpret_cast<const uint4*>(wpe + (size_t)(local % segs.seq[r]) * d);
    uint4* o = reinterpret_cast<uint4*>(x + (size_t)t * d);
    for (uint32_t v = lane; v < nv; v += 64) {
      float fa[8], fb[8], q[8];
      unpack8(a[v], fa); unpack8(b[v], fb);
      for (int i = 0; i < 8; ++i) q[i] = fa[i] + fb[i];
      o[v] = pack8(q);
    }
  }
  kernel_end(ctl, true);
}

constexpr int EB_MAXC = 16;   // columns per thread: d <= 4096

// Block t owns token t.  If an earlier token has the same id the block has nothing to do; otherwise it adds the
// rows dx[j] of every token j >= t with that id, in ascending j, to dwte[id].
__global__ __launch_bounds__(256) void embed_bwd_wte_kernel(const int32_t* __restrict__ ids, const bf16_t* __restrict__ dx,
                                                            bf16_t* __restrict__ dwte, uint32_t tokens, uint32_t d, uint32_t vocab, KCtl ctl) {
  __shared__ int sflag[256];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t t = blockIdx.x;
  const uint32_t id = clamp_id(ids[t], vocab);
  int seen = 0;
  for (uint32_t j = threadIdx.x; j < t; j += 256) seen |= (clamp_id(ids[j], vocab) == id);
  if (!__syncthreads_or(seen)) {
    float acc[EB_MAXC];
#pragma unroll
    for (int i = 0; i < EB_MAXC; ++i) acc[i] = 0.f;
    for (uint32_t base = t; base < tokens; base += 256) {
      const uint32_t j = base + threadIdx.x;
      const int hit = (j < tokens) && (clamp_id(ids[j], vocab) == id);
      __syncthreads();
      sflag[threadIdx.x] = hit;
      if (__syncthreads_or(hit)) {
        for (uint32_t w = 0; w < 256; ++w) {
          if (sflag[w]) {
            const bf16_t* row = dx + (size_t)(base + w) * d;
#pragma unroll
            for (int i = 0; i < EB_MAXC; ++i) { const uint32_t c = threadIdx.x + 256 * i; if (c < d) acc[i] += bf2f(row[c]); }
          }
        }
      }
    }
    bf16_t* out = dwte + (size_t)id * d;
#pragma unroll
    for (int i = 0; i < EB_MAXC; ++i) { const uint32_t c = threadIdx.x + 256 * i; if (c < d) out[c] = f2bf(bf2f(out[c]) + acc[i]); }
  }
  kernel_end(ctl, true);
}

// The same sums (bit for bit) for up to 16384 tokens and d a multiple of 8, without every block reading every id from
// global memory twice: a block owns 32 consecutive tokens, keeps all ids in LDS, finds for its tokens in one sweep
// over them which have an earlier token with the same id (nothing to do) and which later ones (noted in a list),
// adds the rows of the tokens that have neither - nearly all, with a vocabulary much larger than the batch - as
// 16-byte vectors, and for the few that own later rows as well takes these from the list in ascending order.  A list
// that overflows (a tiny vocabulary) sends the block down the old path, on the ids in LDS.
constexpr uint32_t EB_LDS_TOKENS = 16384, EB_OWN = 32, EB_LIST = 1024;
__global__ __launch_bounds__(256) void embed_bwd_wte_lds_kernel(const int32_t* __restrict__ ids, const bf16_t* __restrict__ dx,
                                                                bf16_t* __restrict__ dwte, uint32_t tokens, uint32_t d, uint32_t vocab, KCtl ctl) {
  __shared__ uint32_t sid[EB_LDS_TOKENS];
  __shared__ uint32_t smask[8];
  __shared__ int sflag[256];
  __shared__ uint32_t s_cnt, s_list[EB_LIST];          // (own token u << 14) | later token j with the same id
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t t0 = blockIdx.x * EB_OWN, nloc = min(EB_OWN, tokens - t0), lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (uint32_t j = threadIdx.x; j < tokens; j += 256) sid[j] = clamp_id(ids[j], vocab);
  if (threadIdx.x == 0) s_cnt = 0;
  __syncthreads();
  uint32_t seen = 0, later = 0;                  // bit u: token t0 + u has an earlier / a later token with its id
  uint32_t own[EB_OWN];                          // the block's ids, the same in every lane: scalar registers
#pragma unroll
  for (uint32_t u = 0; u < EB_OWN; ++u) own[u] = __builtin_amdgcn_readfirstlane(sid[min(t0 + u, tokens - 1)]);
  const uint32_t valid = nloc >= 32 ? 0xFFFFFFFFu : (1u << nloc) - 1u;
  for (uint32_t j = threadIdx.x; j < tokens; j += 256) {
    const uint32_t idj = sid[j];
    uint32_t eq = 0;
#pragma unroll
    for (uint32_t u = 0; u < EB_OWN; ++u) eq |= idj == own[u] ? 1u << u : 0u;
    // own tokens below j: u < j - t0; own tokens above j: u > j - t0
    const uint32_t below = j <= t0 ? 0u : (j - t0 >= 32 ? 0xFFFFFFFFu : (1u << (j - t0)) - 1u);
    const uint32_t above = j < t0 ? 0xFFFFFFFFu : (j - t0 >= 31 ? 0u : ~((2u << (j - t0)) - 1u));
    seen |= eq & above & valid;
    uint32_t mine = eq & below & valid;          // own tokens that token j comes after with the same id (rare)
    later |= mine;
    while (mine) {
      const uint32_t u = __builtin_ctz(mine);
      mine &= mine - 1;
      const uint32_t k = atomicAdd(&s_cnt, 1u);
      if (k < EB_LIST) s_list[k] = (u << 14) | j;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { seen |= __shfl_xor(seen, o, 64); later |= __shfl_xor(later, o, 64); }
  if (lane == 0) { smask[wave] = seen; smask[4 + wave] = later; }
  __syncthreads();
  seen = smask[0] | smask[1] | smask[2] | smask[3];
  later = smask[4] | smask[5] | smask[6] | smask[7];
  // tokens that are alone with their id: dwte[id] += dx[t], eight columns per item, four items' loads at a time
  const uint32_t nv = d >> 3, alone = ~(seen | later) & valid, n_items = nloc * nv;
  for (uint32_t first = threadIdx.x; first < n_items; first += 4 * 256) {
    uint4 o4[4], x4[4];
    uint4* out[4];
    bool on[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t item = first + q * 256, u = min(item / nv, nloc - 1), v = item - u * nv;
      on[q] = item < n_items && ((alone >> u) & 1u);
      out[q] = reinterpret_cast<uint4*>(dwte + (size_t)sid[t0 + u] * d) + v;
      if (on[q]) { o4[q] = *out[q]; x4[q] = reinterpret_cast<const uint4*>(dx + (size_t)(t0 + u) * d)[v]; }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (!on[q]) continue;
      float a[8], b[8];
      unpack8(o4[q], a); unpack8(x4[q], b);
#pragma unroll
      for (int i = 0; i < 8; ++i) a[i] = a[i] + (0.f + b[i]);
      *out[q] = pack8(a);
    }
  }
  // tokens that are the first of several with their id: their rows in ascending order, as in embed_bwd_wte_kernel
  const uint32_t n_list = s_cnt;                 // (written before the barrier in front of the masks)
  const uint32_t first_of_several = later & ~seen & valid;
  if (n_list <= EB_LIST) {
    // a wavefront per such token, 8 columns per lane and pass: the token's own row, then again and again the lowest
    // listed token above the last one taken (nothing here waits for another wavefront)
    uint32_t todo = first_of_several;
    for (uint32_t n = 0; todo != 0; ++n) {
      const uint32_t u = __builtin_ctz(todo);
      todo &= todo - 1;
      if ((n & 3u) != wave) continue;
      const uint32_t t = t0 + u;
      for (uint32_t v0 = 0; v0 < nv; v0 += 64) {
        const uint32_t v = v0 + lane;
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        uint32_t take = t;
        while (take != kNone) {
          if (v < nv) {
            float b[8];
            unpack8(reinterpret_cast<const uint4*>(dx + (size_t)take * d)[v], b);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] += b[i];
          }
          uint32_t best = kNone;
          for (uint32_t k = lane; k < n_list; k += 64) {
            const uint32_t e = s_list[k], jj = e & 0x3FFFu;
            if ((e >> 14) == u && jj > take && jj < best) best = jj;
          }
#pragma unroll
          for (int o = 32; o > 0; o >>= 1) best = min(best, (uint32_t)__shfl_xor(best, o, 64));
          take = best;
        }
        if (v < nv) {
          uint4* out = reinterpret_cast<uint4*>(dwte + (size_t)sid[t] * d) + v;
          float a[8];
          unpack8(*out, a);
#pragma unroll
          for (int i = 0; i < 8; ++i) a[i] = a[i] + acc[i];
          *out = pack8(a);
        }
      }
    }
  } else {
    for (uint32_t u = 0; u < nloc; ++u) {
      if (!((first_of_several >> u) & 1u)) continue;
      const uint32_t t = t0 + u, id = sid[t];
      float acc[EB_MAXC];
#pragma unroll
      for (int i = 0; i < EB_MAXC; ++i) acc[i] = 0.f;
      for (uint32_t base = t; base < tokens; base += 256) {
        const uint32_t j = base + threadIdx.x;
        const int hit = (j < tokens) && (sid[j] == id);
        __syncthreads();
        sflag[threadIdx.x] = hit;
        if (__syncthreads_or(hit)) {
          for (uint32_t w = 0; w < 256; ++w) {
            if (sflag[w]) {
              const bf16_t* row = dx + (size_t)(base + w) * d;
#pragma unroll
              for (int i = 0; i < EB_MAXC; ++i) { const uint32_t c = threadIdx.x + 256 * i; if (c < d) acc[i] += bf2f(row[c]); }
            }
          }
        }
      }
      bf16_t* out = dwte + (size_t)id * d;
#pragma unroll
      for (int i = 0; i < EB_MAXC; ++i) { const uint32_t c = threadIdx.x + 256 * i; if (c < d) out[c] = f2bf(bf2f(out[c]) + acc[i]); }
    }
  }
  kernel_end(ctl, true);
}

__global__ __launch_bounds__(256) void embed_bwd_wpe_kernel(const bf16_t* __restrict__ dx, bf16_t* __restrict__ dwpe,
                                                            uint32_t tokens, uint32_t seq, uint32_t d, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t s = blockIdx.x;
  for (uint32_t c = threadIdx.x; c < d; c += 256) {
    float a = 0.f;
    for (uint32_t t = s; t < tokens; t += seq) a += bf2f(dx[(size_t)t * d + c]);
    dwpe[(size_t)s * d + c] = f2bf(a);
  }
  kernel_end(ctl, true);
}

// ---------------------------------------------------------------------------------------------- cross entropy
// One block per token; the row of logits is staged in LDS (up to 144 KB of the CU's 160 KB), reduced, and
// written back as the gradient.
__global__ __launch_bounds__(1024) void xent_kernel(bf16_t* __restrict__ logits, const int32_t* __restrict__ targets,
                                                    float* __restrict__ loss, uint32_t tokens, uint32_t vocab, uint32_t ld, KCtl ctl) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  __shared__ float sred[16];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  uint4* row_s = reinterpret_cast<uint4*>(smem_raw);
  bf16_t* row_e = reinterpret_cast<bf16_t*>(smem_raw);
  const uint32_t t = blockIdx.x, nv = ld >> 3;
  uint4* gr = reinterpret_cast<uint4*>(logits + (size_t)t * ld);
  float mx = -INFINITY;
  for (uint32_t v = threadIdx.x; v < nv; v += blockDim.x) {
    const uint4 q = gr[v];
    row_s[v] = q;
    float f[8];
    unpack8(q, f);
    for (int i = 0; i < 8; ++i) if (v * 8 + i < vocab) mx = fmaxf(mx, f[i]);
  }
  mx = block_max(mx, sred);
  float sum = 0.f;
  for (uint32_t v = threadIdx.x; v < nv; v += blockDim.x) {
    float f[8];
    unpack8(row_s[v], f);
    for (int i = 0; i < 8; ++i) if (v * 8 + i < vocab) sum += __expf(f[i] - mx);
  }
  sum = block_sum(sum, sred);
  const int32_t tg = (int32_t)clamp_id(targets[t], vocab);
  const float inv = 1.0f / sum, invn = 1.0f / (float)tokens;
  if (threadIdx.x == 0) loss[t] = (mx + __logf(sum)) - bf2f(row_e[tg]);
  __syncthreads();
  for (uint32_t v = threadIdx.x; v < nv; v += blockDim.x) {
    float f[8], o[8];
    unpack8(row_s[v], f);
    for (int i = 0; i < 8; ++i) {
      const uint32_t c = v * 8 + i;
      o[i] = c < vocab ? (__expf(f[i] - mx) * inv - (c == (uint32_t)tg ? 1.f : 0.f)) * invn : 0.f;
    }
    gr[v] = pack8(o);
  }
  kernel_end(ctl, true);
}

// The same with the row kept in registers (at most MAXV vectors of 8 columns per thread) instead of LDS, as fp32:
// the kernel is bound by its arithmetic as much as by memory (two exponentials and two dozen instructions per logit
// when written naively), so every exponential is taken once and kept, whole vectors inside the vocabulary take a path
// without per-column checks, and the target's column is corrected afterwards instead of being compared with every
// column.  Two blocks of 512 threads per CU: one row's reductions overlap the other's loads and stores.  Per row the
// values and the order of the additions are those of xent_kernel, so the results have the same bits.
template <int MAXV, int THREADS>
__global__ __launch_bounds__(THREADS, (THREADS <= 512 ? 2 : 1)) void xent_reg_kernel(bf16_t* __restrict__ logits, const int32_t* __restrict__ targets,
                                                        float* __restrict__ loss, uint32_t tokens, uint32_t vocab, uint32_t ld, KCtl ctl) {
  __shared__ float sred[16];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t t = blockIdx.x, nv = ld >> 3, nfull = vocab >> 3;      // nfull: vectors that lie wholly inside the vocabulary
  uint4* gr = reinterpret_cast<uint4*>(logits + (size_t)t * ld);
  const int32_t tg = (int32_t)clamp_id(targets[t], vocab);
  const float at_target = bf2f(logits[(size_t)t * ld + tg]);      // read before anything is written back
  float e[MAXV][8];
  {
    uint4 raw[MAXV];
#pragma unroll
    for (int k = 0; k < MAXV; ++k) {
      const uint32_t v = threadIdx.x + k * THREADS;
      raw[k] = v < nv ? gr[v] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int k = 0; k < MAXV; ++k) {
      const uint32_t v = threadIdx.x + k * THREADS;
      unpack8(raw[k], e[k]);
      if (v >= nfull) {                  // padding columns (and vectors past the row) count as minus infinity: exp gives 0
#pragma unroll
        for (int i = 0; i < 8; ++i) if (v >= nv || v * 8 + i >= vocab) e[k][i] = -INFINITY;
      }
    }
  }
  float mx = -INFINITY;
#pragma unroll
  for (int k = 0; k < MAXV; ++k)
#pragma unroll
    for (int i = 0; i < 8; ++i) mx = fmaxf(mx, e[k][i]);
  mx = block_max(mx, sred);
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < MAXV; ++k)
#pragma unroll
    for (int i = 0; i < 8; ++i) { e[k][i] = __expf(e[k][i] - mx); sum += e[k][i]; }
  sum = block_sum(sum, sred);
  const float inv = 1.0f / sum, invn = 1.0f / (float)tokens;
  if (threadIdx.x == 0) loss[t] = (mx + __logf(sum)) - at_target;
  const uint32_t v_tg = (uint32_t)tg >> 3, i_tg = (uint32_t)tg & 7u;
#pragma unroll
  for (int k = 0; k < MAXV; ++k) {
    const uint32_t v = threadIdx.x + k * THREADS;
    if (v >= nv) continue;
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = e[k][i] * inv * invn;
    if (v == v_tg) {
#pragma unroll
      for (int i = 0; i < 8; ++i) if ((uint32_t)i == i_tg) o[i] = (e[k][i] * inv - 1.f) * invn;
    }
    gr[v] = pack8(o);
  }
  kernel_end(ctl, true);
}

// The register variant as one block per CU that works through rows one after the other: the next row's loads are
// issued before the current row is reduced and travel meanwhile, the current row's stores drain during the next row's
// reductions.  A block's first two rows are fixed (blockIdx.x and blockIdx.x + gridDim.x); a monitored launch hands out
// the others through a counter in the stream's record, asked for one row ahead so that the answer is there when it
// is needed: a block that starts late (its CU was held by a kernel of the other stream) then simply takes fewer rows.
// Same values, same order of additions per row.
template <int MAXV, int THREADS>
__global__ __launch_bounds__(THREADS, 1) void xent_stream_kernel(bf16_t* __restrict__ logits, const int32_t* __restrict__ targets,
                                                                 float* __restrict__ loss, uint32_t tokens, uint32_t vocab, uint32_t ld, KCtl ctl) {
  __shared__ float sred[16];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint32_t nv = ld >> 3, nfull = vocab >> 3;
  const float invn = 1.0f / (float)tokens;
  uint4 raw[MAXV];
  auto fetch = [&](uint32_t t_) {
    const uint4* src = reinterpret_cast<const uint4*>(logits + (size_t)t_ * ld);
#pragma unroll
    for (int k = 0; k < MAXV; ++k) {
      const uint32_t v = threadIdx.x + k * THREADS;
      raw[k] = v < nv ? src[v] : make_uint4(0, 0, 0, 0);
    }
  };
  __shared__ uint32_t s_row;
  const bool dynamic = ctl.rec != nullptr;
  uint32_t t = blockIdx.x, next = blockIdx.x + gridDim.x;
  if (t < tokens) fetch(t);
  while (t < tokens) {
    uint4* gr = reinterpret_cast<uint4*>(logits + (size_t)t * ld);
    const int32_t tg = (int32_t)clamp_id(targets[t], vocab);
    const float at_target = bf2f(logits[(size_t)t * ld + tg]);      // read before anything of this row is written back
    uint32_t asked = 0;
    if (dynamic && threadIdx.x == 0) asked = atomicAdd(&ctl.rec->tile_next[0], 1u);      // the row after the next one
    float e[MAXV][8];
#pragma unroll
    for (int k = 0; k < MAXV; ++k) {
      const uint32_t v = threadIdx.x + k * THREADS;
      unpack8(raw[k], e[k]);
      if (v >= nfull) {
#pragma unroll
        for (int i = 0; i < 8; ++i) if (v >= nv || v * 8 + i >= vocab) e[k][i] = -INFINITY;
      }
    }
    if (next < tokens) fetch(next);                                   // the raw registers are free again: next row's loads go out now
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < MAXV; ++k)
#pragma unroll
      for (int i = 0; i < 8; ++i) mx = fmaxf(mx, e[k][i]);
    mx = block_max(mx, sred);
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < MAXV; ++k)
#pragma unroll
      for (int i = 0; i < 8; ++i) { e[k][i] = __expf(e[k][i] - mx); sum += e[k][i]; }
    if (threadIdx.x == 0) s_row = dynamic ? 2u * gridDim.x + asked : next + gridDim.x;
    sum = block_sum(sum, sred);                                       // (its barriers also publish s_row)
    const uint32_t after = s_row;
    const float inv = 1.0f / sum;
    if (threadIdx.x == 0) loss[t] = (mx + __logf(sum)) - at_target;
    const uint32_t v_tg = (uint32_t)tg >> 3, i_tg = (uint32_t)tg & 7u;
#pragma unroll
    for (int k = 0; k < MAXV; ++k) {
      const uint32_t v = threadIdx.x + k * THREADS;
      if (v >= nv) continue;
      float o[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = e[k][i] * inv * invn;
      if (v == v_tg) {
#pragma unroll
        for (int i = 0; i < 8; ++i) if ((uint32_t)i == i_tg) o[i] = (e[k][i] * inv - 1.f) * invn;
      }
      gr[v] = pack8(o);
    }
    t = next;
    next = after;
  }
  kernel_end(ctl, true);
}

__global__ __launch_bounds__(1024) void reduce_sum_kernel(const float* __restrict__ x, float* __restrict__ out, uint32_t n, float scale, KCtl ctl) {
  __shared__ float sred[16];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  float s = 0.f;
  for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) s += x[i];
  s = block_sum(s, sred);
  if (threadIdx.x == 0) out[0] = s * scale;
  kernel_end(ctl, true);
}

// ---------------------------------------------------------------------------------------------- optimizer
__global__ __launch_bounds__(256) void sgd_bf16_kernel(float* __restrict__ master, const bf16_t* __restrict__ grad,
                                                       bf16_t* __restrict__ work, uint64_t n, float lr, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const uint64_t nv = n >> 3;
  for (uint64_t v = (uint64_t)blockIdx.x * 256 + threadIdx.x; v < nv; v += (uint64_t)gridDim.x * 256) {
    float4 m0 = reinterpret_cast<float4*>(master)[2 * v], m1 = reinterpret_cast<float4*>(master)[2 * v + 1];
    float w[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
    if (lr != 0.f) {
      float g[8];
      unpack8(reinterpret_cast<const uint4*>(grad)[v], g);
      for (int i = 0; i < 8; ++i) w[i] = w[i] - lr * g[i];
      reinterpret_cast<float4*>(master)[2 * v] = make_float4(w[0], w[1], w[2], w[3]);
      reinterpret_cast<float4*>(master)[2 * v + 1] = make_float4(w[4], w[5], w[6], w[7]);
    }
    reinterpret_cast<uint4*>(work)[v] = pack8(w);
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 7)) {        // ragged tail
    const uint64_t i = (nv << 3) + threadIdx.x;
    float w = master[i];
    if (lr != 0.f) { w = w - lr * bf2f(grad[i]); master[i] = w; }
    work[i] = f2bf(w);
  }
  kernel_end(ctl, true);
}

__global__ __launch_bounds__(256) void sgd_f32_kernel(float* __restrict__ p, const float* __restrict__ g, uint64_t n, float lr, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256) p[i] = p[i] - lr * g[i];
  kernel_end(ctl, true);
}

// d = (y - t)/n, loss = sum (y-t)^2 / (2n); one block, fixed order.
__global__ __launch_bounds__(1024) void mse_kernel(const float* __restrict__ y, const float* __restrict__ t, float* __restrict__ d,
                                                   float* __restrict__ loss, uint32_t n, KCtl ctl) {
  __shared__ float sred[16];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  float s = 0.f;
  const float invn = 1.0f / (float)n;
  for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) { const float e = y[i] - t[i]; d[i] = e * invn; s += e * e; }
  s = block_sum(s, sred);
  if (threadIdx.x == 0 && loss != nullptr) loss[0] = 0.5f * s * invn;
  kernel_end(ctl, true);
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t* __restrict__ p, uint32_t v, uint64_t n, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256) p[i] = v;
  kernel_end(ctl, true);
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, uint64_t nv, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (uint64_t)gridDim.x * 256) dst[i] = src[i];
  kernel_end(ctl, true);
}

// out[i] = bf16([out[i] +] sum_s part[s][i]) in ascending s joins the K slices of a split weight-gradient product;
// all split products of a backward pass are done in one launch: grid (blocks, items).
__global__ __launch_bounds__(256) void reduce_splits_batch_kernel(const RedItem* __restrict__ items, uint32_t acc, KCtl ctl) {
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }
  const RedItem it = items[blockIdx.y];
  const uint64_t nv = it.n >> 3;
  for (uint64_t v = (uint64_t)blockIdx.x * 256 + threadIdx.x; v < nv; v += (uint64_t)gridDim.x * 256) {
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (acc) unpack8(reinterpret_cast<const uint4*>(it.out)[v], a);
#pragma unroll 4
    for (uint32_t s = 0; s < it.splits; ++s) {
      const float4* ps = reinterpret_cast<const float4*>(it.part + (size_t)s * it.n);
      const float4 x0 = ps[2 * v], x1 = ps[2 * v + 1];
      a[0] += x0.x; a[1] += x0.y; a[2] += x0.z; a[3] += x0.w; a[4] += x1.x; a[5] += x1.y; a[6] += x1.z; a[7] += x1.w;
    }
    reinterpret_cast<uint4*>(it.out)[v] = pack8(a);
  }
  kernel_end(ctl, true);
}

// ---------------------------------------------------------------------------------------------- launchers
static bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
#define REQ(cond, msg) do { if (!(cond)) return fail(SIF_E_INVAL, msg); } while (0)

static sif_status check_segs(const char* who, const RowSegs& segs, uint32_t rows) {
  if (segs.n == 0 || segs.n > kMaxRowSegs || segs.row0[0] != 0 || segs.row0[segs.n] != rows) return fail(SIF_E_INVAL, "%s: bad row segments", who);
  for (uint32_t r = 0; r < segs.n; ++r)
    if (segs.row0[r + 1] <= segs.row0[r] || segs.ptr[r] == nullptr || !al16(segs.ptr[r])) return fail(SIF_E_INVAL, "%s: bad row segments", who);
  return SIF_OK;
}

sif_status launch_layernorm_fwd(const void* x, const void* g, const void* b, void* y, float* mean, float* rstd,
                                uint32_t rows, uint32_t d, hipStream_t s, const KCtl& c, const RowSegs* segs) {
  REQ(x && g && b && (y || segs) && rows > 0 && d > 0, "layernorm_fwd: null or empty");
  REQ((d & 7) == 0 && al16(x) && al16(g) && al16(b) && al16(y), "layernorm_fwd: d must be a multiple of 8, pointers 16-byte aligned");
  REQ((mean == nullptr) == (rstd == nullptr), "layernorm_fwd: mean and rstd go together");
  RowSegs sg = {};
  if (segs != nullptr) {
    if (sif_status st = check_segs("layernorm_fwd", *segs, rows)) return st;
    sg = *segs;
  }
  // at most eight blocks of four wavefronts per CU: every wavefront then has a row in flight while it works on another
  const uint32_t blocks = std::min<uint32_t>((rows + 3) / 4, 8u * n_cus());
#define LNF(V) hipLaunchKernelGGL((layernorm_fwd_kernel<V>), dim3(blocks), dim3(256), 0, s, (const bf16_t*)x, (const bf16_t*)g, \
                                  (const bf16_t*)b, (bf16_t*)y, mean, rstd, rows, d, sg, c)
  if (d <= 1024) LNF(2); else if (d <= 2048) LNF(4); else LNF(0);
#undef LNF
  return check_launch("layernorm_fwd");
}

sif_status launch_layernorm_bwd_dx(const void* dy, const void* x, const void* g, const float* mean, const float* rstd, const void* res,
                                   void* dx, float* part, uint32_t rows, uint32_t d, uint32_t with_sum, hipStream_t s, const KCtl& c) {
  REQ(dy && x && g && mean && rstd && dx && part && rows > 0, "layernorm_bwd: null or empty");
  REQ((d & 7) == 0 && d <= 8 * 64 * LN_MAXV, "layernorm_bwd: d must be a multiple of 8 and <= 4096");
  REQ(al16(dy) && al16(x) && al16(g) && al16(dx) && (res == nullptr || al16(res)), "layernorm_bwd: pointers must be 16-byte aligned");
  const uint32_t parts = colsum_parts(rows);
#define LNB(V, W) hipLaunchKernelGGL((layernorm_bwd_kernel<V, W>), dim3(parts), dim3(256), 0, s, (const bf16_t*)dy, (const bf16_t*)x, \
                                     (const bf16_t*)g, mean, rstd, (const bf16_t*)res, (bf16_t*)dx, part, rows, d, parts, c)
  if (d <= 1024) { if (with_sum) LNB(2, true); else LNB(2, false); }
  else if (d <= 2048) { if (with_sum) LNB(4, true); else LNB(4, false); }
  else { if (with_sum) LNB(8, true); else LNB(8, false); }
#undef LNB
  return check_launch("layernorm_bwd");
}

sif_status launch_layernorm_bwd_fin(const float* part, void* dg, void* db, void* dsum, uint32_t rows, uint32_t d, uint32_t acc, hipStream_t s,
                                    const KCtl& c) {
  REQ(part && dg && db, "layernorm_bwd_fin: null");
  hipLaunchKernelGGL(layernorm_bwd_fin_kernel, dim3((d + 63) / 64), dim3(1024), 0, s, part, (bf16_t*)dg, (bf16_t*)db, (bf16_t*)dsum,
                     colsum_parts(rows), d, acc, c);
  return check_launch("layernorm_bwd_fin");
}

sif_status launch_colsum_part(const void* x, uint32_t ld, float* part, uint32_t rows, uint32_t n, hipStream_t s, const KCtl& c) {
  REQ(x && part && rows > 0 && n > 0, "colsum: null or empty");
  REQ((n & 7) == 0 && (ld & 7) == 0 && ld >= n && al16(x), "colsum: n and ld must be multiples of 8, x 16-byte aligned");
  const uint32_t parts = colsum_parts(rows);
  hipLaunchKernelGGL(colsum_part_kernel, dim3((n + 511) / 512, parts), dim3(256), 0, s, (const bf16_t*)x, ld, part, rows, n, parts, c);
  return check_launch("colsum_part");
}

sif_status launch_colsum_fin(const float* part, void* out, uint32_t rows, uint32_t n, uint32_t acc, hipStream_t s, const KCtl& c) {
  REQ(part && out, "colsum_fin: null");
  hipLaunchKernelGGL(colsum_fin_kernel, dim3((n + 63) / 64), dim3(1024), 0, s, part, (bf16_t*)out, colsum_parts(rows), n, acc, c);
  return check_launch("colsum_fin");
}

sif_status launch_fin_batch(const FinItem* items_dev, uint32_t n_items, uint32_t max_n, uint32_t acc, hipStream_t s, const KCtl& c) {
  REQ(items_dev && n_items > 0 && n_items <= 65535 && max_n > 0, "fin_batch: bad arguments");
  hipLaunchKernelGGL(fin_batch_kernel, dim3((max_n + 63) / 64, n_items), dim3(1024), 0, s, items_dev, acc, c);
  return check_launch("fin_batch");
}

sif_status launch_colsum_f32(const float* x, uint32_t ld, float* out, uint32_t rows, uint32_t n, hipStream_t s, const KCtl& c) {
  REQ(x && out && rows > 0 && n > 0 && ld >= n, "colsum_f32: bad arguments");
  hipLaunchKernelGGL(colsum_f32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, x, ld, out, rows, n, c);
  return check_launch("colsum_f32");
}

sif_status launch_softmax_fwd(const float* sc, void* p, uint32_t batch, uint32_t rows, uint32_t cols, uint32_t ld_s,
                              uint32_t ld_p, uint32_t causal, hipStream_t s, const KCtl& c) {
  REQ(sc && p && batch > 0 && rows > 0 && cols > 0, "softmax_fwd: null or empty");
  REQ(cols <= 256 * SM_MAXT && ld_p <= 256 * SM_MAXT, "softmax_fwd: at most 2048 columns");
  REQ((ld_s & 3) == 0 && (ld_p & 3) == 0 && ld_s >= ((cols + 3) & ~3u) && ld_p >= cols && al16(sc) && al16(p), "softmax_fwd: ld must be multiples of 4 and cover cols");
  REQ(batch <= 65535, "softmax_fwd: batch too large");
  hipLaunchKernelGGL(softmax_fwd_kernel, dim3((rows + 3) / 4, batch), dim3(256), 0, s, sc, (bf16_t*)p, rows, cols, ld_s, ld_p, causal, c);
  return check_launch("softmax_fwd");
}

sif_status launch_softmax_bwd(const float* dp, const void* p, void* ds, uint32_t batch, uint32_t rows, uint32_t cols,
                              uint32_t ld, float scale, uint32_t causal, hipStream_t s, const KCtl& c) {
  REQ(dp && p && ds && batch > 0 && rows > 0 && cols > 0, "softmax_bwd: null or empty");
  REQ(ld <= 256 * SM_MAXT && (ld & 3) == 0 && ld >= cols && al16(dp) && al16(p) && al16(ds), "softmax_bwd: ld must be a multiple of 4, cover cols, at most 2048");
  REQ(batch <= 65535, "softmax_bwd: batch too large");
  hipLaunchKernelGGL(softmax_bwd_kernel, dim3((rows + 3) / 4, batch), dim3(256), 0, s, dp, (const bf16_t*)p, (bf16_t*)ds, rows, cols, ld, scale, causal, c);
  return check_launch("softmax_bwd");
}

sif_status launch_embed_fwd(const int32_t* ids, const void* wte, const void* wpe, void* x, uint32_t vocab, uint32_t tokens,
                            uint32_t seq, uint32_t d, hipStream_t s, const KCtl& c) {
  REQ(ids && wte && wpe && x && tokens > 0 && seq > 0 && vocab > 0, "embed_fwd: null or empty");
  REQ((d & 7) == 0 && al16(wte) && al16(wpe) && al16(x), "embed_fwd: d must be a multiple of 8, pointers 16-byte aligned");
  hipLaunchKernelGGL(embed_fwd_kernel, dim3((tokens + 3) / 4), dim3(256), 0, s, ids, (const bf16_t*)wte, (const bf16_t*)wpe, (bf16_t*)x, tokens, seq, d, vocab, c);
  return check_launch("embed_fwd");
}

sif_status launch_embed_fwd_segs(const RowSegs& segs, const void* wte, const void* wpe, void* x, uint32_t vocab, uint32_t d, hipStream_t s, const KCtl& c) {
  REQ(wte && wpe && x && segs.n > 0 && segs.n <= kMaxRowSegs && vocab > 0, "embed_fwd: null or empty");
  REQ((d & 7) == 0 && al16(wte) && al16(wpe) && al16(x), "embed_fwd: d must be a multiple of 8, pointers 16-byte aligned");
  const uint32_t tokens = segs.row0[segs.n];
  if (sif_status st = check_segs("embed_fwd", segs, tokens)) return st;
  for (uint32_t r = 0; r < segs.n; ++r) REQ(segs.seq[r] > 0, "embed_fwd: empty sequence");
  hipLaunchKernelGGL(embed_fwd_segs_kernel, dim3((tokens + 3) / 4), dim3(256), 0, s, segs, (const bf16_t*)wte, (const bf16_t*)wpe, (bf16_t*)x, tokens, d, vocab, c);
  return check_launch("embed_fwd");
}

sif_status launch_embed_bwd_wte(const int32_t* ids, const void* dx, void* dwte, uint32_t vocab, uint32_t tokens, uint32_t d, hipStream_t s, const KCtl& c) {
  REQ(ids && dx && dwte && tokens > 0 && vocab > 0, "embed_bwd: null or empty");
  REQ(d <= 256 * EB_MAXC, "embed_bwd: d must be <= 4096");
  if (tokens <= EB_LDS_TOKENS && (d & 7) == 0 && al16(dx) && al16(dwte))
    hipLaunchKernelGGL(embed_bwd_wte_lds_kernel, dim3((tokens + EB_OWN - 1) / EB_OWN), dim3(256), 0, s, ids, (const bf16_t*)dx, (bf16_t*)dwte, tokens, d, vocab, c);
  else
    hipLaunchKernelGGL(embed_bwd_wte_kernel, dim3(tokens), dim3(256), 0, s, ids, (const bf16_t*)dx, (bf16_t*)dwte, tokens, d, vocab, c);
  return check_launch("embed_bwd_wte");
}

sif_status launch_embed_bwd_wpe(const void* dx, void* dwpe, uint32_t tokens, uint32_t seq, uint32_t d, hipStream_t s, const KCtl& c) {
  REQ(dx && dwpe && tokens > 0 && seq > 0 && seq <= tokens, "embed_bwd_wpe: bad arguments");
  hipLaunchKernelGGL(embed_bwd_wpe_kernel, dim3(seq), dim3(256), 0, s, (const bf16_t*)dx, (bf16_t*)dwpe, tokens, seq, d, c);
  return check_launch("embed_bwd_wpe");
}

sif_status launch_xent(void* logits, const int32_t* targets, float* loss, uint32_t tokens, uint32_t vocab, uint32_t ld,
                       hipStream_t s, const KCtl& c) {
  REQ(logits && targets && loss && tokens > 0 && vocab > 0, "xent: null or empty");
  REQ((ld & 7) == 0 && ld >= vocab && al16(logits), "xent: ld must be a multiple of 8 and >= vocab");
  if (ld <= 8 * 512 * 13) {          // the row fits in the registers of a block of 512 threads
    // (344 us for 8192 x 50257 with one row per block, two blocks per CU; 328 us as one block per CU with two rows in flight)
    hipLaunchKernelGGL((xent_stream_kernel<13, 512>), dim3(std::min<uint32_t>(tokens, n_cus())), dim3(512), 0, s, (bf16_t*)logits, targets, loss, tokens, vocab, ld, c);
    return check_launch("xent");
  }
  if (ld <= 8 * 1024 * 8) {          // up to 65536 columns: 1024 threads, one block per CU
    hipLaunchKernelGGL((xent_reg_kernel<8, 1024>), dim3(tokens), dim3(1024), 0, s, (bf16_t*)logits, targets, loss, tokens, vocab, ld, c);
    return check_launch("xent");
  }
  const size_t lds = (size_t)ld * sizeof(bf16_t);
  REQ(lds <= 144 * 1024, "xent: row does not fit in LDS (vocab <= 73728)");
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(xent_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024);
    if (e != hipSuccess) return fail_hip(e, "xent: hipFuncSetAttribute");
    attr_set = true;
  }
  hipLaunchKernelGGL(xent_kernel, dim3(tokens), dim3(1024), lds, s, (bf16_t*)logits, targets, loss, tokens, vocab, ld, c);
  return check_launch("xent");
}

sif_status launch_reduce_sum(const float* x, float* out, uint32_t n, float scale, hipStream_t s, const KCtl& c) {
  REQ(x && out && n > 0, "reduce_sum: null or empty");
  hipLaunchKernelGGL(reduce_sum_kernel, dim3(1), dim3(1024), 0, s, x, out, n, scale, c);
  return check_launch("reduce_sum");
}

static uint32_t grid_for(uint64_t work_items) {
  uint64_t b = (work_items + 255) / 256;
  return (uint32_t)(b < 1 ? 1 : (b > 4096 ? 4096 : b));
}

sif_status launch_sgd_bf16(float* master, const void* grad, void* work, uint64_t n, float lr, hipStream_t s, const KCtl& c) {
  REQ(master && work && n > 0 && (grad || lr == 0.f), "sgd_bf16: null or empty");
  REQ(al16(master) && al16(work) && (grad == nullptr || al16(grad)), "sgd_bf16: pointers must be 16-byte aligned");
  hipLaunchKernelGGL(sgd_bf16_kernel, dim3(grid_for(n >> 3)), dim3(256), 0, s, master, (const bf16_t*)grad, (bf16_t*)work, n, lr, c);
  return check_launch("sgd_bf16");
}

sif_status launch_sgd_f32(float* p, const float* g, uint64_t n, float lr, hipStream_t s, const KCtl& c) {
  REQ(p && g && n > 0, "sgd_f32: null or empty");
  hipLaunchKernelGGL(sgd_f32_kernel, dim3(grid_for(n)), dim3(256), 0, s, p, g, n, lr, c);
  return check_launch("sgd_f32");
}

sif_status launch_mse(const float* y, const float* t, float* d, float* loss, uint32_t n, hipStream_t s, const KCtl& c) {
  REQ(y && t && d && n > 0, "mse: null or empty");
  hipLaunchKernelGGL(mse_kernel, dim3(1), dim3(1024), 0, s, y, t, d, loss, n, c);
  return check_launch("mse");
}

sif_status launch_copy(void* dst, const void* src, uint64_t bytes, hipStream_t s, const KCtl& c) {
  REQ(dst && src && bytes > 0 && (bytes & 15) == 0 && al16(dst) && al16(src), "copy: needs 16-byte aligned buffers and size");
  hipLaunchKernelGGL(copy_kernel, dim3(grid_for(bytes >> 4)), dim3(256), 0, s, (uint4*)dst, (const uint4*)src, bytes >> 4, c);
  return check_launch("copy");
}

sif_status launch_reduce_splits_batch(const RedItem* items_dev, uint32_t n_items, uint32_t acc, hipStream_t s, const KCtl& c) {
  REQ(items_dev && n_items > 0 && n_items <= 65535, "reduce_splits_batch: bad arguments");
  // about 2048 blocks in all (eight per CU), at least 128 per item: a launch with a single item (the LM head's data
  // gradient) must still cover the chip
  const uint32_t bx = std::max<uint32_t>(128u, (2048u + n_items - 1) / n_items);
  hipLaunchKernelGGL(reduce_splits_batch_kernel, dim3(bx, n_items), dim3(256), 0, s, items_dev, acc, c);
  return check_launch("reduce_splits_batch");
}

sif_status launch_fill_u32(uint32_t* p, uint32_t v, uint64_t n, hipStream_t s, const KCtl& c) {
  REQ(p && n > 0, "fill: null or empty");
  hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for(n)), dim3(256), 0, s, p, v, n, c);
  return check_launch("fill");
}

}  // namespace sif
