// bf16 matrix product on the gfx950 MFMA units, fp32 accumulation, fused epilogues.
//
//   C[M,N] = alpha * sum_k A(m,k) B(k,n)   (+ bias, GELU, residual, GELU' multiply)
//
// One kernel serves every dense contraction of the training step and of the inference forward pass (the
// "kernels issued by the training instance" and the inference kernels the Kernel Barrier releases, Sec. 3.1):
// forward products (A [M][K], B [N][K]), data gradients (B [K][N]), weight gradients (A [K][M], B [K][N]) and
// the per-head attention products via two batch strides.
//
// Tiling: 128x128 block tile, K step 64, 256 threads = 4 wavefronts in a 2x2 grid, each wavefront owns a 64x64
// tile as 2x2 v_mfma_f32_32x32x16_bf16 accumulators.  Operand tiles are staged through LDS with K contiguous
// (row stride 72 elements so that 16-byte reads of consecutive rows spread over the banks); an operand whose
// memory layout has the other dimension contiguous is transposed while it is written to LDS.  Global loads of
// the next K step are issued before the MFMAs of the current one (register prefetch, two LDS buffers).
//
// Results do not depend on the grid: each output element is reduced over K in one fixed order by one
// wavefront, so launching a row range of the same problem gives bit-identical rows.
#include "common.h"
#include "specinf.h"
#include "launch.h"

namespace sif {

constexpr int BM = 128, BN = 128, BK = 64, LDS_LD = BK + 8;
constexpr int GEMM_THREADS = 256;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct GemmP {
  const bf16_t* a; const bf16_t* b; void* c; const bf16_t* bias; const void* res; bf16_t* aux;
  uint32_t m, n, k, lda, ldb, ldc, epi, k_causal, batch_inner;
  long long a_so, a_si, b_so, b_si, c_so, c_si;
  float alpha;
};

// Loads one 128 x 64 operand tile into registers (4 x 16 bytes per thread).  LAYOUT 0: memory [row][k];
// LAYOUT 1: memory [k][row].  Vectors outside the logical extents read as zero.
template <int LAYOUT>
__device__ __forceinline__ void load_tile(uint4 (&r)[4], const bf16_t* __restrict__ base, uint32_t ld, uint32_t row0,
                                          uint32_t rows, uint32_t k0, uint32_t k_end) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t v = threadIdx.x + i * GEMM_THREADS;
    uint32_t rr, kk;
    if (LAYOUT == 0) { rr = row0 + (v >> 3); kk = k0 + (v & 7) * 8; }
    else { kk = k0 + (v >> 4); rr = row0 + (v & 15) * 8; }
    bool ok = rr < rows && kk < k_end;
    const bf16_t* p = LAYOUT == 0 ? base + (size_t)rr * ld + kk : base + (size_t)kk * ld + rr;
    r[i] = ok ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
  }
}

template <int LAYOUT>
__device__ __forceinline__ void store_tile(bf16_t* lds, const uint4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t v = threadIdx.x + i * GEMM_THREADS;
    if (LAYOUT == 0) {
      uint32_t rr = v >> 3, kk = (v & 7) * 8;
      *reinterpret_cast<uint4*>(lds + rr * LDS_LD + kk) = r[i];
    } else {
      uint32_t kk = v >> 4, rr = (v & 15) * 8;
      uint32_t w[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        lds[(rr + 2 * j) * LDS_LD + kk] = (bf16_t)(w[j] & 0xFFFFu);
        lds[(rr + 2 * j + 1) * LDS_LD + kk] = (bf16_t)(w[j] >> 16);
      }
    }
  }
}

template <int ALAY, int BLAY>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(GemmP p, KCtl ctl) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);            // [2][BM][LDS_LD]
  bf16_t* sB = sA + 2 * BM * LDS_LD;                           // [2][BN][LDS_LD]
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }

  const uint32_t m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const bool skip = (p.epi & SIF_EPI_CAUSAL_SKIP) && n0 > m0 + BM - 1;
  if (!skip) {
    const uint32_t bo = blockIdx.z / p.batch_inner, bi = blockIdx.z % p.batch_inner;
    const bf16_t* A = p.a + bo * p.a_so + bi * p.a_si;
    const bf16_t* B = p.b + bo * p.b_so + bi * p.b_si;
    uint32_t k_begin = 0, k_end = p.k;
    if (p.k_causal == 1) k_end = min(p.k, m0 + BM);
    if (p.k_causal == 2) k_begin = (m0 / BK) * BK;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 ra[4], rb[4];
    load_tile<ALAY>(ra, A, p.lda, m0, p.m, k_begin, k_end);
    load_tile<BLAY>(rb, B, p.ldb, n0, p.n, k_begin, k_end);
    store_tile<ALAY>(sA, ra);
    store_tile<BLAY>(sB, rb);
    __syncthreads();

    int buf = 0;
    for (uint32_t k0 = k_begin; k0 < k_end; k0 += BK) {
      const bool more = k0 + BK < k_end;
      if (more) {
        load_tile<ALAY>(ra, A, p.lda, m0, p.m, k0 + BK, k_end);
        load_tile<BLAY>(rb, B, p.ldb, n0, p.n, k0 + BK, k_end);
      }
      const bf16_t* cA = sA + buf * BM * LDS_LD + (wm * 64 + (lane & 31)) * LDS_LD + (lane >> 5) * 8;
      const bf16_t* cB = sB + buf * BN * LDS_LD + (wn * 64 + (lane & 31)) * LDS_LD + (lane >> 5) * 8;
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8 fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          fa[i] = *reinterpret_cast<const bf16x8*>(cA + i * 32 * LDS_LD + ks * 16);
          fb[i] = *reinterpret_cast<const bf16x8*>(cB + i * 32 * LDS_LD + ks * 16);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
      if (more) {
        store_tile<ALAY>(sA + (buf ^ 1) * BM * LDS_LD, ra);
        store_tile<BLAY>(sB + (buf ^ 1) * BN * LDS_LD, rb);
      }
      __syncthreads();
      buf ^= 1;
    }

    // Epilogue.  Accumulator element r of lane l is row (r/4)*8 + (l/32)*4 + r%4, column l%32 of its 32x32 tile.
    const uint32_t epi = p.epi;
    const size_t c_off = (size_t)(bo * p.c_so + bi * p.c_si);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t n = n0 + wn * 64 + j * 32 + (lane & 31);
      if (n >= p.n) continue;
      const float bias = (p.bias != nullptr) ? bf2f(p.bias[n]) : 0.f;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const uint32_t m = m0 + wm * 64 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
          if (m >= p.m) continue;
          const size_t idx = c_off + (size_t)m * p.ldc + n;
          float v = acc[i][j][r] * p.alpha + bias;
          if (epi & SIF_EPI_GELU) {
            if (p.aux != nullptr) p.aux[idx] = f2bf(v);
            v = gelu_f(v);
          }
          if (epi & SIF_EPI_GELU_GRAD) v *= gelu_grad_f(bf2f(p.aux[idx]));
          if (epi & SIF_EPI_OUT_F32) {
            if (epi & SIF_EPI_RESIDUAL) v += reinterpret_cast<const float*>(p.res)[idx];
            reinterpret_cast<float*>(p.c)[idx] = v;
          } else {
            if (epi & SIF_EPI_RESIDUAL) v += bf2f(reinterpret_cast<const bf16_t*>(p.res)[idx]);
            reinterpret_cast<bf16_t*>(p.c)[idx] = f2bf(v);
          }
        }
      }
    }
  }
  kernel_end(ctl, true);
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

sif_status launch_gemm_bf16(const sif_gemm_args* a, hipStream_t stream, const KCtl& ctl) {
  if (a == nullptr || a->struct_size != sizeof(sif_gemm_args)) return fail(SIF_E_INVAL, "gemm: bad args struct");
  if (a->m == 0 || a->n == 0 || a->k == 0) return fail(SIF_E_INVAL, "gemm: empty extent");
  if (a->a_layout > 1 || a->b_layout > 1) return fail(SIF_E_INVAL, "gemm: bad layout");
  if (!a->a_dev || !a->b_dev || !a->c_dev) return fail(SIF_E_INVAL, "gemm: null operand");
  if (!aligned16(a->a_dev) || !aligned16(a->b_dev) || !aligned16(a->c_dev)) return fail(SIF_E_INVAL, "gemm: operands must be 16-byte aligned");
  if ((a->lda & 7) || (a->ldb & 7)) return fail(SIF_E_INVAL, "gemm: lda/ldb must be multiples of 8");
  if ((a->a_stride_outer | a->a_stride_inner | a->b_stride_outer | a->b_stride_inner) & 7) return fail(SIF_E_INVAL, "gemm: batch strides must be multiples of 8");
  const uint32_t a_contig = a->a_layout == SIF_A_ROW_K ? a->k : a->m;
  const uint32_t b_contig = a->b_layout == SIF_B_ROW_K ? a->k : a->n;
  if (a->lda < ((a_contig + 7) & ~7u) || a->ldb < ((b_contig + 7) & ~7u) || a->ldc < a->n) return fail(SIF_E_INVAL, "gemm: leading dimension too small");
  if (a->batch_outer == 0 || a->batch_inner == 0) return fail(SIF_E_INVAL, "gemm: batch counts must be >= 1");
  if ((a->epilogue & SIF_EPI_GELU_GRAD) && !a->aux_dev) return fail(SIF_E_INVAL, "gemm: GELU_GRAD needs aux");
  if ((a->epilogue & SIF_EPI_RESIDUAL) && !a->res_dev) return fail(SIF_E_INVAL, "gemm: RESIDUAL needs res");
  if ((a->epilogue & (SIF_EPI_BIAS | SIF_EPI_GELU)) == SIF_EPI_BIAS && !a->bias_dev) return fail(SIF_E_INVAL, "gemm: BIAS needs bias");
  if (a->k_causal > 2) return fail(SIF_E_INVAL, "gemm: bad k_causal");
  GemmP p;
  p.a = (const bf16_t*)a->a_dev; p.b = (const bf16_t*)a->b_dev; p.c = a->c_dev;
  p.bias = (a->epilogue & (SIF_EPI_BIAS | SIF_EPI_GELU)) ? (const bf16_t*)a->bias_dev : nullptr;
  p.res = a->res_dev; p.aux = (bf16_t*)a->aux_dev;
  p.m = a->m; p.n = a->n; p.k = a->k; p.lda = a->lda; p.ldb = a->ldb; p.ldc = a->ldc;
  p.epi = a->epilogue; p.k_causal = a->k_causal; p.batch_inner = a->batch_inner;
  p.a_so = a->a_stride_outer; p.a_si = a->a_stride_inner; p.b_so = a->b_stride_outer; p.b_si = a->b_stride_inner;
  p.c_so = a->c_stride_outer; p.c_si = a->c_stride_inner; p.alpha = a->alpha;
  dim3 grid((a->n + BN - 1) / BN, (a->m + BM - 1) / BM, a->batch_outer * a->batch_inner);
  if (grid.y > 65535 || grid.z > 65535) return fail(SIF_E_INVAL, "gemm: grid too large");
  const size_t lds = (size_t)2 * (BM + BN) * LDS_LD * sizeof(bf16_t);
  typedef void (*kern_t)(GemmP, KCtl);
  static const kern_t table[2][2] = {{gemm_bf16_kernel<0, 0>, gemm_bf16_kernel<0, 1>},
                                     {gemm_bf16_kernel<1, 0>, gemm_bf16_kernel<1, 1>}};
  kern_t kern = table[a->a_layout][a->b_layout];
  static bool attr_set[2][2] = {{false, false}, {false, false}};
  if (!attr_set[a->a_layout][a->b_layout]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return fail_hip(e, "gemm: hipFuncSetAttribute");
    attr_set[a->a_layout][a->b_layout] = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(GEMM_THREADS), lds, stream, p, ctl);
  return check_launch("gemm_bf16");
}

}  // namespace sif
