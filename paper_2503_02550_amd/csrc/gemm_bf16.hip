// bf16 matrix product on the gfx950 MFMA units, fp32 accumulation, fused epilogues.
//
//   C[M,N] = alpha * sum_k A(m,k) B(k,n)   (+ bias, GELU, residual, GELU' multiply)
//
// One kernel serves every dense contraction of the training step and of the inference forward pass (the
// "kernels issued by the training instance" and the inference kernels the Kernel Barrier releases, Sec. 3.1):
// forward products (A [M][K], B [N][K]), data gradients (B [K][N]), weight gradients (A [K][M], B [K][N]) and
// the per-head attention products via two batch strides.
//
// Tiling: block tile BM x BN, K step 64, WM x WN wavefronts, each owning a (BM/WM) x (BN/WN) tile as a grid of
// v_mfma_f32_32x32x16_bf16 accumulators.  128x128 with 2x2 wavefronts (64x64 each), two blocks per CU, is the
// working configuration; 256x256 with 2x4 wavefronts (128x64 each: six operand reads from LDS per eight MFMAs
// instead of eight, half the global fetches per MFMA), one block per CU, takes over where a fitted timing model
// says so (many tiles in whole rounds, or a long K).  Operand tiles are staged through LDS with K contiguous (unpadded rows of 128 bytes, XOR-swizzled
// in 16-byte chunks so that reads and writes spread over the banks); an operand whose memory layout has the other
// dimension contiguous is staged as it lies and transposed by the LDS read itself (ds_read_b64_tr_b16).  Interior
// tiles are fetched from global memory straight into LDS, tile t+1 while tile t is multiplied; tiles on a ragged
// edge of the 128x128 configuration go through registers (two K steps of prefetch) so that they can be zero-filled.
//
// What the main loop waits for is neither the MFMA units nor LDS but the operand fetches: a CU sustains about 28 bytes
// per cycle of loads that miss its L1 (measured; whatever their destination), a 256x256 tile needs 31 bytes per cycle
// at full MFMA rate and a 128x128 tile twice that.  Hence the large tile wherever it fills the chip, fetches that hand
// over 32-bit offsets (buffer loads), and result stores that do not claim L2 lines the operand panels are reused from.
//
// Results depend neither on the grid nor on the tile configuration: each output element is reduced over K in one
// fixed order (ascending, 16 at a time) by one wavefront, so launching a row range of the same problem, or the other
// configuration, gives bit-identical values.
#include <algorithm>

#include "common.h"
#include "specinf.h"
#include "launch.h"

namespace sif {

constexpr int BK = 64;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes of a result, stored with the non-temporal hint.  A product's output is written once and read by a later
// kernel, and the chip's CUs write their tiles in bursts that exceed what the L2 takes in at once: stores that do not
// claim L2 lines are acknowledged sooner (the wavefront waits for them at its next wait for a fetch), and they leave
// the operand panels, which the tiles of an XCD share, in the L2.
__device__ __forceinline__ void store_result16(void* p, const uint4& v) {
  const u32x4 x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, reinterpret_cast<u32x4*>(p));
}
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct GemmP {
  const bf16_t* a; const bf16_t* b; void* c; const bf16_t* bias; const void* res; bf16_t* aux;
  uint32_t m, n, k, lda, ldb, ldc, epi, k_causal, batch_inner, tiles_m, tiles_n, k_limit;
  long long a_so, a_si, b_so, b_si, c_so, c_si;
  float alpha;
  // a launch over several products at once (128x128 tiles, no batch): `group` points to their records in device memory,
  // each with the number of the launch's first block that works on it (a multiple of 8)
  const GemmP* group;
  uint32_t group_n, tile_base;
};

// LDS tile: rows x 64 k (bf16), 128 bytes per row = eight 16-byte chunks, no padding.  Chunk c of row r
// lives at chunk position c ^ key(r).  The key makes eight consecutive rows use eight different chunk positions
// (conflict-free 16-byte reads with 32 banks) and sixteen consecutive rows sixteen different (row parity, position)
// pairs (conflict-free with 64 banks) for the same logical chunk, which is how the MFMA operands are read.
__device__ __forceinline__ uint32_t swz_key(uint32_t row) { return (row & 7u) ^ ((row >> 3) & 1u); }
__device__ __forceinline__ uint32_t lds_off(uint32_t row, uint32_t chunk) { return row * BK + ((chunk ^ swz_key(row)) << 3); }

// A K-major operand (memory [k][row]) is staged as it lies in memory: LDS tile [64 k][ROWS], 2*ROWS bytes per k,
// the 64-byte segments (32 rows) of k-row k stored at segment position seg ^ (k % 4).  The MFMA operand - eight
// consecutive k for one row per lane - is then fetched with the transposing LDS read of gfx950
// (ds_read_b64_tr_b16): within each group of 16 lanes, source lane s supplies the address of four consecutive rows
// at k = k0 + s/4, rows r0 + 4*(s%4).., and lane i receives rows r0 + i at k0..k0+3.  Two such reads make one
// operand; the four k-rows a half-wavefront touches lie in four different 64-byte bank groups.
typedef short short4_lds __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint32_t kmajor_off(uint32_t k, uint32_t row, uint32_t rows_pitch) {
  return k * rows_pitch + ((((row >> 5) ^ (k & 3u)) << 5) | (row & 31u));
}
template <int ROWS>
__device__ __forceinline__ bf16x8 kmajor_frag(const bf16_t* tile, uint32_t rowbase32, uint32_t kbase8) {
  // rowbase32: first of the 32 operand rows (a multiple of 32); kbase8: first of this lane half's eight k
  const uint32_t lane = threadIdx.x & 63, s = lane & 15, sw = s >> 2;
  const bf16_t* p = tile + (kbase8 + sw) * ROWS + ((((rowbase32 >> 5) ^ sw) << 5) | (((lane >> 4) & 1u) * 16 + 4 * (s & 3u)));
  typedef __attribute__((address_space(3))) short4_lds* lds_ptr;
  const short4_lds lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p);
  const short4_lds hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * ROWS));
  typedef short short8_v __attribute__((ext_vector_type(8)));
  const short8_v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// How the threads of a block cover one operand tile (ROWS rows x 64 k), four 16-byte vectors each
// (vector v = thread + i * THREADS):
//   LAYOUT 0: memory [row][k]: row v/8, k chunk v%8.
//   LAYOUT 1: memory [k][row]: k-row v/(ROWS/8), row chunk v%(ROWS/8).
// Loads one operand tile into registers.  Vectors outside the logical extents read as zero.  The loads are
// unconditional (an out-of-range vector reads the operand's first element instead and is zeroed afterwards), so
// that they can be issued back to back and waited for selectively.
template <int LAYOUT, int THREADS, int ROWS>
__device__ __forceinline__ uint32_t load_tile(uint4 (&r)[4], const bf16_t* __restrict__ base, uint32_t ld, uint32_t row0,
                                              uint32_t rows, uint32_t k0, uint32_t k_end) {
  bool ok[4];
  const bf16_t* ptr[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t v = threadIdx.x + i * THREADS;
    if (LAYOUT == 0) {
      const uint32_t rr = row0 + (v >> 3), kk = k0 + (v & 7) * 8;
      ok[i] = rr < rows && kk < k_end;
      ptr[i] = ok[i] ? base + (size_t)rr * ld + kk : base;
    } else {
      const uint32_t rr = row0 + (v % (ROWS / 8)) * 8, kk = k0 + v / (ROWS / 8);
      ok[i] = rr < rows && kk < k_end;
      ptr[i] = ok[i] ? base + (size_t)kk * ld + rr : base;
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) r[i] = *reinterpret_cast<const uint4*>(ptr[i]);
  // bit i set = vector i is inside the operand; applied when the registers are written to LDS, not here, so that
  // nothing waits for the loads before their data is needed
  return (ok[0] ? 1u : 0u) | (ok[1] ? 2u : 0u) | (ok[2] ? 4u : 0u) | (ok[3] ? 8u : 0u);
}

template <int LAYOUT, int THREADS, int ROWS>
__device__ __forceinline__ void store_tile(bf16_t* lds, const uint4 (&rin)[4], uint32_t okmask) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t keep = (okmask >> i) & 1u ? 0xFFFFFFFFu : 0u;       // folds away for a constant all-ones mask
    const uint4 r = make_uint4(rin[i].x & keep, rin[i].y & keep, rin[i].z & keep, rin[i].w & keep);
    const uint32_t v = threadIdx.x + i * THREADS;
    if (LAYOUT == 0) *reinterpret_cast<uint4*>(lds + lds_off(v >> 3, v & 7)) = r;
    else *reinterpret_cast<uint4*>(lds + kmajor_off(v / (ROWS / 8), (v % (ROWS / 8)) * 8, ROWS)) = r;
  }
}

// Interior tiles go from global memory straight into LDS (buffer_load_dwordx4 ... lds: no staging registers, no LDS
// store instructions; the buffer form, whose lanes hand over a 32-bit offset instead of a 64-bit address, runs the
// products 2-5 % faster than global_load_lds_dwordx4).  One such instruction writes the 64 lanes' 16 bytes to consecutive LDS addresses, 1 KB per
// wavefront, so the lane's position in the tile is fixed and the swizzle is applied to what it fetches: lane l of
// wavefront w, instruction i covers
//   LAYOUT 0: tile row 32*i + 8*w + l/8, chunk position l%8 = logical chunk (l%8) ^ key(row)
//   LAYOUT 1: k-row 16*i + 4*w + l/16, 16-byte unit l%16 = segment position (l%16)/4 -> logical segment ^ (k%4)
// (with 256 threads; 512 threads cover twice the rows or k-rows per instruction).
typedef __attribute__((address_space(3))) void* lds_void_ptr;
template <int LAYOUT, int ROWS, int THREADS>
struct DmaStream {
  static constexpr int NV = ROWS * 8 / THREADS;       // 16-byte vectors per thread and tile
  const char* tile;
  size_t step;
  uint32_t voff[NV];
  // rows >= `rows` (a ragged last tile) fetch the tile's first row instead: what they produce is never stored
  __device__ __forceinline__ DmaStream(const bf16_t* b, uint32_t ld, uint32_t row0, uint32_t rows, uint32_t k_begin) {
    if (LAYOUT == 0) {
      tile = (const char*)(b + (size_t)row0 * ld + k_begin);
      step = BK * sizeof(bf16_t);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const uint32_t r = i * (THREADS / 8) + (threadIdx.x >> 3), c = (threadIdx.x & 7u) ^ swz_key(r);
        voff[i] = ((row0 + r < rows ? r : 0u) * ld + c * 8) * (uint32_t)sizeof(bf16_t);
      }
    } else {
      constexpr uint32_t UR = ROWS / 8;          // 16-byte units per k-row
      tile = (const char*)(b + (size_t)k_begin * ld + row0);
      step = (size_t)BK * ld * sizeof(bf16_t);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const uint32_t k = i * (THREADS / UR) + threadIdx.x / UR, u = threadIdx.x % UR, seg = (u >> 2) ^ (k & 3u);
        const uint32_t r = seg * 32 + (u & 3u) * 8;
        voff[i] = (k * ld + (row0 + r < rows ? r : 0u)) * (uint32_t)sizeof(bf16_t);
      }
    }
  }
  // fetches the next tile into `stage` (a whole tile buffer of ROWS x 64 elements)
  __device__ __forceinline__ void next(bf16_t* stage) {
    // the LDS address of a fetch is taken from a scalar register: say that the wavefront number is uniform
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // a buffer resource over the tile's memory (raw bytes, no stride; the extent is left open: every offset below was
    // formed from a row and a k inside the operand) - only a 32-bit offset per lane then travels to the memory pipeline
#if defined(__HIP_DEVICE_COMPILE__)      // the resource type exists in the device pass only (with it in the host pass the
                                         // compiler drops, without a word, the host stubs of most instantiations)
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)tile, (short)0, -1, 0x00020000);
#pragma unroll
    for (int i = 0; i < NV; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(stage + i * (THREADS * 8) + wave * 512), 16, voff[i], 0, 0, 0);
#endif
    tile += step;
  }
};

// Epilogue of eight consecutive columns n..n+7 of row m (both inside the result): scale, bias, GELU, GELU' multiply,
// residual, store; `vec` says that every access may be a 16-byte vector, and then b holds the eight bias values,
// aux_q the eight auxiliary values (GELU_GRAD) and res_q the eight bf16 residual values.
__device__ __forceinline__ void gemm_epilogue8(const GemmP& p, size_t c_off, uint32_t m, uint32_t n, float (&v)[8], const float (&b)[8], bool vec,
                                               const uint4& aux_q, const uint4& res_q) {
  const uint32_t epi = p.epi;
  const size_t idx = c_off + (size_t)m * p.ldc + n;
  if (vec) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = v[e] * p.alpha + b[e];
    if (epi & SIF_EPI_GELU) {
      if (p.aux != nullptr)
        *reinterpret_cast<uint4*>(p.aux + idx) = make_uint4(pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]), pack_bf2(v[4], v[5]), pack_bf2(v[6], v[7]));
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = gelu_fast(v[e]);
    }
    if (epi & SIF_EPI_GELU_GRAD) {
      const uint4 q = aux_q;                  // fetched before the staging pass
      const float z[8] = {bflo(q.x), bfhi(q.x), bflo(q.y), bfhi(q.y), bflo(q.z), bfhi(q.z), bflo(q.w), bfhi(q.w)};
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_fast(z[e]);
    }
    if (epi & SIF_EPI_OUT_F32) {
      float* cp = reinterpret_cast<float*>(p.c) + idx;
      if (epi & SIF_EPI_RESIDUAL) {
        const float* rp = reinterpret_cast<const float*>(p.res) + idx;
        const float4 r0 = *reinterpret_cast<const float4*>(rp), r1 = *reinterpret_cast<const float4*>(rp + 4);
        v[0] += r0.x; v[1] += r0.y; v[2] += r0.z; v[3] += r0.w; v[4] += r1.x; v[5] += r1.y; v[6] += r1.z; v[7] += r1.w;
      }
      *reinterpret_cast<float4*>(cp) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4*>(cp + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
      if (epi & SIF_EPI_RESIDUAL) {
        const uint4 q = res_q;                // fetched before the staging pass
        v[0] += bflo(q.x); v[1] += bfhi(q.x); v[2] += bflo(q.y); v[3] += bfhi(q.y); v[4] += bflo(q.z); v[5] += bfhi(q.z); v[6] += bflo(q.w); v[7] += bfhi(q.w);
      }
      store_result16(reinterpret_cast<bf16_t*>(p.c) + idx, make_uint4(pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]), pack_bf2(v[4], v[5]), pack_bf2(v[6], v[7])));
    }
  } else {
    // ragged N (or an output slice that is not 16-byte aligned): one element at a time
    for (int e = 0; e < 8 && n + e < p.n; ++e) {
      float x = v[e] * p.alpha + (p.bias != nullptr ? bf2f(p.bias[n + e]) : 0.f);
      if (epi & SIF_EPI_GELU) {
        if (p.aux != nullptr) p.aux[idx + e] = f2bf(x);
        x = gelu_fast(x);
      }
      if (epi & SIF_EPI_GELU_GRAD) x *= gelu_grad_fast(bf2f(p.aux[idx + e]));
      if (epi & SIF_EPI_OUT_F32) {
        if (epi & SIF_EPI_RESIDUAL) x += reinterpret_cast<const float*>(p.res)[idx + e];
        reinterpret_cast<float*>(p.c)[idx + e] = x;
      } else {
        if (epi & SIF_EPI_RESIDUAL) x += bf2f(reinterpret_cast<const bf16_t*>(p.res)[idx + e]);
        reinterpret_cast<bf16_t*>(p.c)[idx + e] = f2bf(x);
      }
    }
  }
}

// Epilogue of one wavefront's (TI*32) x 64 part of an output tile, first row mw, first column nw.  The accumulators
// pass, 32 rows at a time, through a staging area `sW` of the wavefront's own in LDS (8 KB) so that every global
// access of the epilogue - bias, residual, auxiliary tensor, result - is a 16-byte vector along a row; no block-wide
// barrier is needed.  Accumulator element r of lane l is row (r/4)*8 + (l/32)*4 + r%4, column l%32 of its 32x32
// tile.  Chunk c (four floats) of staging row r lives at c ^ (8*((r/4)%2) | r%2): the two half-wavefronts of a
// store and the eight rows of a load then fall on different banks.  bias_q: the bias of columns nw + 8*(l%8)...
template <int TI, int TJ>
__device__ __forceinline__ void gemm_store_tile(const GemmP& p, floatx16 (&acc)[TI][TJ], float* sW, uint32_t mw, uint32_t nw, size_t c_off, const uint4& bias_q) {
  constexpr int WCOLS = TJ * 32;
  const uint32_t lane = threadIdx.x & 63;
  const bool vec_ok = (p.n & 7) == 0 && ((c_off & 7) == 0);
  const float bias8[8] = {bflo(bias_q.x), bfhi(bias_q.x), bflo(bias_q.y), bfhi(bias_q.y), bflo(bias_q.z), bfhi(bias_q.z), bflo(bias_q.w), bfhi(bias_q.w)};
  // Epilogues that read nothing but the bias (plain, bias, bias + GELU without the pre-activation output) are
  // finished in the accumulator layout, where a lane's column is fixed, and staged as bf16: two vertically adjacent
  // results share a 32-bit word, the staging area is [16 row pairs][64 columns] words, half the LDS traffic of the
  // fp32 staging below.  A lane then reads eight words = eight columns of two rows, separates the rows with byte
  // permutes and stores two 16-byte row vectors.  The arithmetic per element is the same as in gemm_epilogue8.
  const bool packed = vec_ok && (p.epi & (SIF_EPI_RESIDUAL | SIF_EPI_GELU_GRAD | SIF_EPI_OUT_F32)) == 0 &&
                      !((p.epi & SIF_EPI_GELU) && p.aux != nullptr);
  if (packed) {
    uint32_t* sP = reinterpret_cast<uint32_t*>(sW);
    float bcol[TJ];
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
      const uint32_t n = nw + j * 32 + (lane & 31);
      bcol[j] = (p.bias != nullptr && n < p.n) ? bf2f(p.bias[n]) : 0.f;
    }
    const uint32_t hh = lane >> 5;
#pragma unroll
    for (int i = 0; i < TI; ++i) {
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          float x0 = acc[i][j][r] * p.alpha + bcol[j], x1 = acc[i][j][r + 1] * p.alpha + bcol[j];
          if (p.epi & SIF_EPI_GELU) { x0 = gelu_fast(x0); x1 = gelu_fast(x1); }
          const uint32_t pr = (r >> 2) * 4 + hh * 2 + ((r & 3) >> 1), col = (j * 32 + (lane & 31)) ^ (hh << 5);
          sP[pr * WCOLS + col] = pack_bf2(x0, x1);
        }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const uint32_t item = lane + it * 64, pr = item >> 3, c8 = item & 7;     // 16 row pairs x 8 chunks of 8 columns
        const uint32_t pos = (c8 ^ (((pr >> 1) & 1u) << 2)) * 8;
        const uint4 w0 = *reinterpret_cast<const uint4*>(sP + pr * WCOLS + pos), w1 = *reinterpret_cast<const uint4*>(sP + pr * WCOLS + pos + 4);
        const uint4 even = make_uint4(__builtin_amdgcn_perm(w0.y, w0.x, 0x05040100), __builtin_amdgcn_perm(w0.w, w0.z, 0x05040100),
                                      __builtin_amdgcn_perm(w1.y, w1.x, 0x05040100), __builtin_amdgcn_perm(w1.w, w1.z, 0x05040100));
        const uint4 odd = make_uint4(__builtin_amdgcn_perm(w0.y, w0.x, 0x07060302), __builtin_amdgcn_perm(w0.w, w0.z, 0x07060302),
                                     __builtin_amdgcn_perm(w1.y, w1.x, 0x07060302), __builtin_amdgcn_perm(w1.w, w1.z, 0x07060302));
        const uint32_t m = mw + i * 32 + 2 * pr, n = nw + c8 * 8;
        bf16_t* cp = reinterpret_cast<bf16_t*>(p.c) + c_off + (size_t)m * p.ldc + n;
        if (n < p.n) {
          if (m < p.m) store_result16(cp, even);
          if (m + 1 < p.m) store_result16(cp + p.ldc, odd);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  } else
#pragma unroll
  for (int i = 0; i < TI; ++i) {
    // what the epilogue reads from global memory for this pass is requested before the staging, not inside it
    uint4 aux_q[WCOLS / 16], res_q[WCOLS / 16];
#pragma unroll
    for (int it = 0; it < WCOLS / 16; ++it) {
      const uint32_t ch = lane + it * 64, row = ch >> 3, c8 = ch & 7;
      const uint32_t m = mw + i * 32 + row, n = nw + c8 * 8;
      aux_q[it] = make_uint4(0, 0, 0, 0); res_q[it] = make_uint4(0, 0, 0, 0);
      if (vec_ok && m < p.m && n < p.n) {
        const size_t idx = c_off + (size_t)m * p.ldc + n;
        if (p.epi & SIF_EPI_GELU_GRAD) aux_q[it] = *reinterpret_cast<const uint4*>(p.aux + idx);
        if ((p.epi & (SIF_EPI_RESIDUAL | SIF_EPI_OUT_F32)) == SIF_EPI_RESIDUAL) res_q[it] = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(p.res) + idx);
      }
    }
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t row = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3), col = j * 32 + (lane & 31);
        sW[row * WCOLS + ((((col >> 2) ^ ((((row >> 2) & 1) << 3) | (row & 1))) << 2) | (col & 3))] = acc[i][j][r];
      }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < WCOLS / 16; ++it) {
      const uint32_t ch = lane + it * 64, row = ch >> 3, c8 = ch & 7;      // 32 rows x 8 chunks of 8 columns
      const uint32_t key = (((row >> 2) & 1) << 3) | (row & 1);
      const float4 q0 = *reinterpret_cast<const float4*>(sW + row * WCOLS + (((2 * c8) ^ key) << 2));
      const float4 q1 = *reinterpret_cast<const float4*>(sW + row * WCOLS + (((2 * c8 + 1) ^ key) << 2));
      float v[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
      const uint32_t m = mw + i * 32 + row, n = nw + c8 * 8;
      if (m < p.m && n < p.n) gemm_epilogue8(p, c_off, m, n, v, bias8, vec_ok, aux_q[it], res_q[it]);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

// Scheduling pipeline of one K step, from MFMA number G on (NS slices of NM MFMAs): after each MFMA its share of the
// next slice's ND LDS reads and of the step's FETCHES global -> LDS fetches.
template <int V> struct Int { static constexpr int value = V; };
template <int NM, int ND, int NS, int FETCHES, int G>
__device__ __forceinline__ void sched_pipeline() {
  if constexpr (G < NS * NM) {
    constexpr int ks = G / NM, m = G % NM;
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if constexpr (ks + 1 < NS) {
      constexpr int d0 = (m * ND) / NM, d1 = ((m + 1) * ND) / NM;
      if constexpr (d1 > d0) __builtin_amdgcn_sched_group_barrier(0x100, d1 - d0, 0);
    }
    constexpr int f0 = (G * FETCHES) / (NS * NM), f1 = ((G + 1) * FETCHES) / (NS * NM);
    if constexpr (f1 > f0) __builtin_amdgcn_sched_group_barrier(0x010, f1 - f0, 0);
    sched_pipeline<NM, ND, NS, FETCHES, G + 1>();
  }
}

// Block -> tile.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Every XCD
// gets a contiguous run of tiles (tile number pid belongs to XCD pid % 8 and is the (pid / 8)-th of its run), and each
// run is walked in bands of 8 tile rows, so that the tiles an XCD works on at one time share their A and B panels in
// that XCD's L2.
__device__ __forceinline__ void gemm_tile_of(const GemmP& p, uint32_t total_tiles, uint32_t pid, uint32_t& tm, uint32_t& tn) {
  const uint32_t per = (total_tiles + 7) / 8, tall = (total_tiles % 8) ? (total_tiles % 8) : 8, xcd = pid % 8, local = pid / 8;
  const uint32_t logical = xcd < tall ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
  const uint32_t width = 8 * p.tiles_n, group = logical / width, first = group * 8;
  const uint32_t gsz = min(p.tiles_m - first, 8u), in = logical % width;
  tm = first + in % gsz;
  tn = in / gsz;
}
__device__ __forceinline__ uint32_t gemm_tiles_of_xcd(uint32_t total_tiles, uint32_t x) { return x < total_tiles ? (total_tiles - x + 7u) / 8u : 0u; }
// One thread: takes a tile from the per-XCD counters of the stream's record, own XCD first: a tile number, else kNone.
__device__ __forceinline__ uint32_t gemm_steal_tile(StreamRec* rec, uint32_t total_tiles, uint32_t my_x) {
  for (uint32_t r = 0; r < 8; ++r) {
    const uint32_t x = (my_x + r) & 7u, cnt = gemm_tiles_of_xcd(total_tiles, x);
    uint32_t* ctr = &rec->tile_next[x * 32u];
    if (ld_relaxed(ctr) >= cnt) continue;
    const uint32_t l = atomicAdd(ctr, 1u);
    if (l < cnt) return l * 8u + x;
  }
  return kNone;
}

// Registers: two wavefronts per SIMD may take 256 of its 512 each, and the 256x256 configuration would.  It is held to
// 248 (the attribute counts in pairs): a one-wavefront kernel that sits on a CU for the length of a bubble (the
// training stream's wait) then still fits beside a block, which otherwise stays off that CU, and the tiles of 255 CUs
// end a round later (65536 x 768 x 768: 92 -> 153 us beside such a wavefront, 92 with the limit).
template <int ALAY, int BLAY, int BM, int BN, int WM, int WN, bool EDGE, bool GROUPED = false>
__global__ __launch_bounds__(64 * WM * WN, BM == 128 ? 2 : 1) __attribute__((amdgpu_num_vgpr(124))) void gemm_bf16_kernel(GemmP p_in, KCtl ctl) {
  static_assert(!GROUPED || EDGE, "several products in one launch: one block per tile");
  // (an instantiation of its own for launches over several products: in the others the product's record stays the
  // kernel argument, in scalar registers)
  GemmP p = p_in;
  constexpr int THREADS = 64 * WM * WN, TI = BM / (WM * 32), TJ = BN / (WN * 32), WCOLS = TJ * 32;
  static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "whole 16-byte vectors per thread and operand tile");
  static_assert(!EDGE || (BM * 8 == 4 * THREADS && BN * 8 == 4 * THREADS), "the register path moves four vectors per thread and operand");
  constexpr int FETCHES = (BM + BN) * 8 / THREADS;      // global -> LDS fetches per thread and K step
  static_assert(WCOLS == 64, "the epilogue staging is laid out for 64 columns per wavefront");
  // two tile buffers per operand, as four objects so that the compiler can tell a buffer being filled from the one being read
  __shared__ __align__(1024) bf16_t sA0[BM * BK];
  __shared__ __align__(1024) bf16_t sA1[BM * BK];
  __shared__ __align__(1024) bf16_t sB0[BN * BK];
  __shared__ __align__(1024) bf16_t sB1[BN * BK];
  if (!kernel_begin(ctl)) { kernel_end(ctl, false); return; }

  if constexpr (GROUPED) {                     // several products in one launch: which one is this block's
    uint32_t g = 0;
    while (g + 1 < p_in.group_n && blockIdx.x >= p_in.group[g + 1].tile_base) ++g;
    // the record is the same for every lane: word by word into scalar registers
    static_assert(sizeof(GemmP) % 4 == 0, "copied as 32-bit words");
    uint32_t words[sizeof(GemmP) / 4];
    const uint32_t* src = reinterpret_cast<const uint32_t*>(p_in.group + g);
#pragma unroll
    for (uint32_t w = 0; w < sizeof(GemmP) / 4; ++w) words[w] = __builtin_amdgcn_readfirstlane(src[w]);
    __builtin_memcpy(&p, words, sizeof(GemmP));
  }
  const uint32_t total_tiles = p.tiles_m * p.tiles_n;
  auto tile_of = [&](uint32_t pid, uint32_t& tm, uint32_t& tn) { gemm_tile_of(p, total_tiles, pid, tm, tn); };
  const uint32_t bo = blockIdx.z / p.batch_inner, bi = blockIdx.z % p.batch_inner;
  const bf16_t* A = p.a + bo * p.a_so + bi * p.a_si;
  const bf16_t* B = p.b + bo * p.b_so + bi * p.b_si;
  // The configuration without ragged tiles is launched with one block per CU that works through tiles one after the
  // other: wavefronts, LDS and the prologue are set up once, the first operand tiles of the next output tile are
  // fetched while the current one's epilogue runs, and the epilogue's stores drain under the next main loop.  The
  // other configuration is launched with one block per tile and passes through this loop once.
  // Which tile comes next: a monitored launch hands its tiles out through counters in the stream's record, one per
  // XCD (a block takes the tiles of its own XCD's run in order and, when that run is exhausted, helps the others), so
  // that a block that starts late - its CU was held by a kernel of the other stream - simply takes fewer tiles; with a
  // fixed share per block the whole launch would wait for the late one.  An unmonitored launch has no record: every
  // block takes each gridDim.x-th tile (a stride that is a multiple of 8 keeps it on its XCD's run).
  __shared__ uint32_t s_next;
  const bool dynamic = !EDGE && ctl.rec != nullptr && gridDim.z == 1 && gridDim.x < total_tiles;
  const uint32_t my_x = blockIdx.x & 7u;
  auto tiles_of_xcd = [&](uint32_t x) { return gemm_tiles_of_xcd(total_tiles, x); };
  auto steal = [&]() -> uint32_t { return gemm_steal_tile(ctl.rec, total_tiles, my_x); };
  uint32_t pid = blockIdx.x - p.tile_base;
  if (dynamic) {
    if (threadIdx.x == 0) s_next = steal();
    __syncthreads();
    pid = s_next;
  }
  DmaStream<ALAY, BM, THREADS> ta(A, p.lda, 0, p.m, 0);
  DmaStream<BLAY, BN, THREADS> tb(B, p.ldb, 0, p.n, 0);
  bool fetched_ahead = false;
  while (pid < total_tiles) {
  uint32_t next_pid = kNone;
  uint32_t tile_m, tile_n;
  tile_of(pid, tile_m, tile_n);
  const uint32_t m0 = tile_m * BM, n0 = tile_n * BN;
  const bool skip = (p.epi & SIF_EPI_CAUSAL_SKIP) && n0 > m0 + BM - 1;
  if (!skip) {
    uint32_t k_begin = 0, k_end = p.k;
    if (p.k_limit != 0) k_end = min(p.k, p.k_limit - bi * p.k);      // slices of one long K: the last may be shorter
    if (p.k_causal == 1) k_end = min(p.k, m0 + BM);
    if (p.k_causal == 2) k_begin = (m0 / BK) * BK;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WN, wn = wave % WN;
    floatx16 acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // A lane stores the same eight columns in every pass of the epilogue: their bias is fetched once, here, so that
    // the main loop hides the latency.
    uint4 bias_q = make_uint4(0, 0, 0, 0);
    {
      const uint32_t n = n0 + wn * WCOLS + (lane & 7) * 8;
      const size_t c_off0 = (size_t)(bo * p.c_so + bi * p.c_si);
      if ((p.n & 7) == 0 && (c_off0 & 7) == 0 && p.bias != nullptr && n < p.n) bias_q = *reinterpret_cast<const uint4*>(p.bias + n);
    }
    // Register prefetch two K steps deep: set[t & 1] carries tile t from global memory to LDS.  While tile t is
    // multiplied out of LDS buffer t & 1, tile t+1 is landing in the other set and the load of tile t+2 is issued
    // into the set tile t has just left, so every global load has two iterations of MFMA work to hide behind.
    uint4 ra0[4], rb0[4], ra1[4], rb1[4];
    const uint32_t fra = wm * (TI * 32) + (lane & 31), frb = wn * (TJ * 32) + (lane & 31), kh = lane >> 5;
    // Fragments of K slice ks + 1 are read from LDS into a second register set before the MFMAs of slice ks are
    // issued, so that an LDS read has four MFMAs (128 cycles) to land behind instead of being waited for at once.
    auto load_frags = [&](const bf16_t* cA, const bf16_t* cB, int ks, bf16x8 (&fa)[TI], bf16x8 (&fb)[TJ]) {
#pragma unroll
      for (int i = 0; i < TI; ++i)
        fa[i] = ALAY == 0 ? *reinterpret_cast<const bf16x8*>(cA + lds_off(fra + i * 32, ks * 2 + kh))
                          : kmajor_frag<BM>(cA, wm * (TI * 32) + i * 32, ks * 16 + kh * 8);
#pragma unroll
      for (int j = 0; j < TJ; ++j)
        fb[j] = BLAY == 0 ? *reinterpret_cast<const bf16x8*>(cB + lds_off(frb + j * 32, ks * 2 + kh))
                          : kmajor_frag<BN>(cB, wn * (TJ * 32) + j * 32, ks * 16 + kh * 8);
    };
    // `fetches` says how many global -> LDS fetches were issued just before (they sit in the same scheduling region).
    // The order wanted for one K step: the reads of slice 0, then per slice its MFMAs with the LDS reads of the next
    // slice and a share of the fetches spread evenly between them.  A wavefront issues in order, and a fetch that finds
    // the memory pipeline full holds up the MFMAs behind it, so the fetches must not come in one burst (after a barrier
    // every wavefront of the CU would issue its burst at the same time).
    auto compute = [&](const bf16_t* cA, const bf16_t* cB, auto fetches) {
      constexpr int NS = BK / 16, NM = TI * TJ, ND = (ALAY == 0 ? 1 : 2) * TI + (BLAY == 0 ? 1 : 2) * TJ;
      bf16x8 fa[2][TI], fb[2][TJ];
      load_frags(cA, cB, 0, fa[0], fb[0]);
#pragma unroll
      for (int ks = 0; ks < NS; ++ks) {
        if (ks + 1 < NS) load_frags(cA, cB, ks + 1, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
          for (int j = 0; j < TJ; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, ND, 0);                 // LDS reads of slice 0
      sched_pipeline<NM, ND, NS, decltype(fetches)::value, 0>();
    };
    // The loop takes two K steps per trip (the register sets and LDS buffers alternate by name) and has no exit in
    // its middle, so that the accumulators stay in the same registers throughout; an odd last tile is done after it.
    const uint32_t nt = (k_end - k_begin + BK - 1) / BK;
    uint32_t l_own = 0;
    // Whole K steps take the direct fetches, also in a tile that is ragged in M or N (its missing rows fetch the tile's
    // first row and are never stored); a ragged K needs the zero fill of the register path.  Without EDGE the launcher
    // guarantees whole K steps.
    const bool interior = !EDGE || ((k_end - k_begin) % BK) == 0;
    if (interior) {
      // tile t+1 is fetched into the other pair of buffers while tile t is multiplied; the other block of the CU
      // covers what the fetch latency exceeds one K step
      if (!fetched_ahead) {
        ta = DmaStream<ALAY, BM, THREADS>(A, p.lda, m0, p.m, k_begin);
        tb = DmaStream<BLAY, BN, THREADS>(B, p.ldb, n0, p.n, k_begin);
        ta.next(sA0); tb.next(sB0);
      }
      wait_fetches();
      __syncthreads();
      // the block's next tile is asked for now; the answer is looked at when this tile's main loop is over
      if (dynamic && threadIdx.x == 0) l_own = atomicAdd(&ctl.rec->tile_next[my_x * 32u], 1u);
      for (uint32_t t = 0; t + 2 <= nt; t += 2) {
        ta.next(sA1); tb.next(sB1);
        compute(sA0, sB0, Int<FETCHES>());
        wait_fetches();          // every wavefront's part of the next tile has landed before the barrier lets anyone read it
        __syncthreads();
        if (t + 2 < nt) { ta.next(sA0); tb.next(sB0); }
        compute(sA1, sB1, Int<FETCHES>());
        wait_fetches();
        __syncthreads();
      }
    } else if (EDGE) {
      uint32_t oka0 = load_tile<ALAY, THREADS, BM>(ra0, A, p.lda, m0, p.m, k_begin, k_end);
      uint32_t okb0 = load_tile<BLAY, THREADS, BN>(rb0, B, p.ldb, n0, p.n, k_begin, k_end);
      uint32_t oka1 = load_tile<ALAY, THREADS, BM>(ra1, A, p.lda, m0, p.m, k_begin + BK, k_end);       // reads as zero past k_end
      uint32_t okb1 = load_tile<BLAY, THREADS, BN>(rb1, B, p.ldb, n0, p.n, k_begin + BK, k_end);
      store_tile<ALAY, THREADS, BM>(sA0, ra0, oka0);
      store_tile<BLAY, THREADS, BN>(sB0, rb0, okb0);
      __syncthreads();
      for (uint32_t t = 0; t + 2 <= nt; t += 2) {
        const uint32_t k0 = k_begin + t * BK;
        oka0 = load_tile<ALAY, THREADS, BM>(ra0, A, p.lda, m0, p.m, k0 + 2 * BK, k_end);
        okb0 = load_tile<BLAY, THREADS, BN>(rb0, B, p.ldb, n0, p.n, k0 + 2 * BK, k_end);
        compute(sA0, sB0, Int<0>());
        store_tile<ALAY, THREADS, BM>(sA1, ra1, oka1);
        store_tile<BLAY, THREADS, BN>(sB1, rb1, okb1);
        __syncthreads();
        oka1 = load_tile<ALAY, THREADS, BM>(ra1, A, p.lda, m0, p.m, k0 + 3 * BK, k_end);
        okb1 = load_tile<BLAY, THREADS, BN>(rb1, B, p.ldb, n0, p.n, k0 + 3 * BK, k_end);
        compute(sA1, sB1, Int<0>());
        store_tile<ALAY, THREADS, BM>(sA0, ra0, oka0);
        store_tile<BLAY, THREADS, BN>(sB0, rb0, okb0);
        __syncthreads();
      }
    }
    if (nt & 1u) compute(sA0, sB0, Int<0>());

    // Epilogue.  Each wavefront passes its accumulators, 32 rows at a time, through a staging area of its own in
    // LDS (fp32 [32][64], the operand buffers are free by now) so that every global access of the epilogue - bias,
    // residual, auxiliary tensor, result - is a 16-byte vector along a row; no block-wide barrier is needed after
    // the first.  Accumulator element r of lane l is row (r/4)*8 + (l/32)*4 + r%4, column l%32 of its 32x32 tile.
    // Chunk c (four floats) of staging row r lives at c ^ (8*((r/4)%2) | r%2): the two half-wavefronts of a store
    // and the eight rows of a load then fall on different banks.
    if (!EDGE && threadIdx.x == 0) {
      uint32_t np = kNone;
      if (dynamic) np = l_own < tiles_of_xcd(my_x) ? l_own * 8u + my_x : steal();
      else if (pid + gridDim.x < total_tiles) np = pid + gridDim.x;
      s_next = np;
    }
    __syncthreads();
    // the block's next output tile: its first operand tiles travel into sA0 / sB0 while this epilogue runs (the staging
    // area below is sA1 / sB1, which the next main loop fills only after its first barrier)
    fetched_ahead = false;
    if (!EDGE) next_pid = s_next;
    if (!EDGE && next_pid < total_tiles) {
      uint32_t nm, nn;
      tile_of(next_pid, nm, nn);
      ta = DmaStream<ALAY, BM, THREADS>(A, p.lda, nm * BM, p.m, 0);
      tb = DmaStream<BLAY, BN, THREADS>(B, p.ldb, nn * BN, p.n, 0);
      ta.next(sA0); tb.next(sB0);
      fetched_ahead = true;
    }
    float* sW = reinterpret_cast<float*>(wave < WM * WN / 2 ? sA1 : sB1) + (wave % (WM * WN / 2)) * (32 * WCOLS);
    gemm_store_tile<TI, TJ>(p, acc, sW, m0 + wm * (TI * 32), n0 + wn * WCOLS, (size_t)(bo * p.c_so + bi * p.c_si), bias_q);
  }
  pid = next_pid;
  }
  kernel_end(ctl, true);
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// 256x256 tiles (one block of eight wavefronts per CU, 128x64 per wavefront: a quarter fewer LDS reads and half the
// global fetches per MFMA); they need whole K steps - also in the last, shorter slice of a K cut into slices - and no
// causal skipping
bool gemm_can_use_big_tiles(const sif_gemm_args& a) {
  const bool causal = a.k_causal != 0 || (a.epilogue & SIF_EPI_CAUSAL_SKIP);
  if (causal || (a.k % BK) != 0) return false;
  if (a.k_limit == 0) return true;
  const uint64_t before_last = (uint64_t)(a.batch_inner - 1) * a.k;
  return a.k_limit > before_last && ((a.k_limit - before_last) % BK) == 0;
}

// Which configuration is faster follows a two-line model fitted to measurements on gfx950 (time of one round of
// tiles over the chip, us, K in steps of 64): 128x128, two blocks per CU: 1.0 + 1.19 steps, and a CU that holds a
// single block runs it faster, so a partly filled round costs about its share (never less than 0.85 of a round);
// 256x256, one persistent block per CU: 4.0 + 1.75 steps for four times the outputs per block, and a partly filled
// last round costs a whole one.  (65536 x 2304 x 768: 233 against 289 us, 65536 x 768 x 768: 101 against 122,
// 65536 x 3072 x 768 + GELU: 351 against 424, 65536 x 768 x 3072: 295 against 360, 8192 x 50304 x 768: 690 against
// 892, 8192^3: 864 against 1044; the other way round 8192 x 2304 x 768: 47 against 43, 8192 x 3072 x 768: 55 against 52.)
bool gemm_big_tiles(const sif_gemm_args& a) {
  if (a.tile == 256) return true;
  if (a.tile == 128 || !gemm_can_use_big_tiles(a)) return false;
  const uint64_t batches = (uint64_t)a.batch_outer * a.batch_inner;
  const uint64_t tiles256 = (uint64_t)((a.m + 255) / 256) * ((a.n + 255) / 256) * batches;
  const uint64_t tiles128 = (uint64_t)((a.m + 127) / 128) * ((a.n + 127) / 128) * batches;
  const double steps = (double)(a.k / BK);
  const double t128 = (1.0 + 1.19 * steps) * std::max(0.85, (double)tiles128 / 512.0);
  const double t256 = (4.0 + 1.75 * steps) * (double)((tiles256 + 255) / 256);
  return t256 < t128;
}

// checks one product's arguments and fills its kernel record; *big: the 256x256 configuration was chosen
static sif_status gemm_fill(const sif_gemm_args* a, GemmP& p, bool* big_out) {
  if (a == nullptr || a->struct_size != sizeof(sif_gemm_args)) return fail(SIF_E_INVAL, "gemm: bad args struct");
  if (a->m == 0 || a->n == 0 || a->k == 0) return fail(SIF_E_INVAL, "gemm: empty extent");
  if (a->a_layout > 1 || a->b_layout > 1) return fail(SIF_E_INVAL, "gemm: bad layout");
  if (!a->a_dev || !a->b_dev || !a->c_dev) return fail(SIF_E_INVAL, "gemm: null operand");
  if (!aligned16(a->a_dev) || !aligned16(a->b_dev) || !aligned16(a->c_dev)) return fail(SIF_E_INVAL, "gemm: operands must be 16-byte aligned");
  if ((a->lda & 7) || (a->ldb & 7)) return fail(SIF_E_INVAL, "gemm: lda/ldb must be multiples of 8");
  // a lane's offset within an operand tile (up to 255 rows of ld elements) is kept in 32 bits
  if (a->lda > (1u << 22) || a->ldb > (1u << 22)) return fail(SIF_E_INVAL, "gemm: lda/ldb above 4194304 elements are not supported");
  if ((a->a_stride_outer | a->a_stride_inner | a->b_stride_outer | a->b_stride_inner) & 7) return fail(SIF_E_INVAL, "gemm: batch strides must be multiples of 8");
  const uint32_t a_contig = a->a_layout == SIF_A_ROW_K ? a->k : a->m;
  const uint32_t b_contig = a->b_layout == SIF_B_ROW_K ? a->k : a->n;
  if (a->lda < ((a_contig + 7) & ~7u) || a->ldb < ((b_contig + 7) & ~7u) || a->ldc < a->n) return fail(SIF_E_INVAL, "gemm: leading dimension too small");
  if (a->batch_outer == 0 || a->batch_inner == 0) return fail(SIF_E_INVAL, "gemm: batch counts must be >= 1");
  if ((a->epilogue & SIF_EPI_GELU_GRAD) && !a->aux_dev) return fail(SIF_E_INVAL, "gemm: GELU_GRAD needs aux");
  if ((a->epilogue & SIF_EPI_RESIDUAL) && !a->res_dev) return fail(SIF_E_INVAL, "gemm: RESIDUAL needs res");
  if ((a->epilogue & (SIF_EPI_BIAS | SIF_EPI_GELU)) == SIF_EPI_BIAS && !a->bias_dev) return fail(SIF_E_INVAL, "gemm: BIAS needs bias");
  if (a->k_causal > 2) return fail(SIF_E_INVAL, "gemm: bad k_causal");
  if (a->k_limit != 0 && (a->k_causal != 0 || (uint64_t)(a->batch_inner - 1) * a->k >= a->k_limit || a->k_limit > (uint64_t)a->batch_inner * a->k))
    return fail(SIF_E_INVAL, "gemm: k_limit must lie in the last of the batch_inner slices of k (no k_causal)");
  if ((a->n & 7) == 0) {
    // vector epilogue: rows of C, the residual and the auxiliary tensor are accessed 8 elements at a time
    if ((a->ldc & 7) || ((a->c_stride_outer | a->c_stride_inner) & 7)) return fail(SIF_E_INVAL, "gemm: ldc and the output batch strides must be multiples of 8 when n is");
    if ((a->bias_dev && !aligned16(a->bias_dev)) || (a->res_dev && !aligned16(a->res_dev)) || (a->aux_dev && !aligned16(a->aux_dev))) return fail(SIF_E_INVAL, "gemm: bias, residual and aux must be 16-byte aligned");
  }
  if (a->tile != 0 && a->tile != 128 && a->tile != 256) return fail(SIF_E_INVAL, "gemm: tile must be 0, 128 or 256");
  if (a->tile == 256 && !gemm_can_use_big_tiles(*a)) return fail(SIF_E_INVAL, "gemm: 256-wide tiles need k (and the last slice under k_limit) to be a multiple of 64 and no causal variant");
  const uint64_t batches = (uint64_t)a->batch_outer * a->batch_inner;
  const bool big = gemm_big_tiles(*a);
  const uint32_t bm = big ? 256 : 128, bn = bm;
  p.a = (const bf16_t*)a->a_dev; p.b = (const bf16_t*)a->b_dev; p.c = a->c_dev;
  p.bias = (a->epilogue & (SIF_EPI_BIAS | SIF_EPI_GELU)) ? (const bf16_t*)a->bias_dev : nullptr;
  p.res = a->res_dev; p.aux = (bf16_t*)a->aux_dev;
  p.m = a->m; p.n = a->n; p.k = a->k; p.lda = a->lda; p.ldb = a->ldb; p.ldc = a->ldc;
  p.epi = a->epilogue; p.k_causal = a->k_causal; p.batch_inner = a->batch_inner; p.k_limit = a->k_limit;
  p.a_so = a->a_stride_outer; p.a_si = a->a_stride_inner; p.b_so = a->b_stride_outer; p.b_si = a->b_stride_inner;
  p.c_so = a->c_stride_outer; p.c_si = a->c_stride_inner; p.alpha = a->alpha;
  p.tiles_n = (a->n + bn - 1) / bn; p.tiles_m = (a->m + bm - 1) / bm;
  p.group = nullptr; p.group_n = 0; p.tile_base = 0;
  if (batches > 65535) return fail(SIF_E_INVAL, "gemm: grid too large");
  *big_out = big;
  return SIF_OK;
}

typedef void (*gemm_kern_fn)(GemmP, KCtl);
static const gemm_kern_fn kGemm128[2][2] = {{gemm_bf16_kernel<0, 0, 128, 128, 2, 2, true>, gemm_bf16_kernel<0, 1, 128, 128, 2, 2, true>},
                                            {gemm_bf16_kernel<1, 0, 128, 128, 2, 2, true>, gemm_bf16_kernel<1, 1, 128, 128, 2, 2, true>}};
static const gemm_kern_fn kGemm256[2][2] = {{gemm_bf16_kernel<0, 0, 256, 256, 2, 4, false>, gemm_bf16_kernel<0, 1, 256, 256, 2, 4, false>},
                                            {gemm_bf16_kernel<1, 0, 256, 256, 2, 4, false>, gemm_bf16_kernel<1, 1, 256, 256, 2, 4, false>}};

sif_status launch_gemm_bf16(const sif_gemm_args* a, hipStream_t stream, const KCtl& ctl) {
  GemmP p;
  bool big = false;
  if (sif_status st = gemm_fill(a, p, &big)) return st;
  const uint64_t batches = (uint64_t)a->batch_outer * a->batch_inner;
  // 256x256 tiles: one block per CU, each working through every (number of CUs)-th tile; a stride that is a multiple of
  // 8 keeps a block on the tiles of its own XCD
  uint32_t grid_x = p.tiles_m * p.tiles_n;
  if (big && batches == 1) {
    static const uint32_t cus = [] {
      int dev = 0, n = 0;
      if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
      return (uint32_t)(n / 8 * 8);
    }();
    if (grid_x > cus) grid_x = cus;
  }
  dim3 grid(grid_x, 1, (uint32_t)batches);
  if (big) hipLaunchKernelGGL(kGemm256[a->a_layout][a->b_layout], grid, dim3(512), 0, stream, p, ctl);
  else hipLaunchKernelGGL(kGemm128[a->a_layout][a->b_layout], grid, dim3(256), 0, stream, p, ctl);
  return check_launch("gemm_bf16");
}

// Several products of the same operand layouts as ONE launch of 128x128 tiles (the weight gradients of a layer: each
// by itself has too few tiles for the chip and would have to be cut along K, with fp32 partial results written, read
// again and summed; together they fill it).  gemm_group_fill checks the products and writes their kernel records, to
// be copied to `gemm_group_bytes(n)` bytes of device memory once; launch_gemm_bf16_group then takes that copy.
uint64_t gemm_group_bytes(uint32_t n) { return (uint64_t)n * sizeof(GemmP); }

sif_status gemm_group_fill(const sif_gemm_args* list, uint32_t n, void* host_records, uint32_t* grid_out) {
  if (list == nullptr || n == 0 || n > 16 || host_records == nullptr || grid_out == nullptr) return fail(SIF_E_INVAL, "gemm group: bad arguments");
  GemmP* rec = static_cast<GemmP*>(host_records);
  uint32_t base = 0;
  for (uint32_t i = 0; i < n; ++i) {
    sif_gemm_args a = list[i];
    a.tile = 128;
    if (a.a_layout != list[0].a_layout || a.b_layout != list[0].b_layout) return fail(SIF_E_INVAL, "gemm group: the products must share their operand layouts");
    if ((uint64_t)a.batch_outer * a.batch_inner != 1) return fail(SIF_E_INVAL, "gemm group: no batched products");
    bool big = false;
    if (sif_status st = gemm_fill(&a, rec[i], &big)) return st;
    rec[i].tile_base = base;
    base += (rec[i].tiles_m * rec[i].tiles_n + 7u) & ~7u;       // a multiple of 8 keeps the tile order's idea of the XCDs
  }
  *grid_out = base;
  return SIF_OK;
}

sif_status launch_gemm_bf16_group(const void* dev_records, uint32_t n, uint32_t grid, uint32_t a_layout, uint32_t b_layout, hipStream_t stream, const KCtl& ctl) {
  if (dev_records == nullptr || n == 0 || grid == 0 || a_layout > 1 || b_layout > 1) return fail(SIF_E_INVAL, "gemm group: bad arguments");
  GemmP head = {};
  head.group = static_cast<const GemmP*>(dev_records);
  head.group_n = n;
  // (instantiated for the layouts of weight gradients, A [K][M] and B [K][N]; other layouts would need their own)
  if (a_layout != SIF_A_ROW_M || b_layout != SIF_B_ROW_N) return fail(SIF_E_INVAL, "gemm group: only A stored [K][M] with B stored [K][N]");
  hipLaunchKernelGGL((gemm_bf16_kernel<1, 1, 128, 128, 2, 2, true, true>), dim3(grid), dim3(256), 0, stream, head, ctl);
  return check_launch("gemm_bf16_group");
}

}  // namespace sif
