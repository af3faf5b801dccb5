// sif_k_colsum_static: the column sum of sif_k_colsum for callers that cannot allocate device memory (code under
// HIP graph capture, serving loops, harnesses that forbid hipMalloc).  The per-block partial sums, which
// sif_k_colsum keeps in a buffer the caller brings, live here in a file-scope device array of fixed size.
//
// The array's name is a host-side stand-in in host code; its device address is looked up once per device with
// hipGetSymbolAddress and only that address is ever handed to a kernel.  Every GPU the library runs on holds its
// own copy of the array (4 MiB) until the process ends.
#include <mutex>

#include "launch.h"

namespace sif {

constexpr uint64_t kStaticScratchFloats = 1ull << 20;      // 4 MiB of partial sums
static __device__ __align__(256) float scratch[kStaticScratchFloats];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static float* g_scratch_ptr[kMaxDevices];                  // device address of `scratch` on each device, once known

// Address of the array on the current device (looked up the first time a device is used).
static sif_status static_scratch(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "colsum_static: hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(SIF_E_INVAL, "colsum_static: device %d out of range", dev);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    float* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e, "colsum_static: hipGetSymbolAddress");
    if (p == nullptr) return fail(SIF_E_DEVICE, "colsum_static: the scratch array has no address on device %d", dev);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SIF_OK;
}

}  // namespace sif

using namespace sif;

extern "C" {

uint64_t sif_colsum_static_max_floats(void) { return kStaticScratchFloats; }

sif_status sif_k_colsum_static(const void* x_dev, uint32_t ld, void* out_dev, uint32_t rows, uint32_t n, void* stream) {
  if (!out_dev) return fail(SIF_E_INVAL, "colsum_static: null out");
  if (rows == 0 || n == 0) return fail(SIF_E_INVAL, "colsum_static: empty input");
  const uint64_t need = (uint64_t)colsum_parts(rows) * n;
  if (need > kStaticScratchFloats)
    return fail(SIF_E_NOMEM, "colsum_static: %u rows x %u columns need %llu floats of scratch, the static buffer holds %llu; use sif_k_colsum",
                rows, n, (unsigned long long)need, (unsigned long long)kStaticScratchFloats);
  float* part = nullptr;
  sif_status st = static_scratch(&part);
  if (st != SIF_OK) return st;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  // every partial sum the second kernel reads is written by the first (all `parts` rows of all n columns): nothing
  // has to start at zero, whatever an earlier call left behind
  st = launch_colsum_part(x_dev, ld, part, rows, n, s, no_ctl());
  if (st != SIF_OK) return st;
  return launch_colsum_fin(part, out_dev, rows, n, 0, s, no_ctl());
}

}  // extern "C"
