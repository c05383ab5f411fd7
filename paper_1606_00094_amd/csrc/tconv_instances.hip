// Instantiations of the tiled MFMA convolution kernel, one group of variants.def
// rows per translation unit (BCONV_GROUP is set on the compiler command line).
#include <atomic>
#include <cstdio>
#include <cstdlib>

#include "bconv_internal.h"
#include "tconv_mfma.hpp"

namespace bconv {

static void report(const char* what, hipError_t e) {
  if (std::getenv("BCONV_DEBUG"))
    std::fprintf(stderr, "bconv: %s: %s\n", what, hipGetErrorString(e));
}

template <typename KernelT>
static hipError_t launch_tile_kernel(KernelT kernel, int nthr, const TconvParams& p, dim3 grid,
                                     size_t lds_bytes, hipStream_t st,
                                     std::atomic<size_t>* lds_allowed) {
  // Dynamic LDS above the default limit must be allowed per kernel and device.
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { report("hipGetDevice", e); return e; }
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  // (host threads may race here: the attribute call is idempotent and the largest value wins)
  if (lds_bytes > 32768 && lds_bytes > lds_allowed[dev].load(std::memory_order_relaxed)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) { report("hipFuncSetAttribute", e); (void)hipGetLastError(); return e; }
    lds_allowed[dev].store(lds_bytes, std::memory_order_relaxed);
  }
  e = launch_kernel(kernel, grid, dim3(nthr), lds_bytes, st, p);
  if (e != hipSuccess) report("kernel launch", e);
  return e;
}

#define X(name, R, S, STR, WM, WN, MT, NT, KR, EPT, AV, KS, BV, PD, WPE, MS)                                          \
  hipError_t launch_##name(const TconvParams& p, dim3 grid, size_t lds_bytes, hipStream_t st) { \
    static std::atomic<size_t> lds_allowed[64];                                                        \
    return launch_tile_kernel(tconv_mfma_kernel<R, S, STR, WM, WN, MT, NT, KR, EPT, AV, KS, BV, PD, WPE, MS>,  \
                              WM * WN * KS * 64, p, grid, lds_bytes, st, lds_allowed);                \
  }                                                                                             \
  hipError_t launch_f16_##name(const TconvParams& p, dim3 grid, size_t lds_bytes, hipStream_t st) { \
    static std::atomic<size_t> lds_allowed[64];                                                        \
    return launch_tile_kernel(tconv_mfma_kernel<R, S, STR, WM, WN, MT, NT, KR, EPT, AV, KS, BV, PD, WPE, MS, _Float16>,  \
                              WM * WN * KS * 64, p, grid, lds_bytes, st, lds_allowed);                \
  }
#include "variants.def"
#undef X

}  // namespace bconv
