// Instantiations of the tiled MFMA convolution kernel, one group of variants.def
// rows per translation unit (BCONV_GROUP is set on the compiler command line).
#include "bconv_internal.h"
#include "tconv_mfma.hpp"

namespace bconv {

template <typename KernelT>
static hipError_t launch_tile_kernel(KernelT kernel, int nthr, const TconvParams& p, dim3 grid,
                                     size_t lds_bytes, hipStream_t st, bool* attr_set) {
  // Dynamic LDS above 64 KB must be allowed once per kernel and device.
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!attr_set[dev]) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimitBytes);
    if (e != hipSuccess) return e;
    attr_set[dev] = true;
  }
  hipLaunchKernelGGL(kernel, grid, dim3(nthr), lds_bytes, st, p);
  return hipGetLastError();
}

#define X(name, R, S, STR, WM, WN, MT, NT, KR, EPT)                                          \
  hipError_t launch_##name(const TconvParams& p, dim3 grid, size_t lds_bytes, hipStream_t st) { \
    static bool attr_set[64] = {false};                                                       \
    return launch_tile_kernel(tconv_mfma_kernel<R, S, STR, WM, WN, MT, NT, KR, EPT>,          \
                              WM * WN * 64, p, grid, lds_bytes, st, attr_set);                \
  }
#include "variants.def"
#undef X

}  // namespace bconv
