// Host-side declarations shared by the translation units of libbconv.
#pragma once
#include <hip/hip_runtime.h>

#include "bconv_plan.h"

namespace bconv {

typedef hipError_t (*TileLaunchFn)(const TconvParams& p, dim3 grid, size_t lds_bytes,
                                   hipStream_t st);

#define X(name, R, S, STR, WM, WN, MT, NT, KR, EPT, AV, KS, BV, PD, WPE) \
  hipError_t launch_##name(const TconvParams& p, dim3 grid, size_t lds_bytes, hipStream_t st);
#include "variants.def"
#undef X

// Auxiliary kernels (aux_kernels.hip).
hipError_t launch_direct_conv(const float* in, const float* filt, const float* bias, float* out,
                              const Shape& s, int relu, hipStream_t st);
hipError_t launch_splitk_reduce(const float* partial, const float* bias, float* out, int nsplit,
                                int out_elems, int K, int PQ, int relu, hipStream_t st);
hipError_t launch_maxpool(const float* in, float* out, int N, int C, int H, int W, int ksz,
                          int stride, int P, int Q, hipStream_t st);

hipError_t launch_mfma_loop(float* out, int workgroups, int iters, hipStream_t st);

}  // namespace bconv
