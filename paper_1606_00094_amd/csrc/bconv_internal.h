// Host-side declarations shared by the translation units of libbconv.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "bconv_plan.h"

namespace bconv {

// Launches `kernel` and returns the status of this launch alone.  (A launch written with the
// triple-bracket syntax reports through hipGetLastError, which also hands back an error that
// an earlier, unrelated call left behind in the thread: the caller would then be told that
// nothing was enqueued when the kernel was.)  Arguments convert to the kernel's own
// parameter types.
template <typename... P>
inline hipError_t launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds_bytes,
                                hipStream_t st, std::common_type_t<P>... args) {
  void* ptrs[] = {const_cast<void*>(static_cast<const void*>(&args))...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, st);
}

typedef hipError_t (*TileLaunchFn)(const TconvParams& p, dim3 grid, size_t lds_bytes,
                                   hipStream_t st);

// launch_<tile>: fp32 tensors; launch_f16_<tile>: half-precision tensors behind the same
// argument block (its float pointers then address _Float16 elements; bias and partial
// sums stay fp32).
#define X(name, R, S, STR, WM, WN, MT, NT, KR, EPT, AV, KS, BV, PD, WPE, MS) \
  hipError_t launch_##name(const TconvParams& p, dim3 grid, size_t lds_bytes, hipStream_t st); \
  hipError_t launch_f16_##name(const TconvParams& p, dim3 grid, size_t lds_bytes, hipStream_t st);
#include "variants.def"
#undef X

// Auxiliary kernels (aux_kernels.hip).
// f16: in, filt and out address _Float16 elements (bias and partial sums are fp32 always).
hipError_t launch_direct_conv(const float* in, const float* filt, const float* bias, float* out,
                              const Shape& s, int relu, bool f16, hipStream_t st);
// (c8: the output is octet-interleaved, [N][K/8][PQ][8]; only the bias index depends on it)
hipError_t launch_splitk_reduce(const float* partial, const float* bias, float* out, int nsplit,
                                int out_elems, int K, int PQ, int relu, bool f16, bool c8, hipStream_t st);
hipError_t launch_splitk_reduce_pool(const float* partial, const float* bias, float* out, int nsplit,
                                     int out_elems, int N, int K, int P, int Q, int ksz, int pstride,
                                     int relu, hipStream_t st);
hipError_t launch_maxpool(const float* in, float* out, int N, int C, int H, int W, int ksz,
                          int stride, int P, int Q, hipStream_t st);

hipError_t launch_mfma_loop(float* out, int workgroups, int iters, hipStream_t st);

// Register-blocked vector-FMA kernels for first-layer shapes (fma_conv.hip); `which` indexes
// its small catalogue.  fp32 storage only, no reduction split, no workspace.
int fma_num_variants();
const char* fma_variant_name(int which);
bool fma_conv_applicable(int which, const Shape& s);
hipError_t launch_fma_conv(int which, const float* in, const float* filt, const float* bias, float* out,
                           const Shape& s, int relu, hipStream_t st);

// Half-precision convolution on the fp16 matrix cores (hconv_mfma.hip); `which` indexes its
// catalogue.  fp16 storage only; needs hconv_workspace_bytes of device scratch for the re-laid
// filters.
// First-layer kernels on the fp16 matrix cores (hconv_first.hip): C <= 3, 11x11 step 4 or 7x7
// step 2; `which` indexes their own list, which hconv_* appends to its catalogue.
int hfl_num_variants();
const char* hfl_variant_name(int which);
bool hfl_applicable(int which, const Shape& s);
size_t hfl_workspace_bytes(int which, const Shape& s);
long long hfl_tiles(int which, const Shape& s);     // pixel tiles of the launch (0 if not applicable)
hipError_t launch_hfl(int which, const void* in, const void* filt, const float* bias, void* out, const Shape& s,
                      int relu, int out_c8, void* ws, hipStream_t st);
// (false for the first-layer tiles: their filters cannot be packed ahead of the call, they
// need workspace for the padded input as well)
bool hconv_packable(int which);
int hconv_num_variants();
const char* hconv_variant_name(int which);
bool hconv_applicable(int which, const Shape& s);
size_t hconv_workspace_bytes(int which, const Shape& s);
// (any_size: also for launches too small to fill the chip, where the widening kernel would win
// on NCHW activations -- the octet-interleaved layout has no other kernel)
int hconv_select(const Shape& s, bool any_size = false);
// (in_c8 / out_c8: octet-interleaved activations; the first-layer tiles take NCHW input only,
// C8 output needs K % 8 == 0 and, for the channel-octet tiles, C8 input)
hipError_t launch_hconv(int which, const void* in, const void* filt, const float* bias, void* out,
                        const Shape& s, int relu, int in_c8, int out_c8, void* ws, hipStream_t st);
hipError_t launch_hconv_pack(int which, const void* filt, void* packed, const Shape& s, hipStream_t st);
hipError_t launch_hconv_packed(int which, const void* in, const void* packed, const float* bias, void* out,
                               const Shape& s, int relu, int in_c8, int out_c8, void* scratch, hipStream_t st);
double hconv_model_cost(int which, const Shape& s);      // the selection's estimate in us, < 0 if none
int hconv_variant_split(int which);                       // reduction split of a catalogue entry
size_t hconv_packed_bytes(int which, const Shape& s);     // re-laid filters alone
size_t hconv_partial_bytes(int which, const Shape& s);    // partial sums of a split variant (else 0)
// fp16 activations between NCHW and the octet-interleaved layout [N][C/8][H*W][8]
// (n_times_c = N * C, a multiple of eight); to_c8 = 1: NCHW -> C8, 0: back.
// Max pooling of fp16 activations, NCHW (c8 = 0) or octet-interleaved (c8 = 1).
hipError_t launch_maxpool_f16(const void* in, void* out, long long n_times_c, int H, int W, int ksz, int stride,
                              int P, int Q, int c8, hipStream_t st);
hipError_t launch_f16_layout(const void* in, void* out, long long n_times_c, int HW, int to_c8, hipStream_t st);

}  // namespace bconv
