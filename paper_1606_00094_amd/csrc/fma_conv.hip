// Register-blocked vector-FMA convolution for first-layer shapes (few input channels, a
// kernel several times wider than its stride): the second contender for the layers the MFMA
// tiles serve through their k11s4 / k7s2 families, kept so that the choice between the
// two is a measured one.
//
// Lane layout.  With stride STR (2 or 4) a wave takes 64 / STR consecutive output pixels of
// one output row and gives each pixel STR lanes; lane l = pixel * STR + j works on the kernel
// columns s = j, j + STR, j + 2 STR, ...  Pixel q reads input column q * STR - pad + s, so
// for a fixed step i (s = i * STR + j) the 64 lanes read 64 CONSECUTIVE input words: the
// stride that makes a first layer's loads gather-like for a lane-per-pixel kernel is
// absorbed by the lane split and every global load is one contiguous 256-byte run.  Each lane
// keeps KB accumulators (KB filters of the workgroup's filter group) in registers; its
// partial sums over the columns of its phase j are added to those of the other STR - 1
// lanes of the pixel with DPP quad permutes at the end (no LDS, no shuffles through memory).
//
// The filters of the group are staged once per workgroup in LDS, transposed to
// [c][r][i][j][k] so that a lane reads the KB values of its (step, phase) with 16-byte LDS
// reads that are uniform over the pixels; columns s >= S of the last step hold zeros.  A
// workgroup (four waves) then walks pixel groups of its filter group until the grid has
// covered them all.
//
// Vector FMAs run at 64 lanes x 2 flop / 4 cycles per SIMD, half the rate of the fp32 matrix
// pipe (packed two-wide fp32 instructions are not used in this library), so this kernel
// cannot win where the MFMA tiles are limited by the matrix pipe; it is a contender where
// they are limited by latency.
#include "bconv_internal.h"

namespace bconv {

template <int CTRL>
__device__ __forceinline__ float quad_perm_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true);
  return v + __builtin_bit_cast(float, moved);
}

struct FmaParams {
  const float* in;
  const float* filt;
  const float* bias;     // may be null
  float* out;
  int N, C, H, W, K, R, S, pad, P, Q;
  int relu;
  int NI;                // steps per kernel row: ceil(S / STR)
  int GQ;                // pixel groups per output row
  int groups;            // N * P * GQ
  FastDiv fdGQ, fdP;
};

template <int STR, int KB>
__global__ __launch_bounds__(256)
void fma_conv_kernel(const FmaParams p) {
  static_assert(STR == 2 || STR == 4, "lanes per pixel");
  static_assert(KB % 4 == 0 && KB % STR == 0, "filters per group");
  constexpr int PXW = 64 / STR;                 // pixels per wave
  extern __shared__ __attribute__((aligned(16))) float fl[];   // [C*R*NI][STR][KB]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int k0 = blockIdx.y * KB;
  const int steps = p.C * p.R * p.NI;

  // ---- filters of this group into LDS, transposed; zeros for columns past S and filters past K
  const int CRS = p.C * p.R * p.S;
  for (int e = tid; e < steps * STR * KB; e += 256) {
    const int k = e % KB, sj = e / KB;          // sj = step * STR + j
    const int j = sj % STR, step = sj / STR;
    const int i = step % p.NI, cr = step / p.NI;
    const int s = i * STR + j;
    float v = 0.0f;
    if (s < p.S && k0 + k < p.K) v = p.filt[(size_t)(k0 + k) * CRS + (size_t)cr * p.S + s];
    fl[e] = v;
  }
  __syncthreads();

  const int j = lane % STR, px = lane / STR;
  for (int g = blockIdx.x * 4 + wave; g < p.groups; g += gridDim.x * 4) {
    const int row = fd_div(g, p.fdGQ), gq = g - row * p.GQ;       // row = n * P + pp
    const int n = fd_div(row, p.fdP), pp = row - n * p.P;
    const int q = gq * PXW + px;
    // input column of this lane at step i = 0; every step adds STR
    const int x0 = gq * PXW * STR - p.pad + lane;
    float acc[KB];
#pragma unroll
    for (int k = 0; k < KB; ++k) acc[k] = 0.0f;
    const float* flp = fl + j * KB;
    for (int c = 0; c < p.C; ++c) {
      for (int r = 0; r < p.R; ++r) {
        const int iy = pp * STR - p.pad + r;
        const bool rowok = (unsigned)iy < (unsigned)p.H;
        const float* src = p.in + ((size_t)(n * p.C + c) * p.H + (rowok ? iy : 0)) * p.W;
        for (int i = 0; i < p.NI; ++i) {
          const int x = x0 + i * STR;
          // (a column past S multiplies a zero filter word, and must be zero itself: it belongs
          // to the next pixel's window, and 0 x Inf would be NaN)
          const float v = (rowok && (unsigned)x < (unsigned)p.W && i * STR + j < p.S) ? src[x] : 0.0f;
#pragma unroll
          for (int k4 = 0; k4 < KB; k4 += 4) {
            const float4 f = *reinterpret_cast<const float4*>(flp + k4);
            acc[k4] = fmaf(v, f.x, acc[k4]);
            acc[k4 + 1] = fmaf(v, f.y, acc[k4 + 1]);
            acc[k4 + 2] = fmaf(v, f.z, acc[k4 + 2]);
            acc[k4 + 3] = fmaf(v, f.w, acc[k4 + 3]);
          }
          flp += STR * KB;
        }
      }
    }
    // ---- sum over the STR lanes of each pixel: quad permutes [1,0,3,2], then [2,3,0,1]
#pragma unroll
    for (int k = 0; k < KB; ++k) {
      acc[k] = quad_perm_add<0xB1>(acc[k]);
      if constexpr (STR == 4) acc[k] = quad_perm_add<0x4E>(acc[k]);
    }
    // ---- bias + ReLU + store: every lane of a pixel holds all sums; lane j stores filters
    // j, j + STR, ... of the group, so that all 64 lanes store
    if (q < p.Q) {
      float* dst = p.out + ((size_t)n * p.K + k0) * p.P * p.Q + (size_t)pp * p.Q + q;
#pragma unroll
      for (int k = 0; k < KB; ++k) {
        if (k % STR == j && k0 + k < p.K) {
          float v = acc[k] + (p.bias ? p.bias[k0 + k] : 0.0f);
          if (p.relu) v = v > 0.0f ? v : 0.0f;
          dst[(size_t)k * p.P * p.Q] = v;
        }
      }
    }
  }
}

struct FmaVariant {
  const char* name;
  int STR, KB;
};
static const FmaVariant kFma[] = {{"fmaq4_kb32", 4, 32}, {"fmaq4_kb16", 4, 16}, {"fmaq2_kb32", 2, 32}};

int fma_num_variants() { return (int)(sizeof(kFma) / sizeof(kFma[0])); }
const char* fma_variant_name(int which) { return kFma[which].name; }

static size_t fma_lds_bytes(const Shape& s, const FmaVariant& v) {
  const int NI = (s.S + v.STR - 1) / v.STR;
  return (size_t)s.C * s.R * NI * v.STR * v.KB * sizeof(float);
}

// First-layer shapes only: the stride the lanes are split by, fp32 storage, a filter group
// that fits LDS, 32-bit indexing inside an image plane and over the pixel groups.
bool fma_conv_applicable(int which, const Shape& s) {
  const FmaVariant& v = kFma[which];
  if (s.stride != v.STR || s.S < v.STR) return false;
  if (fma_lds_bytes(s, v) > 64 * 1024) return false;
  const long long i31 = (1LL << 31) - 1;
  const long long GQ = (s.Q + 64 / v.STR - 1) / (64 / v.STR);
  if ((long long)s.N * s.P * GQ > i31 || (long long)s.N * s.C > i31 || (long long)s.W * v.STR + s.S + 64 > i31)
    return false;
  return true;
}

hipError_t launch_fma_conv(int which, const float* in, const float* filt, const float* bias, float* out,
                           const Shape& s, int relu, hipStream_t st) {
  const FmaVariant& v = kFma[which];
  FmaParams p;
  p.in = in; p.filt = filt; p.bias = bias; p.out = out;
  p.N = s.N; p.C = s.C; p.H = s.H; p.W = s.W; p.K = s.K; p.R = s.R; p.S = s.S; p.pad = s.pad;
  p.P = s.P; p.Q = s.Q; p.relu = relu;
  p.NI = (s.S + v.STR - 1) / v.STR;
  p.GQ = (s.Q + 64 / v.STR - 1) / (64 / v.STR);
  p.groups = s.N * s.P * p.GQ;
  p.fdGQ = make_fastdiv((unsigned)p.GQ);
  p.fdP = make_fastdiv((unsigned)s.P);
  const unsigned gy = (unsigned)((s.K + v.KB - 1) / v.KB);
  // enough workgroups to fill the chip a few times over, each walking its share of the groups
  long long gx = ((long long)p.groups + 3) / 4;
  const long long cap = (256 * 8 + gy - 1) / gy;
  if (gx > cap) gx = cap;
  const size_t lds = fma_lds_bytes(s, v);
  const dim3 grid((unsigned)gx, gy), block(256);
  if (v.STR == 4 && v.KB == 32) {
    if (lds > 32768) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fma_conv_kernel<4, 32>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    return launch_kernel(fma_conv_kernel<4, 32>, grid, block, lds, st, p);
  }
  if (v.STR == 4 && v.KB == 16) return launch_kernel(fma_conv_kernel<4, 16>, grid, block, lds, st, p);
  if (lds > 32768) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fma_conv_kernel<2, 32>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  return launch_kernel(fma_conv_kernel<2, 32>, grid, block, lds, st, p);
}

}  // namespace bconv
