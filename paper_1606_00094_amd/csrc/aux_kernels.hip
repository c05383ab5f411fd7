// Small kernels around the tiled MFMA convolution: the plain direct convolution
// (always-applicable fallback, variant 0), the split-K reduction with the fused
// bias + ReLU epilogue (optionally with max pooling folded in), max pooling, and a
// register-only MFMA loop used as a measurement aid.
#include <cstdint>

#include "bconv_internal.h"

namespace bconv {

// One thread per output point, loops over (c, r, s): the definition of the
// paper's Section II executed literally, fp32 accumulation, 64-bit indexing.
// T is the storage type of input, filters and output (float or _Float16).
template <typename T>
__global__ __launch_bounds__(256)
void direct_conv_kernel(const T* __restrict__ in, const T* __restrict__ filt,
                        const float* __restrict__ bias, T* __restrict__ out, Shape s,
                        int relu, long long total) {
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    int q = (int)(idx % s.Q);
    long long t = idx / s.Q;
    int p = (int)(t % s.P);
    t /= s.P;
    int k = (int)(t % s.K);
    int n = (int)(t / s.K);
    const int ih0 = p * s.stride - s.pad, iw0 = q * s.stride - s.pad;
    float acc = 0.0f;
    for (int c = 0; c < s.C; ++c) {
      const T* ip = in + ((long long)n * s.C + c) * s.H * s.W;
      const T* fp = filt + ((long long)k * s.C + c) * s.R * s.S;
      for (int r = 0; r < s.R; ++r) {
        int ih = ih0 + r;
        if (ih < 0 || ih >= s.H) continue;
        for (int ss = 0; ss < s.S; ++ss) {
          int iw = iw0 + ss;
          if (iw < 0 || iw >= s.W) continue;
          acc = fmaf((float)ip[(long long)ih * s.W + iw], (float)fp[r * s.S + ss], acc);
        }
      }
    }
    if (bias) acc += bias[k];
    if (relu) acc = acc > 0.0f ? acc : 0.0f;
    out[idx] = (T)acc;
  }
}

hipError_t launch_direct_conv(const float* in, const float* filt, const float* bias, float* out,
                              const Shape& s, int relu, bool f16, hipStream_t st) {
  long long total = (long long)s.N * s.K * s.P * s.Q;
  long long blocks = (total + 255) / 256;
  if (blocks > 65536 * 16) blocks = 65536 * 16;
  if (f16)
    return launch_kernel(direct_conv_kernel<_Float16>, dim3((unsigned)blocks), dim3(256), 0, st,
                         reinterpret_cast<const _Float16*>(in), reinterpret_cast<const _Float16*>(filt),
                         bias, reinterpret_cast<_Float16*>(out), s, relu, total);
  return launch_kernel(direct_conv_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, in, filt,
                       bias, out, s, relu, total);
}

// Filter index of output element e of an N x K x PQ tensor: (e / PQ) % K, the two divisions
// as multiplies and shifts with constants made by the host (a run-time integer division is
// ~30 instructions, and these kernels are a handful of loads long).
// (octet-interleaved output [N][K/8][PQ][8]: the host passes K/8 and 8*PQ, and the filter is
// eight times the octet plus the element's position in its octet)
__device__ __forceinline__ int filter_of(int e, int K, FastDiv fdPQ, FastDiv fdK, int c8 = 0) {
  const int plane = fd_div(e, fdPQ);
  const int k = plane - fd_div(plane, fdK) * K;
  return c8 ? k * 8 + (e & 7) : k;
}

// out[i] = act(bias[k(i)] + sum_z partial[z][i]), summed in split order.
template <typename T>
__global__ __launch_bounds__(256)
void splitk_reduce_kernel(const float* __restrict__ partial, const float* __restrict__ bias,
                          T* __restrict__ out, int nsplit, int out_elems, int K, int PQ,
                          int relu, FastDiv fdPQ, FastDiv fdK, int c8) {
  // (64-bit counter: i + stride may pass 2^31 when out_elems is close to it)
  for (long long i64 = (long long)blockIdx.x * blockDim.x + threadIdx.x; i64 < out_elems;
       i64 += (long long)gridDim.x * blockDim.x) {
    const int i = (int)i64;
    float v = 0.0f;
    for (int z = 0; z < nsplit; ++z) v += partial[(size_t)z * out_elems + i];
    if (bias) v += bias[filter_of(i, K, fdPQ, fdK, c8)];
    if (relu) v = v > 0.0f ? v : 0.0f;
    out[i] = (T)v;
  }
}

// Four results as stored: fp32 (16 bytes) or half precision (8 bytes).
struct alignas(8) Half4 { _Float16 v[4]; };
__device__ __forceinline__ void store_quad(float4* dst, const float4& v) { *dst = v; }
__device__ __forceinline__ void store_quad(Half4* dst, const float4& v) {
  Half4 h;
  h.v[0] = (_Float16)v.x; h.v[1] = (_Float16)v.y; h.v[2] = (_Float16)v.z; h.v[3] = (_Float16)v.w;
  *dst = h;
}

// The same sum four consecutive elements at a time with 16-byte accesses (out_elems % 4 == 0,
// 16-byte aligned partial, out aligned to four elements); the additions per element are in the
// same order.  Q4 is float4 or Half4.
template <typename Q4>
__global__ __launch_bounds__(256)
void splitk_reduce4_kernel(const float4* __restrict__ partial, const float* __restrict__ bias,
                           Q4* __restrict__ out, int nsplit, int out_quads, int K, int PQ,
                           int relu, FastDiv fdPQ, FastDiv fdK, int c8) {
  for (long long i64 = (long long)blockIdx.x * blockDim.x + threadIdx.x; i64 < out_quads;
       i64 += (long long)gridDim.x * blockDim.x) {
    const int i = (int)i64;
    float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    int z = 0;
    // eight, then four loads in flight at a time; the additions stay in split order
    for (; z + 8 <= nsplit; z += 8) {
      float4 w[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) w[u] = partial[(size_t)(z + u) * out_quads + i];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        v.x += w[u].x; v.y += w[u].y; v.z += w[u].z; v.w += w[u].w;
      }
    }
    for (; z + 4 <= nsplit; z += 4) {
      const float4 w0 = partial[(size_t)z * out_quads + i];
      const float4 w1 = partial[(size_t)(z + 1) * out_quads + i];
      const float4 w2 = partial[(size_t)(z + 2) * out_quads + i];
      const float4 w3 = partial[(size_t)(z + 3) * out_quads + i];
      v.x += w0.x; v.y += w0.y; v.z += w0.z; v.w += w0.w;
      v.x += w1.x; v.y += w1.y; v.z += w1.z; v.w += w1.w;
      v.x += w2.x; v.y += w2.y; v.z += w2.z; v.w += w2.w;
      v.x += w3.x; v.y += w3.y; v.z += w3.z; v.w += w3.w;
    }
    for (; z < nsplit; ++z) {
      const float4 w = partial[(size_t)z * out_quads + i];
      v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
    }
    if (bias) {
      const int e = i * 4;
      v.x += bias[filter_of(e, K, fdPQ, fdK, c8)];
      v.y += bias[filter_of(e + 1, K, fdPQ, fdK, c8)];
      v.z += bias[filter_of(e + 2, K, fdPQ, fdK, c8)];
      v.w += bias[filter_of(e + 3, K, fdPQ, fdK, c8)];
    }
    if (relu) {
      v.x = v.x > 0.0f ? v.x : 0.0f; v.y = v.y > 0.0f ? v.y : 0.0f;
      v.z = v.z > 0.0f ? v.z : 0.0f; v.w = v.w > 0.0f ? v.w : 0.0f;
    }
    store_quad(out + i, v);
  }
}

hipError_t launch_splitk_reduce(const float* partial, const float* bias, float* out, int nsplit,
                                int out_elems, int K, int PQ, int relu, bool f16, bool c8, hipStream_t st) {
  if (c8) { K /= 8; PQ *= 8; }
  const int c8i = c8 ? 1 : 0;
  const FastDiv fdPQ = make_fastdiv((unsigned)PQ), fdK = make_fastdiv((unsigned)K);
  const uintptr_t out_mask = f16 ? 7 : 15;
  const bool quads = (out_elems % 4 == 0) && ((reinterpret_cast<uintptr_t>(partial) & 15) == 0) &&
                     ((reinterpret_cast<uintptr_t>(out) & out_mask) == 0);
  if (quads) {
    const int n4 = out_elems / 4;
    int blocks = (n4 + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    const float4* p4 = reinterpret_cast<const float4*>(partial);
    if (f16)
      return launch_kernel(splitk_reduce4_kernel<Half4>, dim3(blocks), dim3(256), 0, st, p4, bias,
                           reinterpret_cast<Half4*>(out), nsplit, n4, K, PQ, relu, fdPQ, fdK, c8i);
    return launch_kernel(splitk_reduce4_kernel<float4>, dim3(blocks), dim3(256), 0, st, p4, bias,
                         reinterpret_cast<float4*>(out), nsplit, n4, K, PQ, relu, fdPQ, fdK, c8i);
  }
  int blocks = (out_elems + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (f16)
    return launch_kernel(splitk_reduce_kernel<_Float16>, dim3(blocks), dim3(256), 0, st, partial, bias,
                         reinterpret_cast<_Float16*>(out), nsplit, out_elems, K, PQ, relu, fdPQ, fdK, c8i);
  return launch_kernel(splitk_reduce_kernel<float>, dim3(blocks), dim3(256), 0, st, partial, bias, out,
                       nsplit, out_elems, K, PQ, relu, fdPQ, fdK, c8i);
}

// Split reduction with the pooling folded in: one thread per pooled output point takes the
// max over its ksz x ksz window of act(bias + sum_z partial[z][.]), each element summed in
// split order exactly as splitk_reduce_kernel does, so the result equals reducing first and
// pooling afterwards bit for bit.  An element shared by neighbouring windows is summed once
// per window (2.25 times on average for 3x3 / 2); the layers that split are the small ones.
__global__ __launch_bounds__(256)
void splitk_reduce_pool_kernel(const float* __restrict__ partial, const float* __restrict__ bias,
                               float* __restrict__ out, int nsplit, int out_elems, int K, int P,
                               int Q, int PP, int PQ2, int ksz, int pstride, int relu,
                               long long total, FastDiv fdPQ2, FastDiv fdPP, FastDiv fdK) {
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    // total <= out_elems < 2^31: the index splits with 32-bit multiply-and-shift divisions
    const int t = fd_div((int)idx, fdPQ2), q2 = (int)idx - t * PQ2;
    const int nk = fd_div(t, fdPP), p2 = t - nk * PP;   // nk = image * K + filter
    const float b = bias ? bias[nk - fd_div(nk, fdK) * K] : 0.0f;
    const long long plane = (long long)nk * P * Q;
    float m = 0.0f;
    for (int r = 0; r < ksz; ++r)
      for (int c = 0; c < ksz; ++c) {
        const long long e = plane + (long long)(p2 * pstride + r) * Q + (q2 * pstride + c);
        float v = 0.0f;
        for (int z = 0; z < nsplit; ++z) v += partial[(size_t)z * out_elems + e];
        v += b;
        if (relu) v = v > 0.0f ? v : 0.0f;
        m = (r == 0 && c == 0) ? v : (v > m ? v : m);
      }
    out[idx] = m;
  }
}

// The same for a window and step fixed at compile time: the KSZ*KSZ elements of a window
// are summed side by side, four splits at a time, so that up to 4*KSZ*KSZ loads are in
// flight per thread instead of one (the generic kernel above pays a memory round trip
// per load).  Per element the additions are still in split order.
template <int KSZ, int PSTRIDE>
__global__ __launch_bounds__(256)
void splitk_reduce_pool_fixed_kernel(const float* __restrict__ partial,
                                     const float* __restrict__ bias, float* __restrict__ out,
                                     int nsplit, int out_elems, int K, int P, int Q, int PP, int PQ2,
                                     int relu, long long total, FastDiv fdPQ2, FastDiv fdPP,
                                     FastDiv fdK) {
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int t = fd_div((int)idx, fdPQ2), q2 = (int)idx - t * PQ2;
    const int nk = fd_div(t, fdPP), p2 = t - nk * PP;
    const float b = bias ? bias[nk - fd_div(nk, fdK) * K] : 0.0f;
    const float* src = partial + (long long)nk * P * Q + (long long)(p2 * PSTRIDE) * Q + q2 * PSTRIDE;
    float v[KSZ * KSZ];
#pragma unroll
    for (int e = 0; e < KSZ * KSZ; ++e) v[e] = 0.0f;
    int z = 0;
    for (; z + 4 <= nsplit; z += 4) {
      float w[4][KSZ * KSZ];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < KSZ * KSZ; ++e)
          w[u][e] = src[(size_t)(z + u) * out_elems + (e / KSZ) * Q + (e % KSZ)];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < KSZ * KSZ; ++e) v[e] += w[u][e];
    }
    for (; z < nsplit; ++z) {
      float w[KSZ * KSZ];
#pragma unroll
      for (int e = 0; e < KSZ * KSZ; ++e) w[e] = src[(size_t)z * out_elems + (e / KSZ) * Q + (e % KSZ)];
#pragma unroll
      for (int e = 0; e < KSZ * KSZ; ++e) v[e] += w[e];
    }
    float m = 0.0f;
#pragma unroll
    for (int e = 0; e < KSZ * KSZ; ++e) {
      float x = v[e] + b;
      if (relu) x = x > 0.0f ? x : 0.0f;
      m = e == 0 ? x : (x > m ? x : m);
    }
    out[idx] = m;
  }
}

hipError_t launch_splitk_reduce_pool(const float* partial, const float* bias, float* out, int nsplit,
                                     int out_elems, int N, int K, int P, int Q, int ksz, int pstride,
                                     int relu, hipStream_t st) {
  const int PP = (P - ksz) / pstride + 1, PQ2 = (Q - ksz) / pstride + 1;
  const long long total = (long long)N * K * PP * PQ2;
  long long blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  const FastDiv fdPQ2 = make_fastdiv((unsigned)PQ2), fdPP = make_fastdiv((unsigned)PP),
                fdK = make_fastdiv((unsigned)K);
  if (ksz == 3 && pstride == 2)
    return launch_kernel(splitk_reduce_pool_fixed_kernel<3, 2>, dim3((unsigned)blocks), dim3(256), 0, st,
                         partial, bias, out, nsplit, out_elems, K, P, Q, PP, PQ2, relu, total, fdPQ2,
                         fdPP, fdK);
  return launch_kernel(splitk_reduce_pool_kernel, dim3((unsigned)blocks), dim3(256), 0, st, partial,
                       bias, out, nsplit, out_elems, K, P, Q, PP, PQ2, ksz, pstride, relu, total, fdPQ2,
                       fdPP, fdK);
}

// One (image, channel) plane per blockIdx.y (strided when there are more planes than the
// grid allows), 256 output points of the plane per block: 32-bit index math, one division.
__global__ __launch_bounds__(256)
void maxpool_kernel(const float* __restrict__ in, float* __restrict__ out, int H, int W, int ksz,
                    int stride, int P, int Q, int planes) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= P * Q) return;
  const int p = o / Q, q = o - p * Q;
  for (long long nc = blockIdx.y; nc < planes; nc += gridDim.y) {
    const float* src = in + (size_t)nc * H * W + (size_t)(p * stride) * W + q * stride;
    float m = src[0];
    for (int r = 0; r < ksz; ++r)
      for (int s = 0; s < ksz; ++s) {
        float v = src[r * W + s];
        m = v > m ? v : m;
      }
    out[(size_t)nc * P * Q + o] = m;
  }
}

// The same for a window and stride fixed at compile time, PPT planes per thread: the
// KSZ*KSZ*PPT loads of a thread are independent and all in flight together, which is what
// a kernel with one load round trip per thread needs to approach the memory bandwidth.
template <int KSZ, int STRIDE, int PPT>
__global__ __launch_bounds__(256)
void maxpool_fixed_kernel(const float* __restrict__ in, float* __restrict__ out, int H, int W, int P,
                          int Q, int planes) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= P * Q) return;
  const int p = o / Q, q = o - p * Q;
  const size_t base = (size_t)(p * STRIDE) * W + q * STRIDE;
  for (long long nc0 = (long long)blockIdx.y * PPT; nc0 < planes; nc0 += (long long)gridDim.y * PPT) {
    float m[PPT];
#pragma unroll
    for (int u = 0; u < PPT; ++u) {
      const long long nc = nc0 + u < planes ? nc0 + u : planes - 1;   // tail: repeat the last plane
      const float* src = in + (size_t)nc * H * W + base;
      m[u] = src[0];
#pragma unroll
      for (int r = 0; r < KSZ; ++r)
#pragma unroll
        for (int s = 0; s < KSZ; ++s) {
          float v = src[r * W + s];
          m[u] = v > m[u] ? v : m[u];
        }
    }
#pragma unroll
    for (int u = 0; u < PPT; ++u)
      if (nc0 + u < planes) out[(size_t)(nc0 + u) * P * Q + o] = m[u];
  }
}

hipError_t launch_maxpool(const float* in, float* out, int N, int C, int H, int W, int ksz,
                          int stride, int P, int Q, hipStream_t st) {
  const long long planes = (long long)N * C;
  const unsigned gx = (unsigned)(((long long)P * Q + 255) / 256);
  if (ksz == 3 && stride == 2 && planes >= 1024) {
    constexpr int kPpt = 4;
    const long long groups = (planes + kPpt - 1) / kPpt;
    const unsigned gy = (unsigned)(groups < 65535 ? groups : 65535);
    return launch_kernel(maxpool_fixed_kernel<3, 2, kPpt>, dim3(gx, gy), dim3(256), 0, st, in, out, H,
                         W, P, Q, (int)planes);
  }
  const unsigned gy = (unsigned)(planes < 65535 ? planes : 65535);
  return launch_kernel(maxpool_kernel, dim3(gx, gy), dim3(256), 0, st, in, out, H, W, ksz, stride, P,
                       Q, (int)planes);
}

// Register-only MFMA loop (no memory traffic in the loop): each wave issues
// iters * 16 v_mfma_f32_32x32x2_f32 on two independent accumulator tiles.  Used by the
// benchmark to report what the matrix pipes sustain on the machine at hand.
typedef float mfma_acc_t __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256)
void mfma_loop_kernel(float* __restrict__ out, int iters) {
  mfma_acc_t acc0, acc1;
  for (int i = 0; i < 16; ++i) { acc0[i] = 0.0f; acc1[i] = 0.0f; }
  const float a = 1.0f + (float)(threadIdx.x & 7), b = 0.5f + (float)(threadIdx.x & 3);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, a, acc1, 0, 0, 0);
    }
  }
  float s = 0.0f;
  for (int i = 0; i < 16; ++i) s += acc0[i] + acc1[i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

hipError_t launch_mfma_loop(float* out, int workgroups, int iters, hipStream_t st) {
  return launch_kernel(mfma_loop_kernel, dim3(workgroups), dim3(256), 0, st, out, iters);
}

}  // namespace bconv
