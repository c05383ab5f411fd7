// Tiled MFMA forward convolution for gfx950 (CDNA4), fp32 in / fp32 accumulate.
//
// One workgroup computes BM filters x BN consecutive output pixels.  The main
// loop has the shape of the paper's SGEMM template (Listing 1: barrier,
// cooperative global->local loads, barrier, unrolled local->register loads and
// multiply-adds) with the register-tile FMAs replaced by
// v_mfma_f32_32x32x2_f32 and the right-hand operand never materialised: as in
// the paper's tiled-convolution variant (Section VI) whole pieces of input rows
// are staged in LDS and the S kernel columns are S shifted LDS reads of the
// same staged row, so global traffic for the input is not multiplied by S.
// A 1x1 layer (the paper's k1conv case) is the same kernel with R = S = 1, the
// host having flattened each image to one row of H*W pixels.
//
// Reduction order inside a chunk of KR reduction rows kk = c*R + r: pairs of
// rows (2j, 2j+1) feed the two k-slices of one MFMA (lanes 0-31 carry row 2j,
// lanes 32-63 row 2j+1), kernel column s innermost.
#pragma once
#include <hip/hip_runtime.h>

#include "bconv_plan.h"

namespace bconv {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// R_/S_/STR_ > 0: compile-time kernel height / width / stride (tap offsets become
// instruction immediates); 0: taken from the argument block at run time, with
// S <= SMAX_GENERIC.
constexpr int SMAX_GENERIC = kSmaxGeneric;

template <int R_, int S_, int STR_, int WM, int WN, int MT, int NT, int KR, int EPT>
struct TconvCfg {
  static constexpr int NTHR = WM * WN * 64;
  static constexpr int BM = WM * MT * 32;
  static constexpr int BN = WN * NT * 32;
  static constexpr int SP = S_ > 0 ? S_ : SMAX_GENERIC;   // A columns per reduction row (bound)
  static constexpr int KRSP = KR * SP;
  static constexpr int APT = (BM * KRSP + NTHR - 1) / NTHR;  // filter words per thread per chunk
  static_assert(KR % 2 == 0, "reduction rows are consumed in pairs");
};

template <int R_, int S_, int STR_, int WM, int WN, int MT, int NT, int KR, int EPT>
__global__ __launch_bounds__(WM * WN * 64)
void tconv_mfma_kernel(const TconvParams p) {
  using Cfg = TconvCfg<R_, S_, STR_, WM, WN, MT, NT, KR, EPT>;
  constexpr int NTHR = Cfg::NTHR, BM = Cfg::BM, BN = Cfg::BN;
  constexpr int KRSP = Cfg::KRSP, APT = Cfg::APT;

  const int R = R_ > 0 ? R_ : p.R;
  const int S = S_ > 0 ? S_ : p.S;
  const int STR = STR_ > 0 ? STR_ : p.stride;
  const int KRS = KR * S;            // valid filter words per row per chunk
  const int ast = p.ast;
  const int plane = p.plane;
  const int phst = p.phst;

  extern __shared__ float smem[];
  const int abuf = BM * ast;
  const int bbuf = KR * plane;
  float* const As = smem;               // [2][BM][ast]
  float* const Bs = smem + 2 * abuf;    // [2][KR][nrows][rowst]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, h = lane >> 5;

  const PixTile t = pix_tile(blockIdx.x, BN, p.NPQ, p.Q);
  const int m0 = blockIdx.y * BM;

  // ---- per-thread staging cells of the input tile (fixed for the whole loop)
  int c_lds[EPT], c_goff[EPT], c_ih0[EPT];
  const int ncell = p.nrows * p.rowst;
#pragma unroll
  for (int i = 0; i < EPT; ++i) {
    int e = tid + i * NTHR;
    BCell c = b_cell(p, t, e < ncell ? e : 0, S, STR);
    c_lds[i] = e < ncell ? c.lds : -1;
    c_goff[i] = c.goff;
    c_ih0[i] = e < ncell ? c.ih0 : kNeverValid;
  }

  // ---- per-lane operand bases
  int laneB[NT], outoff[NT], colvalid[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    BLane bl = b_lane(p, t, (wn * NT + nt) * 32 + l32);
    laneB[nt] = bl.ldsbase + h * plane;
    outoff[nt] = bl.outoff;
    colvalid[nt] = bl.valid;
  }
  const int laneA = (wm * MT * 32 + l32) * ast + h * S;

  floatx16 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][nt][i] = 0.0f;

  const int z = blockIdx.z;
  const int ch_begin = z * p.chunks_per_split;
  int ch_end = ch_begin + p.chunks_per_split;
  if (ch_end > p.nchunks) ch_end = p.nchunks;

  float ra[APT];
  float rb[KR * EPT];

  auto load_chunk = [&](int ch) {
    const int kk0 = ch * KR;
    // filters: BM rows of KRS consecutive words starting at column kk0*S
    const int col0 = kk0 * S;
#pragma unroll
    for (int i = 0; i < APT; ++i) {
      int e = tid + i * NTHR;
      int m = e / KRSP;
      int j = e - m * KRSP;
      bool ok = (m < BM) && (j < KRS) && (m0 + m < p.K) && (col0 + j < p.CRS);
      float v = p.filt[ok ? (m0 + m) * p.CRS + col0 + j : 0];   // word 0 always exists
      ra[i] = ok ? v : 0.0f;
    }
    // input rows: one plane per reduction row kk = (c, r)
    int c = kk0 / R;
    int r = kk0 - c * R;
#pragma unroll
    for (int kl = 0; kl < KR; ++kl) {
      const bool rowok = (kk0 + kl) < p.CRrows;
      const int koff = c * p.HW + r * p.W;
#pragma unroll
      for (int i = 0; i < EPT; ++i) {
        bool ok = rowok && ((unsigned)(c_ih0[i] + r) < (unsigned)p.H);
        float v = p.in[ok ? c_goff[i] + koff : 0];
        rb[kl * EPT + i] = ok ? v : 0.0f;
      }
      if (++r == R) { r = 0; ++c; }
    }
  };

  auto store_chunk = [&](int buf) {
    float* A = As + buf * abuf;
    float* B = Bs + buf * bbuf;
#pragma unroll
    for (int i = 0; i < APT; ++i) {
      int e = tid + i * NTHR;
      int m = e / KRSP;
      int j = e - m * KRSP;
      if ((m < BM) && (j < KRS)) A[m * ast + j] = ra[i];
    }
#pragma unroll
    for (int kl = 0; kl < KR; ++kl)
#pragma unroll
      for (int i = 0; i < EPT; ++i)
        if (c_lds[i] >= 0) B[kl * plane + c_lds[i]] = rb[kl * EPT + i];
  };

  auto mfma_step = [&](const float* A, const float* B, int aoff, int boff) {
    float a[MT], b[NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) a[mt] = A[laneA + mt * 32 * ast + aoff];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) b[nt] = B[laneB[nt] + boff];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
  };

  auto compute_chunk = [&](int buf) {
    const float* A = As + buf * abuf;
    const float* B = Bs + buf * bbuf;
    if constexpr (S_ > 0 && STR_ > 0) {
#pragma unroll
      for (int j = 0; j < KR / 2; ++j)
#pragma unroll
        for (int s = 0; s < S_; ++s)
          mfma_step(A, B, 2 * j * S_ + s, 2 * j * plane + (s % STR_) * phst + s / STR_);
    } else {
      for (int j = 0; j < KR / 2; ++j) {
        int ph = 0, xq = 0;
        for (int s = 0; s < S; ++s) {
          mfma_step(A, B, 2 * j * S + s, 2 * j * plane + ph * phst + xq);
          if (++ph == STR) { ph = 0; ++xq; }
        }
      }
    }
  };

  if (ch_begin < ch_end) {
    load_chunk(ch_begin);
    store_chunk(0);
  }
  __syncthreads();
  int buf = 0;
  for (int ch = ch_begin; ch < ch_end; ++ch) {
    const bool more = (ch + 1) < ch_end;
    if (more) load_chunk(ch + 1);
    compute_chunk(buf);
    if (more) store_chunk(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // ---- epilogue: bias + optional ReLU + store (or raw partial sums for split-K)
  const bool split = p.nsplit > 1;
  float* const dst = split ? p.partial + (size_t)z * (size_t)p.out_elems : p.out;
  float bvals[MT][16];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int k = m0 + (wm * MT + mt) * 32 + acc_row_32(lane, i);
      const bool ok = !split && p.bias && (k < p.K);
      const float v = (p.bias ? p.bias : p.filt)[ok ? k : 0];
      bvals[mt][i] = ok ? v : 0.0f;
    }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int k = m0 + (wm * MT + mt) * 32 + acc_row_32(lane, i);
      if (k < p.K) {
        const float bv = bvals[mt][i];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          if (colvalid[nt]) {
            float v = acc[mt][nt][i] + bv;
            if (!split && p.relu) v = v > 0.0f ? v : 0.0f;
            dst[outoff[nt] + k * p.PQ] = v;
          }
        }
      }
    }
  }
}

}  // namespace bconv
