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
//
// Staging is software-pipelined by hand: while chunk i is consumed from one LDS
// buffer, the global loads of chunk i+1 are issued between the MFMAs of the
// first half of the chunk and their LDS stores (into the other buffer) between
// the MFMAs of the second half, so that a single wave per SIMD keeps the matrix
// pipe fed; one barrier per chunk.
#pragma once
#include <hip/hip_runtime.h>

#include "bconv_plan.h"

namespace bconv {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// R_/S_/STR_ > 0: compile-time kernel height / width / stride (tap offsets become
// instruction immediates); 0: taken from the argument block at run time, with
// S <= kSmaxGeneric.  AV = 4: filter rows are fetched with 16-byte loads (the host
// guarantees CRS % 4 == 0, a 16-byte aligned filter pointer, and KR*S % 4 == 0
// holds by construction); AV = 1: 4-byte loads, no alignment demand.
template <int R_, int S_, int STR_, int WM, int WN, int MT, int NT, int KR, int EPT, int AV>
__global__ __launch_bounds__(WM * WN * 64)
void tconv_mfma_kernel(const TconvParams p) {
  constexpr int NTHR = WM * WN * 64;
  constexpr int BM = WM * MT * 32, BN = WN * NT * 32;
  constexpr int SP = S_ > 0 ? S_ : kSmaxGeneric;   // filter columns per reduction row (bound)
  constexpr int KRSP = KR * SP;
  static_assert(KR % 2 == 0, "reduction rows are consumed in pairs");
  static_assert(AV == 1 || (AV == 4 && S_ > 0 && KRSP % 4 == 0), "vector filter loads need KR*S % 4 == 0");
  constexpr int AGRP = KRSP / AV;                      // load groups per filter row
  constexpr int NA = (BM * AGRP + NTHR - 1) / NTHR;    // filter load items per thread
  constexpr int NB = KR * EPT;                         // input load items per thread
  constexpr int NL = NA + NB;

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
  float* const trash = Bs + 2 * bbuf;   // kLdsTrashWords words nobody reads

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

  float ra[NA * AV];
  float rb[NB];

  // Load item q of chunk ch: q < NA is a group of AV filter words, otherwise the
  // input cell (kl, i) = ((q - NA) / EPT, (q - NA) % EPT).
  auto load_item = [&](int ch, int q) {
    const int kk0 = ch * KR;
    if (q < NA) {
      const int col0 = kk0 * S;
      const int e = tid + q * NTHR;
      const int m = e / AGRP;
      const int j = (e - m * AGRP) * AV;
      const bool ok = (m < BM) && (j < KRS) && (m0 + m < p.K) && (col0 + j < p.CRS);
      const float* src = p.filt + (ok ? (m0 + m) * p.CRS + col0 + j : 0);   // word 0 always exists
      if constexpr (AV == 4) {
        floatx4 v = *reinterpret_cast<const floatx4*>(src);
#pragma unroll
        for (int u = 0; u < 4; ++u) ra[q * 4 + u] = ok ? v[u] : 0.0f;
      } else {
        float v = *src;
        ra[q] = ok ? v : 0.0f;
      }
    } else {
      const int kl = (q - NA) / EPT, i = (q - NA) % EPT;
      const int kk = kk0 + kl;
      const int c = kk / R;
      const int r = kk - c * R;
      const bool ok = (kk < p.CRrows) && ((unsigned)(c_ih0[i] + r) < (unsigned)p.H);
      float v = p.in[ok ? c_goff[i] + c * p.HW + r * p.W : 0];
      rb[q - NA] = ok ? v : 0.0f;
    }
  };

  auto store_item = [&](int buf, int q) {
    if (q < NA) {
      float* A = As + buf * abuf;
      const int e = tid + q * NTHR;
      const int m = e / AGRP;
      const int j = (e - m * AGRP) * AV;
      // words outside the tile go to the trash words behind the buffers, so that
      // the store needs no branch
      const bool ok = (m < BM) && (j < KRS);
      float* dst = ok ? A + m * ast + j : trash;
#pragma unroll
      for (int u = 0; u < AV; ++u) dst[u] = ra[q * AV + u];
    } else {
      float* B = Bs + buf * bbuf;
      const int kl = (q - NA) / EPT, i = (q - NA) % EPT;
      float* dst = c_lds[i] >= 0 ? B + kl * plane + c_lds[i] : trash;
      *dst = rb[q - NA];
    }
  };

  auto read_operands = [&](const float* A, const float* B, int aoff, int boff, float (&a)[MT],
                           float (&b)[NT]) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) a[mt] = A[laneA + mt * 32 * ast + aoff];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) b[nt] = B[laneB[nt] + boff];
  };
  auto mfma_tile = [&](const float (&a)[MT], const float (&b)[NT]) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
  };

  // Consumes LDS buffer `buf`; with STAGE also fetches chunk `next` into buf ^ 1.
  auto compute_chunk = [&](int buf, int next, auto stage_tag) {
    constexpr bool STAGE = decltype(stage_tag)::value;
    const float* A = As + buf * abuf;
    const float* B = Bs + buf * bbuf;
    if constexpr (S_ > 0 && STR_ > 0) {
      constexpr int NSTEPS = (KR / 2) * S_;
      constexpr int LSTEPS = NSTEPS > 1 ? (NSTEPS + 1) / 2 : 1;   // loads issued in steps [0, LSTEPS)
      constexpr int SSTEPS = NSTEPS - LSTEPS;                     // stores in steps [LSTEPS, NSTEPS)
      // operands of step st+1 are read from LDS before the MFMAs of step st issue
      float a[2][MT], b[2][NT];
      read_operands(A, B, 0, 0, a[0], b[0]);
#pragma unroll
      for (int st = 0; st < NSTEPS; ++st) {
        if (st + 1 < NSTEPS) {
          const int j = (st + 1) / S_, s = (st + 1) % S_;
          read_operands(A, B, 2 * j * S_ + s, 2 * j * plane + (s % STR_) * phst + s / STR_,
                        a[(st + 1) & 1], b[(st + 1) & 1]);
        }
        mfma_tile(a[st & 1], b[st & 1]);
        if constexpr (STAGE) {
#pragma unroll
          for (int q = 0; q < NL; ++q) {
            if (q * LSTEPS / NL == st) load_item(next, q);
            if (SSTEPS > 0 && LSTEPS + q * SSTEPS / NL == st) store_item(buf ^ 1, q);
          }
        }
      }
      if constexpr (STAGE && SSTEPS == 0) {
#pragma unroll
        for (int q = 0; q < NL; ++q) store_item(buf ^ 1, q);
      }
    } else {
      if constexpr (STAGE) {
#pragma unroll
        for (int q = 0; q < NL; ++q) load_item(next, q);
      }
      for (int j = 0; j < KR / 2; ++j) {
        int ph = 0, xq = 0;
        for (int s = 0; s < S; ++s) {
          float a[MT], b[NT];
          read_operands(A, B, 2 * j * S + s, 2 * j * plane + ph * phst + xq, a, b);
          mfma_tile(a, b);
          if (++ph == STR) { ph = 0; ++xq; }
        }
      }
      if constexpr (STAGE) {
#pragma unroll
        for (int q = 0; q < NL; ++q) store_item(buf ^ 1, q);
      }
    }
  };

  if (ch_begin < ch_end) {
#pragma unroll
    for (int q = 0; q < NL; ++q) load_item(ch_begin, q);
#pragma unroll
    for (int q = 0; q < NL; ++q) store_item(0, q);
  }
  __syncthreads();
  int buf = 0;
  for (int ch = ch_begin; ch + 1 < ch_end; ++ch) {
    compute_chunk(buf, ch + 1, std::true_type{});
    __syncthreads();
    buf ^= 1;
  }
  if (ch_begin < ch_end) compute_chunk(buf, 0, std::false_type{});

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
