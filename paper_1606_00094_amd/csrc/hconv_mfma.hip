// Half-precision convolution on the fp16 matrix cores (v_mfma_f32_32x32x16_f16): the second
// stage of the paper's Section VII outlook (smaller storage types, here with the matrix
// arithmetic in that type too: fp16 x fp16 products are exact in fp32 and the sums are fp32,
// so the contract of the fp32-arithmetic path -- exact products, fp32 accumulation, one
// rounding to fp16 after bias and ReLU -- is unchanged).  Stride-1 layers with a 1x1, 3x3 or
// 5x5 kernel and a channel count that is a multiple of eight; everything else stays on the
// tiled kernel that widens to fp32.
//
// One MFMA consumes 16 reduction elements; lanes 0-31 carry eight of them, lanes 32-63 the other
// eight, as one 16-byte register quad per operand.  The reduction is therefore ordered
// (kernel row, kernel column, channel) with the channel innermost, and both operands are held
// in LDS as "octets" -- eight consecutive channels of one filter tap, or of one input position,
// in 16 bytes -- so that every operand read is one ds_read_b128:
//   * filters: re-laid once per call by a small kernel from KCRS into
//     [filter][chunk][tap][CC channels] (CC channels per staged chunk, zero beyond C), from
//     where a workgroup's rows of a chunk are contiguous 16-byte units;
//   * input: the tile's halo (every padded input position its pixels touch, as in the fp32
//     kernel's halo staging) is staged per chunk position by position: a thread gathers the
//     eight channels of one position from the NCHW planes (each of the eight loads is
//     coalesced over the positions of a wave), packs them and writes one octet.  The kernel
//     taps are then offsets of the LDS read, uniform over the lanes.
// Software pipeline: the global loads of chunk i+1 are in flight while chunk i is multiplied
// out of one LDS buffer, and are written to the other buffer afterwards; one barrier per chunk.
//
// Activations come in one of two layouts: NCHW, or "C8" = [N][C/8][H][W][8], eight consecutive
// channels of a pixel in 16 contiguous bytes.  C8 is the layout the staging wants (one 16-byte
// load per octet instead of eight 2-byte loads from eight planes) and the one the accumulator
// layout stores well (8-byte stores instead of 2-byte ones), so layers chained in half
// precision keep their activations in it.  This file is compiled once per layout pair
// (HCONV_LAYOUT 0: NCHW in and out; 1: C8 in, NCHW out; 2: C8 in and out); unit 0 also holds
// the host side.
#include <atomic>
#include <cstdint>
#include <cstring>

#include "bconv_internal.h"

#ifndef HCONV_LAYOUT
#define HCONV_LAYOUT 0
#endif
#ifndef HCONV_PF
#define HCONV_PF 2
#endif

namespace bconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float hacc_t __attribute__((ext_vector_type(16)));
typedef unsigned uquad __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

struct HconvParams {
  TconvParams g;            // shape and halo geometry; g.in / g.out address _Float16 elements
  const _Float16* filt2;    // re-laid filters [K][nch][taps][CC]
  int nch;                  // chunks of CC channels
  int npos;                 // staged positions per octet plane
  int coct;                 // C / 8
  int nsplit, cps;          // reduction split over the grid's z: chunks [z*cps, z*cps+cps) each
  float* partial;           // nsplit > 1: fp32 partial sums [nsplit][out_elems], indexed like out
};

// TR: kernel rows of a chunk's filters staged at a time (R_: the whole chunk in one stage; 1: a
// stage per kernel row, which cuts the filters' LDS footprint R_-fold -- what lets a 5x5 tile of
// 64 or 128 filters leave room for several workgroups per compute unit).  The input halo of a
// chunk is staged once and serves all its stages.
template <int R_, int S_, int WM, int WN, int MT, int NT, int CC, int EPB, int TR, bool C8I, bool C8O>
__global__ __launch_bounds__(WM * WN * 64)
void hconv_mfma_kernel(const HconvParams hp) {
  static_assert(R_ % TR == 0, "stages are whole kernel rows");
  constexpr int NTHR = WM * WN * 64;
  constexpr int BM = WM * MT * 32, BN = WN * NT * 32;
  constexpr int TAPS = R_ * S_;
  constexpr int NRS = R_ / TR;            // stages per chunk
  constexpr int STAPS = TR * S_;          // taps per stage
  constexpr int NOCT = CC / 8;            // octets per position (or tap) and chunk
  constexpr int NJ = CC / 16;             // MFMAs per tap and chunk
  constexpr int FROW = TAPS * NOCT;       // 16-byte units per filter row and chunk (packed filters)
  constexpr int AROW = STAPS * NOCT;      // ... and stage
  constexpr int AST = AROW | 1;           // LDS row stride (odd: rows spread over the banks)
  constexpr int NA = (BM * AROW + NTHR - 1) / NTHR;
  constexpr bool PW = (R_ == 1 && S_ == 1);
  static_assert(CC % 16 == 0, "a chunk is a whole number of MFMAs");
  const TconvParams& p = hp.g;
  const int npos = hp.npos;

  extern __shared__ __attribute__((aligned(16))) uquad hsm[];
  uquad* const As = hsm;                           // [2][BM][AST]
  uquad* const Bs = hsm + 2 * BM * AST;            // [2][NOCT][npos]
  const int abuf = BM * AST, bbuf = NOCT * npos;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, gq = lane >> 5;

  const BlockTile bt = xcd_tile(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), gridDim.x,
                                gridDim.y, gridDim.z, p.filter_major);
  const int ch_begin = bt.z * hp.cps;
  const int ch_end = ch_begin + hp.cps < hp.nch ? ch_begin + hp.cps : hp.nch;   // (host: ch_begin < nch)
  const PixTile t = pix_tile(bt.x, BN, p.NPQ, p.Q, p.fdQ);
  const HaloTile ht = PW ? HaloTile{0, 0} : halo_tile(p, t);
  const int m0 = bt.y * BM;
  constexpr unsigned kOob = 0x80000000u;

  // ---- input staging items of this thread: (octet o, position pos), fixed for the whole loop
  unsigned b_voff[EPB];
  int b_lds[EPB], b_oct[EPB];
#pragma unroll
  for (int i = 0; i < EPB; ++i) {
    int e = tid + i * NTHR;
    int o = 0;
    while (o < NOCT && e >= npos) { e -= npos; ++o; }
    const bool item = o < NOCT;
    int goff = 0;
    bool ok = item;
    if (PW) {
      // compact: position = pixel of the tile; a flattened image is one row of H*W pixels
      ok = ok && (e < t.cnt);
      const int gp = t.g0 + (ok ? e : 0);
      const int img = fd_div(gp, p.fdQ);
      goff = img * p.CHW + (gp - img * p.Q);
    } else {
      BCell c = h_cell(p, ht, item ? e : 0, 1);
      ok = ok && (c.ih0 != kNeverValid);
      goff = c.goff;
    }
    b_oct[i] = item ? o : NOCT;                    // NOCT: no item (never loads, stores nowhere)
    b_lds[i] = item ? o * npos + e : 0;
    if (C8I) {
      // octet-interleaved input [N][C/8][H*W][8]: the octet of a position is 16 contiguous bytes
      const int hw = ok ? (int)((unsigned)goff % (unsigned)p.CHW) : 0;
      b_voff[i] = ok ? (unsigned)((goff + 7 * hw + o * 8 * p.HW) * 2) : kOob;
    } else {
      b_voff[i] = ok ? (unsigned)((goff + o * 8 * p.HW) * 2) : kOob;
    }
  }
  // ---- filter staging items: 16-byte unit j of filter row m
  unsigned a_voff[NA];
  int a_lds[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int e = tid + i * NTHR;
    const int m = e / AROW, j = e - m * AROW;
    const bool ok = (e < BM * AROW) && (m0 + m < p.K);
    a_voff[i] = ok ? (unsigned)((((m0 + m) * hp.nch) * FROW + j) * 16) : kOob;
    a_lds[i] = (e < BM * AROW) ? m * AST + j : -1;
  }
  const __amdgpu_buffer_rsrc_t rsrc_in = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(p.in), 0, p.N * p.CHW * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_f = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<_Float16*>(hp.filt2), 0, p.K * hp.nch * FROW * 16, 0x00020000);

  // ---- per-lane operand bases (16-byte units)
  const int laneA = (wm * MT * 32 + l32) * AST + gq;
  int laneB[NT], outoff[NT], colvalid[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int col = (wn * NT + nt) * 32 + l32;
    if (PW) {
      const bool v = col < t.cnt;
      const int cc = v ? col : t.cnt - 1;
      const int gp = t.g0 + cc;
      const int img = fd_div(gp, p.fdQ);
      laneB[nt] = cc + gq * npos;
      outoff[nt] = img * p.K * p.PQ + (gp - img * p.Q);
      colvalid[nt] = v;
    } else {
      BLane bl = h_lane(p, t, ht, col);
      laneB[nt] = bl.ldsbase + gq * npos;
      outoff[nt] = bl.outoff;
      colvalid[nt] = bl.valid;
    }
  }

  if (C8O) {
    // octet-interleaved output [N][K/8][P*Q][8]: pixel pq of image img starts at
    // img*K*PQ + pq*8 (+ 8*PQ per octet of filters); this lane's half of an octet follows
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int kpq = p.K * p.PQ;
      const int img = (int)((unsigned)outoff[nt] / (unsigned)kpq);
      const int pq = outoff[nt] - img * kpq;
      outoff[nt] = img * kpq + pq * 8 + gq * 4;
    }
  }

  hacc_t acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][nt][i] = 0.0f;

  uquad ra[NA];
  unsigned short rb[C8I ? 1 : EPB][8];
  uquad rq[C8I ? EPB : 1];
  // filters of stage rr of chunk ch
  auto load_a = [&](int ch, int rr) {
#pragma unroll
    for (int i = 0; i < NA; ++i)
      ra[i] = __builtin_bit_cast(uquad, __builtin_amdgcn_raw_buffer_load_b128(rsrc_f, a_voff[i],
                                                                              (ch * FROW + rr * AROW) * 16, 0));
  };
  // input halo of chunk ch
  auto load_b = [&](int ch) {
#pragma unroll
    for (int i = 0; i < EPB; ++i) {
      // an octet past the last channel reads nothing (C is a multiple of eight)
      const unsigned voff = (ch * NOCT + b_oct[i] < hp.coct) ? b_voff[i] : kOob;
      if constexpr (C8I) {
        rq[i] = __builtin_bit_cast(uquad, __builtin_amdgcn_raw_buffer_load_b128(rsrc_in, voff, ch * CC * p.HW * 2, 0));
      } else {
#pragma unroll
        for (int u = 0; u < 8; ++u)
          rb[i][u] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rsrc_in, voff, (ch * CC + u) * p.HW * 2, 0);
      }
    }
  };
  auto store_a = [&](int buf) {
    uquad* A = As + buf * abuf;
#pragma unroll
    for (int i = 0; i < NA; ++i)
      if (a_lds[i] >= 0) A[a_lds[i]] = ra[i];
  };
  auto store_b = [&](int buf) {
    uquad* B = Bs + buf * bbuf;
#pragma unroll
    for (int i = 0; i < EPB; ++i) {
      if (b_oct[i] < NOCT) {
        if constexpr (C8I) {
          B[b_lds[i]] = rq[i];
        } else {
          uquad v;
#pragma unroll
          for (int w = 0; w < 4; ++w) v[w] = (unsigned)rb[i][2 * w] | ((unsigned)rb[i][2 * w + 1] << 16);
          B[b_lds[i]] = v;
        }
      }
    }
  };
  // One stage out of filter buffer abuf_i and input buffer bbuf_i.  Operand reads run HCONV_PF
  // steps (a step is one MFMA depth of one tap) ahead of the MFMAs that use them: the reads of
  // step s+PF are issued, then the MFMAs of step s, and the scheduler may not move anything
  // across a step boundary, so a wave's LDS latency hides behind its own MFMAs.  (Measured: two
  // steps ahead 1-5 % over one, three no better.)
  auto compute_stage = [&](int abuf_i, int bbuf_i, int rr) {
    const uquad* A = As + abuf_i * abuf;
    const uquad* B = Bs + bbuf_i * bbuf + (PW ? 0 : rr * TR * p.rowst);
    constexpr int STEPS = STAPS * NJ;
    constexpr int PF = HCONV_PF < STEPS ? HCONV_PF : (STEPS > 1 ? STEPS - 1 : 1);   // steps read ahead
    constexpr int NS = PF + 1;
    half8 a[NS][MT], b[NS][NT];
    auto read_step = [&](int s, int slot) {
      const int tap = s / NJ, jj = s % NJ;
      const int toff = PW ? 0 : (tap / S_) * p.rowst + (tap % S_);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        a[slot][mt] = __builtin_bit_cast(half8, A[laneA + mt * 32 * AST + tap * NOCT + 2 * jj]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        b[slot][nt] = __builtin_bit_cast(half8, B[laneB[nt] + 2 * jj * npos + toff]);
    };
#pragma unroll
    for (int s = 0; s < PF && s < STEPS; ++s) read_step(s, s % NS);
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      if (s + PF < STEPS) read_step(s + PF, (s + PF) % NS);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[s % NS][mt], b[s % NS][nt], acc[mt][nt], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Stage it = ch * NRS + rr multiplies out of filter buffer it & 1 and input buffer ch & 1 while
  // the loads of stage it + 1 (its filters; at the first stage of a chunk also the next chunk's
  // halo) are in flight; they are written to the other buffers afterwards, the halo at the
  // chunk's last stage.  One barrier per stage.
  load_a(ch_begin, 0);
  load_b(ch_begin);
  store_a(0);
  store_b(ch_begin & 1);
  __syncthreads();
  {
    int ch = ch_begin, rr = 0;
    const int nstages = (ch_end - ch_begin) * NRS;
    for (int it = 0; it < nstages; ++it) {
      const bool more = it + 1 < nstages;
      const bool last_of_chunk = rr == NRS - 1;
      const bool more_ch = ch + 1 < ch_end;
      if (more) load_a(last_of_chunk ? ch + 1 : ch, last_of_chunk ? 0 : rr + 1);
      if (rr == 0 && more_ch) load_b(ch + 1);
      __builtin_amdgcn_sched_barrier(0);   // the loads are in flight before the first operand read
      compute_stage(it & 1, ch & 1, rr);
      if (more) store_a((it + 1) & 1);
      if (last_of_chunk && more_ch) store_b((ch + 1) & 1);
      __syncthreads();
      if (last_of_chunk) { rr = 0; ++ch; } else { ++rr; }
    }
  }

  // ---- a split reduction: this workgroup's fp32 partial sums, in the output's own index order
  // (the reduction kernel adds the splits, the bias and the ReLU and rounds once)
  if (hp.nsplit > 1) {
    float* const part = hp.partial + (size_t)bt.z * p.out_elems;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      if constexpr (C8O) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int k = m0 + (wm * MT + mt) * 32 + g * 8 + gq * 4;
          if (k < p.K) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
              if (colvalid[nt]) {
                floatx4 v;
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = acc[mt][nt][4 * g + j];
                *reinterpret_cast<floatx4*>(part + outoff[nt] + (k - gq * 4) * p.PQ) = v;
              }
            }
          }
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int k = m0 + (wm * MT + mt) * 32 + acc_row_32(lane, i);
          if (k < p.K) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              if (colvalid[nt]) part[outoff[nt] + k * p.PQ] = acc[mt][nt][i];
          }
        }
      }
    }
    return;
  }

  // ---- epilogue: bias + optional ReLU, one rounding to fp16, store
  _Float16* const out = reinterpret_cast<_Float16*>(p.out);
  if constexpr (C8O) {
    // accumulator registers 4g .. 4g+3 of a lane are four consecutive filters (half an octet)
    // of one pixel: one 8-byte store; the two lane halves complete the octet, so a wave's
    // store covers 32 pixels x 16 contiguous bytes.  K is a multiple of eight here.
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int k = m0 + (wm * MT + mt) * 32 + g * 8 + gq * 4;
        if (k < p.K) {
          float bv[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) bv[j] = p.bias ? p.bias[k + j] : 0.0f;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            if (colvalid[nt]) {
              half4 h;
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                float v = acc[mt][nt][4 * g + j] + bv[j];
                if (p.relu) v = v > 0.0f ? v : 0.0f;
                h[j] = (_Float16)v;
              }
              *reinterpret_cast<half4*>(out + outoff[nt] + (k - gq * 4) * p.PQ) = h;
            }
          }
        }
      }
    }
  } else {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int k = m0 + (wm * MT + mt) * 32 + acc_row_32(lane, i);
        if (k < p.K) {
          const float bv = p.bias ? p.bias[k] : 0.0f;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            if (colvalid[nt]) {
              float v = acc[mt][nt][i] + bv;
              if (p.relu) v = v > 0.0f ? v : 0.0f;
              out[outoff[nt] + k * p.PQ] = (_Float16)v;
            }
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------ catalogue and planning
struct HTile {
  const char* name;
  int R, S, WM, WN, MT, NT, CC, EPB, TR;
  int BM() const { return WM * MT * 32; }
  int BN() const { return WN * NT * 32; }
  int NTHR() const { return WM * WN * 64; }
};
#define HCONV_TILES(X) \
  X(h16k3_128x128_c16, 3, 3, 2, 2, 2, 2, 16, 3, 3) \
  X(h16k3_64x128_c16, 3, 3, 2, 2, 1, 2, 16, 3, 3) \
  X(h16k3_128x64_c16, 3, 3, 2, 2, 2, 1, 16, 2, 3) \
  X(h16k3_64x64_c16, 3, 3, 2, 2, 1, 1, 16, 2, 3) \
  X(h16k3_64x128_c32, 3, 3, 2, 2, 1, 2, 32, 6, 3) \
  X(h16k5_64x128_c16, 5, 5, 2, 2, 1, 2, 16, 4, 5) \
  X(h16k5_64x64_c16, 5, 5, 2, 2, 1, 1, 16, 3, 5) \
  X(h16k5_32x128_c16, 5, 5, 1, 4, 1, 1, 16, 4, 5) \
  X(h16pw_128x128_c32, 1, 1, 2, 2, 2, 2, 32, 2, 1) \
  X(h16pw_64x128_c32, 1, 1, 2, 2, 1, 2, 32, 2, 1) \
  X(h16pw_128x64_c32, 1, 1, 2, 2, 2, 1, 32, 1, 1) \
  X(h16pw_64x64_c32, 1, 1, 2, 2, 1, 1, 32, 1, 1) \
  X(h16pw_64x64_c64, 1, 1, 2, 2, 1, 1, 64, 2, 1) \
  X(h16k3_32x128_c16, 3, 3, 1, 4, 1, 1, 16, 3, 3) \
  X(h16k3_32x64_c16, 3, 3, 1, 2, 1, 1, 16, 4, 3) \
  X(h16k3_64x64_c32, 3, 3, 2, 2, 1, 1, 32, 4, 3) \
  X(h16pw_32x128_c64, 1, 1, 1, 4, 1, 1, 64, 4, 1) \
  X(h16pw_32x64_c64, 1, 1, 1, 2, 1, 1, 64, 4, 1) \
  X(h16pw_64x32_c64, 1, 1, 2, 1, 1, 1, 64, 2, 1) \
  X(h16k3_128x256_c16, 3, 3, 2, 4, 2, 2, 16, 3, 3) \
  X(h16pw_128x256_c32, 1, 1, 2, 4, 2, 2, 32, 2, 1) \
  X(h16k5_64x256_c16, 5, 5, 2, 4, 1, 2, 16, 3, 5) \
  X(h16k5_64x256_c16r1, 5, 5, 2, 4, 1, 2, 16, 3, 1) \
  X(h16k5_128x256_c16r1, 5, 5, 2, 4, 2, 2, 16, 3, 1) \
  X(h16k5_64x128_c16r1, 5, 5, 2, 2, 1, 2, 16, 4, 1) \
  X(h16k5_32x128_c16r1, 5, 5, 1, 4, 1, 1, 16, 4, 1)

typedef hipError_t (*HLaunchFn)(const HconvParams&, dim3, size_t, hipStream_t);
// One launch table per layout pair, each held by its own translation unit.
HLaunchFn hconv_launch_l0(int which);
HLaunchFn hconv_launch_l1(int which);
HLaunchFn hconv_launch_l2(int which);

// (dynamic LDS above the default limit must be allowed per kernel and device; the largest
// request so far is remembered, host threads may race on it harmlessly)
template <typename KernelT>
static hipError_t launch_h(KernelT kernel, int nthr, const HconvParams& hp, dim3 grid, size_t lds, hipStream_t st,
                           std::atomic<size_t>* allowed) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (lds > 32768 && lds > allowed[dev].load(std::memory_order_relaxed)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds);
    if (e != hipSuccess) { (void)hipGetLastError(); return e; }
    allowed[dev].store(lds, std::memory_order_relaxed);
  }
  return launch_kernel(kernel, grid, dim3(nthr), lds, st, hp);
}
#if HCONV_LAYOUT == 0
#define HCONV_TABLE hconv_launch_l0
#define HCONV_C8I false
#define HCONV_C8O false
#elif HCONV_LAYOUT == 1
#define HCONV_TABLE hconv_launch_l1
#define HCONV_C8I true
#define HCONV_C8O false
#else
#define HCONV_TABLE hconv_launch_l2
#define HCONV_C8I true
#define HCONV_C8O true
#endif
#define X(name, R, S, WM, WN, MT, NT, CC, EPB, TR)                                                    \
  static hipError_t hlaunch_##name(const HconvParams& hp, dim3 grid, size_t lds, hipStream_t st) {    \
    static std::atomic<size_t> allowed[64];                                                           \
    return launch_h(hconv_mfma_kernel<R, S, WM, WN, MT, NT, CC, EPB, TR, HCONV_C8I, HCONV_C8O>, WM * WN * 64, hp,  \
                    grid, lds, st, allowed);                                                          \
  }
HCONV_TILES(X)
#undef X
HLaunchFn HCONV_TABLE(int which) {
  static const HLaunchFn table[] = {
#define X(name, R, S, WM, WN, MT, NT, CC, EPB, TR) hlaunch_##name,
      HCONV_TILES(X)
#undef X
  };
  return table[which];
}

#if HCONV_LAYOUT == 0
// filt KCRS (fp16) -> [K][nch][R*S][CC], zeros for channels past C
__global__ __launch_bounds__(256)
void hconv_repack_kernel(const _Float16* __restrict__ filt, _Float16* __restrict__ filt2, int K, int C,
                         int taps, int CC, int nch, long long total) {
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int cc = (int)(idx % CC);
    long long r = idx / CC;
    const int tap = (int)(r % taps);
    r /= taps;
    const int ch = (int)(r % nch);
    const int k = (int)(r / nch);
    const int c = ch * CC + cc;
    filt2[idx] = c < C ? filt[((long long)k * C + c) * taps + tap] : (_Float16)0.0f;
  }
}

// NCHW -> C8: one thread per (image, octet, pixel) gathers eight planes and writes 16 bytes
__global__ __launch_bounds__(256)
void f16_nchw_to_c8_kernel(const _Float16* __restrict__ in, uquad* __restrict__ out, int HW, long long total) {
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const long long no = idx / HW;                 // image * C/8 + octet
    const int hw = (int)(idx - no * HW);
    const unsigned short* src = reinterpret_cast<const unsigned short*>(in) + no * 8 * HW + hw;
    uquad v;
#pragma unroll
    for (int w = 0; w < 4; ++w)
      v[w] = (unsigned)src[(size_t)(2 * w) * HW] | ((unsigned)src[(size_t)(2 * w + 1) * HW] << 16);
    out[idx] = v;
  }
}

// C8 -> NCHW
__global__ __launch_bounds__(256)
void f16_c8_to_nchw_kernel(const uquad* __restrict__ in, _Float16* __restrict__ out, int HW, long long total) {
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const long long no = idx / HW;
    const int hw = (int)(idx - no * HW);
    const uquad v = in[idx];
    unsigned short* dst = reinterpret_cast<unsigned short*>(out) + no * 8 * HW + hw;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      dst[(size_t)(2 * w) * HW] = (unsigned short)(v[w] & 0xffffu);
      dst[(size_t)(2 * w + 1) * HW] = (unsigned short)(v[w] >> 16);
    }
  }
}

// Max pooling of fp16 activations (window ksz, step `stride`, no padding, floor extents).
// C8: one thread per (image, octet, pooled pixel) reads its window as 16-byte octets and keeps
// the eight running maxima; NCHW: one thread per pooled element.  A maximum of fp16 values is
// one of them, so there is no rounding.
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
__global__ __launch_bounds__(256)
void maxpool_f16_c8_kernel(const half8v* __restrict__ in, half8v* __restrict__ out, int H, int W, int P, int Q,
                           int ksz, int stride, long long total) {
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int q = (int)(idx % Q);
    long long r = idx / Q;
    const int pp = (int)(r % P);
    const long long no = r / P;
    const half8v* src = in + (no * H + (long long)pp * stride) * W + (long long)q * stride;
    half8v m = src[0];
    for (int y = 0; y < ksz; ++y)
      for (int x = 0; x < ksz; ++x) {
        const half8v v = src[(long long)y * W + x];
#pragma unroll
        for (int u = 0; u < 8; ++u) m[u] = v[u] > m[u] ? v[u] : m[u];
      }
    out[idx] = m;
  }
}

__global__ __launch_bounds__(256)
void maxpool_f16_nchw_kernel(const _Float16* __restrict__ in, _Float16* __restrict__ out, int H, int W, int P,
                             int Q, int ksz, int stride, long long total) {
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int q = (int)(idx % Q);
    long long r = idx / Q;
    const int pp = (int)(r % P);
    const long long nc = r / P;
    const _Float16* src = in + (nc * H + (long long)pp * stride) * W + (long long)q * stride;
    _Float16 m = src[0];
    for (int y = 0; y < ksz; ++y)
      for (int x = 0; x < ksz; ++x) {
        const _Float16 v = src[(long long)y * W + x];
        m = v > m ? v : m;
      }
    out[idx] = m;
  }
}

hipError_t launch_maxpool_f16(const void* in, void* out, long long n_times_c, int H, int W, int ksz, int stride,
                              int P, int Q, int c8, hipStream_t st) {
  const long long total = (c8 ? n_times_c / 8 : n_times_c) * P * Q;
  if (total == 0) return hipSuccess;
  long long blocks = (total + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (c8)
    return launch_kernel(maxpool_f16_c8_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                         static_cast<const half8v*>(in), static_cast<half8v*>(out), H, W, P, Q, ksz, stride, total);
  return launch_kernel(maxpool_f16_nchw_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       static_cast<const _Float16*>(in), static_cast<_Float16*>(out), H, W, P, Q, ksz, stride, total);
}

hipError_t launch_f16_layout(const void* in, void* out, long long n_times_c, int HW, int to_c8, hipStream_t st) {
  const long long total = n_times_c / 8 * HW;
  if (total == 0) return hipSuccess;
  long long blocks = (total + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (to_c8)
    return launch_kernel(f16_nchw_to_c8_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                         static_cast<const _Float16*>(in), static_cast<uquad*>(out), HW, total);
  return launch_kernel(f16_c8_to_nchw_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       static_cast<const uquad*>(in), static_cast<_Float16*>(out), HW, total);
}

static const HTile kHTiles[] = {
#define X(name, R, S, WM, WN, MT, NT, CC, EPB, TR) {#name, R, S, WM, WN, MT, NT, CC, EPB, TR},
    HCONV_TILES(X)
#undef X
};
constexpr int kNumHTiles = (int)(sizeof(kHTiles) / sizeof(kHTiles[0]));

// The catalogue of the fp16-matrix-core kernels: the channel-octet tiles of this file, each with
// the reduction splits of kHSplits (index = tile * kNumHSplits + split index), then the
// first-layer tiles (hconv_first.hip), which take NCHW activations and unpacked filters only.
static const int kHSplits[] = {1, 2, 3, 4, 6, 8};
constexpr int kNumHSplits = (int)(sizeof(kHSplits) / sizeof(kHSplits[0]));
constexpr int kNumOctet = kNumHTiles * kNumHSplits;
int hconv_num_variants() { return kNumOctet + hfl_num_variants(); }
const char* hconv_variant_name(int which) {
  return which < kNumOctet ? kHTiles[which / kNumHSplits].name : hfl_variant_name(which - kNumOctet);
}
int hconv_variant_split(int which) { return which < kNumOctet ? kHSplits[which % kNumHSplits] : 1; }
bool hconv_packable(int which) { return which >= 0 && which < kNumOctet; }

struct HPlan {
  HconvParams hp;
  unsigned gx, gy, gz;
  size_t lds_bytes;
  size_t filt2_bytes;
  size_t partial_bytes;     // 0 for an unsplit variant
};

static size_t h_align(size_t b) { return (b + 255) & ~(size_t)255; }

// `which` indexes the channel-octet part of the catalogue (tile and reduction split).
static bool plan_hconv(int which, const Shape& s0, HPlan* pl) {
  if (which < 0 || which >= kNumOctet) return false;
  const HTile& v = kHTiles[which / kNumHSplits];
  const int nsplit = kHSplits[which % kNumHSplits];
  Shape s = s0;
  if (s.R != v.R || s.S != v.S || s.stride != 1 || s.C % 8 != 0) return false;
  const long long i31 = (1LL << 31) - 1;
  if ((long long)s.N * s.C * s.H * s.W * 2 > i31 || (long long)s.N * s.K * s.P * s.Q > i31) return false;
  const bool pw = (s.R == 1 && s.S == 1);
  if (pw && s.pad != 0) return false;
  if (pw) {                        // per-image im2col is the identity: one row of H*W pixels
    s.W = s.H * s.W; s.H = 1; s.Q = s.P * s.Q; s.P = 1;
  }
  TconvParams& p = pl->hp.g;
  std::memset(&pl->hp, 0, sizeof(pl->hp));
  p.N = s.N; p.C = s.C; p.H = s.H; p.W = s.W; p.K = s.K; p.R = s.R; p.S = s.S;
  p.stride = 1; p.pad = s.pad; p.P = s.P; p.Q = s.Q;
  p.PQ = s.P * s.Q; p.NPQ = s.N * p.PQ; p.HW = s.H * s.W; p.CHW = s.C * p.HW;
  p.CRS = s.C * s.R * s.S; p.CRrows = s.C * s.R;
  p.out_elems = s.N * s.K * p.PQ;
  p.fdQ = make_fastdiv((unsigned)p.Q); p.fdP = make_fastdiv((unsigned)p.P);
  p.filter_major = (long long)s.K * s.C * s.R * s.S > (long long)s.N * s.C * s.H * s.W ? 1 : 0;
  p.halo = 1;
  p.hp = s.H + 2 * s.pad; p.wt = s.W + 2 * s.pad;
  p.phst = p.wt; p.rowst = p.wt;
  p.fdHp = make_fastdiv((unsigned)p.hp); p.fdRowst = make_fastdiv((unsigned)p.rowst);
  const int BN = v.BN(), BM = v.BM();
  const long long ntiles = ((long long)p.NPQ + BN - 1) / BN;
  if (ntiles > i31) return false;
  int npos = BN;
  if (!pw) {
    p.vr = 0;
    for (long long ti = 0; ti < ntiles; ++ti) {
      HaloTile h = halo_tile(p, pix_tile((int)ti, BN, p.NPQ, p.Q, p.fdQ));
      if (h.vr > p.vr) p.vr = h.vr;
    }
    p.nrows = p.vr;
    p.plane = p.nrows * p.rowst;
    npos = p.plane;
  }
  const int noct = v.CC / 8;
  if ((long long)noct * npos > (long long)v.EPB * v.NTHR()) return false;
  const int arow = v.R * v.S * noct;                 // per chunk (the packed filters)
  const int ast = (v.TR * v.S * noct) | 1;           // per stage (LDS row stride)
  const size_t lds = (size_t)16 * (2 * (size_t)BM * ast + 2 * (size_t)noct * npos);
  if (lds > kLdsLimitBytes) return false;
  pl->hp.nch = (s.C + v.CC - 1) / v.CC;
  pl->hp.npos = npos;
  pl->hp.coct = s.C / 8;
  pl->filt2_bytes = (size_t)s.K * pl->hp.nch * arow * 16;
  if ((long long)pl->filt2_bytes > i31) return false;
  const long long gy = (s.K + BM - 1) / BM;
  if (gy > 65535) return false;
  // every split takes the same number of chunks and none is empty
  const int cps = (pl->hp.nch + nsplit - 1) / nsplit;
  if ((nsplit - 1) * cps >= pl->hp.nch) return false;
  pl->hp.nsplit = nsplit;
  pl->hp.cps = cps;
  pl->partial_bytes = nsplit > 1 ? (size_t)nsplit * p.out_elems * 4 : 0;
  if ((long long)nsplit * p.out_elems > i31) return false;
  pl->gx = (unsigned)ntiles;
  pl->gy = (unsigned)gy;
  pl->gz = (unsigned)nsplit;
  pl->lds_bytes = lds;
  return true;
}

bool hconv_applicable(int which, const Shape& s) {
  if (which >= kNumOctet) return hfl_applicable(which - kNumOctet, s);
  HPlan pl;
  return plan_hconv(which, s, &pl);
}

// Device scratch of the per-call path: the re-laid filters, then the partial sums of a split.
size_t hconv_workspace_bytes(int which, const Shape& s) {
  if (which >= kNumOctet) return hfl_workspace_bytes(which - kNumOctet, s);
  HPlan pl;
  if (!plan_hconv(which, s, &pl)) return 0;
  return pl.partial_bytes ? h_align(pl.filt2_bytes) + pl.partial_bytes : pl.filt2_bytes;
}
// ... the two parts on their own (packed calls: the caller keeps the filters, the library the sums)
size_t hconv_packed_bytes(int which, const Shape& s) {
  HPlan pl;
  return plan_hconv(which, s, &pl) ? pl.filt2_bytes : 0;
}
size_t hconv_partial_bytes(int which, const Shape& s) {
  HPlan pl;
  return plan_hconv(which, s, &pl) ? pl.partial_bytes : 0;
}

// Estimated microseconds of a channel-octet variant on C8 activations, for shapes the tables do
// not list.  The workgroups of the busiest compute unit run `resident` at a time; one workgroup
// costs its MFMAs (stretched by the waves that share a matrix pipe), a per-stage term (barrier,
// exposed latency), its operand bytes at the rate one unit sustains (shared by its resident
// workgroups), a fixed part and its epilogue; a split adds the reduction kernel.  The eight
// constants are a least-squares fit (log time) to 3074 measured (shape, variant) points: the ten
// benchmark layers at batch 1-128 and ten unlisted shapes at batch 1, 5, 32, every applicable
// tile and split.  Picking by it is 3.4 % (geometric mean; worst 20 %) off the measured best on
// the former and 4.0 % (worst 24 %) on the latter.
static double hconv_cost(int which, const Shape& s) {
  HPlan pl;
  if (!plan_hconv(which, s, &pl)) return -1.0;
  const HTile& v = kHTiles[which / kNumHSplits];
  const double t0 = 3.667, c_mf = 0.021165, c_stage = 0.093718, c_wg = 1.753, r0 = 0.87467, r_b = 0.96214,
               c_b = 7.2175e-6, c_epi = 0.017462;
  const int waves = v.NTHR() / 64, taps = v.R * v.S;
  const long long wgs = (long long)pl.gx * pl.gy * pl.gz;
  long long resident = (long long)(kLdsLimitBytes / pl.lds_bytes);
  if (resident > 32 / waves) resident = 32 / waves;
  if (resident > 8) resident = 8;
  if (resident < 1) resident = 1;
  const long long per_cu = (wgs + 255) / 256;
  const double conc = (double)(per_cu < resident ? per_cu : resident);
  const double rounds = (double)((per_cu + resident - 1) / resident);
  double waves_simd = conc * waves / 4.0;
  if (waves_simd < 1.0) waves_simd = 1.0;
  const double mf = (double)pl.hp.cps * taps * (v.CC / 16) * v.MT * v.NT;
  const double stages = (double)pl.hp.cps * (v.R / v.TR);
  const double bytes_wg = (double)pl.hp.cps * ((double)v.BM() * taps * v.CC * 2 + (double)pl.hp.npos * v.CC * 2);
  const double epi = (double)v.BM() * v.BN() / (waves * 64);
  const double t_wg = mf * c_mf * waves_simd + stages * c_stage + bytes_wg * c_b * conc + c_wg + c_epi * epi;
  double t = t0 + rounds * t_wg;
  if (pl.hp.nsplit > 1) t += r0 + r_b * (double)pl.hp.g.out_elems * (pl.hp.nsplit + 0.5) * 1e-6;
  return t;
}
double hconv_model_cost(int which, const Shape& s) { return which < kNumOctet ? hconv_cost(which, s) : -1.0; }

// The variant the half-precision entry points take for a shape the half-precision tables do not
// list, or -1 when the layer is better left to the widening kernel (not applicable, or, unless
// any_size, too few output points).
int hconv_select(const Shape& s, bool any_size) {
  if (!any_size && (long long)s.N * s.P * s.Q < 1024) return -1;
  int best = -1;
  double best_cost = 0.0;
  for (int w = 0; w < kNumOctet; ++w) {
    const double cost = hconv_cost(w, s);
    if (cost < 0.0) continue;
    if (best < 0 || cost < best_cost) { best = w; best_cost = cost; }
  }
  if (best < 0) {
    // a first layer (measured faster than the widening kernel from batch 1 up): the widest
    // pixel tile that still gives every compute unit a tile, else the narrowest
    int narrowest = -1;
    for (int f = 0; f < hfl_num_variants(); ++f) {
      if (!hfl_applicable(f, s)) continue;
      narrowest = f;
      if (hfl_tiles(f, s) >= 256) return kNumOctet + f;
    }
    if (narrowest >= 0) return kNumOctet + narrowest;
  }
  return best;
}

// The filters re-laid for tile `which` into `packed` (hconv_workspace_bytes bytes).
hipError_t launch_hconv_pack(int which, const void* filt, void* packed, const Shape& s, hipStream_t st) {
  HPlan pl;
  if (!hconv_packable(which) || !plan_hconv(which, s, &pl)) return hipErrorInvalidValue;
  const HTile& v = kHTiles[which / kNumHSplits];
  const long long total = (long long)(pl.filt2_bytes / 2);
  long long blocks = (total + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  return launch_kernel(hconv_repack_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       static_cast<const _Float16*>(filt), static_cast<_Float16*>(packed), s.K, s.C,
                       v.R * v.S, v.CC, pl.hp.nch, total);
}

// The convolution itself on filters that launch_hconv_pack re-laid for the same tile and shape;
// in_c8 / out_c8 say which activations are octet-interleaved (C8 out needs K % 8 == 0; NCHW in
// with C8 out is not built).  A split variant leaves its partial sums in `scratch`
// (hconv_partial_bytes, 16-byte aligned) and a reduction kernel finishes the layer.
hipError_t launch_hconv_packed(int which, const void* in, const void* packed, const float* bias, void* out,
                               const Shape& s, int relu, int in_c8, int out_c8, void* scratch, hipStream_t st) {
  HPlan pl;
  if (!hconv_packable(which) || !plan_hconv(which, s, &pl)) return hipErrorInvalidValue;
  if (out_c8 && (!in_c8 || s.K % 8 != 0)) return hipErrorInvalidValue;
  if (pl.partial_bytes && !scratch) return hipErrorInvalidValue;
  pl.hp.g.in = static_cast<const float*>(in);
  pl.hp.g.bias = bias;
  pl.hp.g.out = static_cast<float*>(out);
  pl.hp.g.relu = relu;
  pl.hp.filt2 = static_cast<const _Float16*>(packed);
  pl.hp.partial = static_cast<float*>(scratch);
  const HLaunchFn fn = out_c8 ? hconv_launch_l2(which / kNumHSplits)
                              : (in_c8 ? hconv_launch_l1(which / kNumHSplits) : hconv_launch_l0(which / kNumHSplits));
  hipError_t e = fn(pl.hp, dim3(pl.gx, pl.gy, pl.gz), pl.lds_bytes, st);
  if (e != hipSuccess || !pl.partial_bytes) return e;
  return launch_splitk_reduce(pl.hp.partial, bias, static_cast<float*>(out), pl.hp.nsplit, pl.hp.g.out_elems, s.K,
                              s.P * s.Q, relu, true, out_c8 != 0, st);
}

hipError_t launch_hconv(int which, const void* in, const void* filt, const float* bias, void* out,
                        const Shape& s, int relu, int in_c8, int out_c8, void* ws, hipStream_t st) {
  if (which >= kNumOctet) {
    if (in_c8) return hipErrorInvalidValue;
    return launch_hfl(which - kNumOctet, in, filt, bias, out, s, relu, out_c8, ws, st);
  }
  HPlan pl;
  if (!plan_hconv(which, s, &pl)) return hipErrorInvalidValue;
  hipError_t e = launch_hconv_pack(which, filt, ws, s, st);
  if (e != hipSuccess) return e;
  void* scratch = pl.partial_bytes ? static_cast<char*>(ws) + h_align(pl.filt2_bytes) : nullptr;
  return launch_hconv_packed(which, in, ws, bias, out, s, relu, in_c8, out_c8, scratch, st);
}

#endif  // HCONV_LAYOUT == 0

}  // namespace bconv
