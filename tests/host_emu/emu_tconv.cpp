// Host-side model of the tiled MFMA convolution kernel, for CPU tests only.
//
// It walks the same index functions (bconv_geom.h) and the same launch plan
// (bconv_plan.h) as the device kernel, thread by thread and chunk by chunk, with
// every LDS and global access bounds-checked and LDS poisoned with NaN before
// each chunk, and models v_mfma_f32_32x32x2_f32 and v_mfma_f32_16x16x4_f32 by their
// definition (D[i][j] += sum_k A[i][k]*B[k][j] over an MS x MS tile, lane l supplying
// A[l%MS][l/MS] and B[l/MS][l%MS]).  It checks the kernel's indexing and staging logic on the CPU;
// it is not part of the library and the library never calls it.
#include <cmath>
#include <cstdio>
#include <limits>
#include <vector>

#include "../../paper_1606_00094_amd/csrc/bconv_plan.h"

using namespace bconv;

namespace {
struct Oob {
  long long count = 0;
  void hit(const char* what, long long idx, long long lim) {
    if (count < 5) std::fprintf(stderr, "emu_tconv: %s index %lld outside [0,%lld)\n", what, idx, lim);
    ++count;
  }
};
}  // namespace

extern "C" int emu_num_tiles() { return kNumTiles; }
extern "C" const char* emu_tile_name(int t) { return (t >= 0 && t < kNumTiles) ? kTileDescs[t].name : ""; }

// Returns 0 on success, 1 if the tile does not apply, or 2 + number of
// out-of-bounds / poisoned accesses.
extern "C" long long emu_tconv(const float* in, const float* filt, const float* bias, float* out,
                               int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               int relu, int tile, int nsplit) {
  if (tile < 0 || tile >= kNumTiles) return 1;
  const TileDesc& v = kTileDescs[tile];
  Shape sh{N, C, H, W, K, R, S, stride, pad, (H + 2 * pad - R) / stride + 1,
           (W + 2 * pad - S) / stride + 1};
  Plan pl;
  if (!plan_tconv(sh, v, nsplit, &pl)) return 1;
  const TconvParams& p = pl.p;
  const int BM = v.BM(), BN = v.BN(), NTHR = v.NTHR(), KR = v.KR, EPT = v.EPT;
  const int Rk = p.R, Sk = p.S, STR = p.stride;
  const int KRS = KR * Sk;
  const int SP = v.S > 0 ? v.S : kSmaxGeneric;
  const int KRSP = KR * SP;
  const int AV = v.AV;
  const int AGRP = KRSP / AV;
  const int NA = (BM * AGRP + NTHR - 1) / NTHR;
  const long long in_elems = (long long)p.N * p.CHW, filt_elems = (long long)p.K * p.CRS;
  const int NPL = p.halo ? KR / p.R : KR;   // LDS planes per input buffer
  const int abuf = BM * p.ast, bbuf = NPL * p.plane;
  if ((size_t)(2 * abuf + 2 * (bbuf + kLdsTrashWords) + kLdsTrashWords) * 4 > pl.lds_bytes) return 2;
  Oob oob;
  const float nanv = std::numeric_limits<float>::quiet_NaN();
  std::vector<float> partial((size_t)p.nsplit * p.out_elems, nanv);
  std::vector<float> As(abuf), Bs(bbuf);
  const int ncell = p.nrows * p.rowst;

  for (unsigned lin = 0; lin < pl.gx * pl.gy * pl.gz; ++lin) {
    const BlockTile bt = xcd_tile(lin, pl.gx, pl.gy, pl.gz, p.filter_major);
    const unsigned bx = (unsigned)bt.x, by = (unsigned)bt.y, bz = (unsigned)bt.z;
    const PixTile t = pix_tile((int)bx, BN, p.NPQ, p.Q, p.fdQ);
    const HaloTile ht = p.halo ? halo_tile(p, t) : HaloTile{0, 0};
    if (p.halo && ht.vr > p.vr) oob.hit("halo rows", ht.vr, p.vr);
    const int m0 = (int)by * BM;
    // accumulators per wave tile as plain matrices [BM][BN]
    const int KS = v.KS, NW = v.WM * v.WN;
    std::vector<float> acc((size_t)KS * BM * BN, 0.0f);   // one accumulator set per reduction group
    const int ch_begin = (int)bz * p.chunks_per_split;
    int ch_end = ch_begin + p.chunks_per_split;
    if (ch_end > p.nchunks) ch_end = p.nchunks;
    const bool a_scalar = NA <= 12;
    const int BVWc = (v.BV == kModeCompact4) ? 4 : 1;
    const int CPP = BN / BVWc;
    const bool flat = !p.halo && v.R == 1 && v.S == 1 && v.STR == 1 && CPP < NTHR && NTHR % CPP == 0 &&
                      KR % (NTHR / CPP) == 0;
    const int PSTEP = flat ? NTHR / CPP : 1;
    const bool has_tail = (long long)p.nchunks * KR * Sk > p.CRS;
    for (int ch = ch_begin; ch < ch_end; ++ch) {
      std::fill(As.begin(), As.end(), nanv);
      std::fill(Bs.begin(), Bs.end(), nanv);
      const int kk0 = ch * KR;
      const int col0 = kk0 * Sk;
      for (int tid = 0; tid < NTHR; ++tid) {
        for (int i = 0; i < NA; ++i) {
          int e = tid + i * NTHR;
          int m = e / AGRP, j = (e - m * AGRP) * AV;
          const bool in_lds = (m < BM) && (j < KRS);
          bool ok;
          long long gi;
          if (a_scalar) {
            // per-lane offset fixed before the loop plus the chunk's column offset,
            // range-checked together against the end of the tensor
            const bool lane_ok = in_lds && (m0 + m < p.K);
            const long long voff = (long long)(m0 + m) * p.CRS + j;
            ok = lane_ok && (voff + col0 + AV <= filt_elems);
            gi = ok ? voff + col0 : 0;
          } else {
            ok = in_lds && (m0 + m < p.K) && (col0 + j < p.CRS);
            gi = ok ? (long long)(m0 + m) * p.CRS + col0 + j : 0;
          }
          if (AV == 4 && (gi % 4) != 0) oob.hit("filt alignment", gi, 4);
          for (int u = 0; u < AV; ++u) {
            if (gi + u < 0 || gi + u >= filt_elems) { oob.hit("filt", gi + u, filt_elems); continue; }
            float val = ok ? filt[gi + u] : 0.0f;
            if (in_lds) {
              int li = m * p.ast + j + u;
              if (li < 0 || li >= abuf) oob.hit("A lds", li, abuf); else As[li] = val;
            }
          }
        }
        // words past the end of the filter row (last chunk of the reduction) are zeroed
        if (a_scalar && has_tail && ch == p.nchunks - 1) {
          for (int i = 0; i < NA; ++i) {
            int e = tid + i * NTHR;
            int m = e / AGRP, j = (e - m * AGRP) * AV;
            if ((m < BM) && (j < KRS) && (col0 + j >= p.CRS))
              for (int u = 0; u < AV; ++u) As[m * p.ast + j + u] = 0.0f;
          }
        }
        if (v.BV == kModeHaloFlat) {
          // flat halo staging: EPT thread groups, group kl0 staging planes kl0, kl0 + EPT, ...;
          // one cell per thread.  What the lanes of a load share (chunk, first plane of the
          // group's stride) decides whether the load is issued at all; a thread whose own
          // plane lies past the last channel then reads the next image (or zeros past the end
          // of the tensor) and the cell is zeroed after the store.
          const int PST = v.EPT, CAP = NTHR / PST;
          const int kl0 = tid / CAP, e = tid - kl0 * CAP;
          if (e < ncell) {
            BCell cell = h_cell(p, ht, e, STR);
            for (int j = 0; j < NPL / PST; ++j) {
              const int kl = kl0 + j * PST;
              const bool sok = ch * NPL + j * PST < p.C;
              long long gi = (long long)cell.goff + (long long)(ch * NPL + kl) * p.HW;
              const bool ok = sok && cell.ih0 != kNeverValid && gi < in_elems;
              if (ok && gi < 0) { oob.hit("in", gi, in_elems); continue; }
              float val = ok ? in[gi] : 0.0f;
              if (ch * NPL + kl >= p.C) val = 0.0f;             // tail cleanup
              if (cell.lds < 0 || cell.lds >= p.plane || kl >= NPL) oob.hit("B lds", cell.lds, p.plane);
              else Bs[(long long)kl * p.plane + cell.lds] = val;
            }
          }
        } else if (p.halo) {
          for (int j = 0; j < NPL; ++j) {
            const int c = ch * NPL + j;
            for (int i = 0; i < EPT; ++i) {
              int e = tid + i * NTHR;
              if (e >= ncell) continue;
              BCell cell = h_cell(p, ht, e, STR);
              bool ok = (c < p.C) && (cell.ih0 != kNeverValid);
              long long gi = ok ? (long long)cell.goff + (long long)c * p.HW : 0;
              if (gi < 0 || gi >= in_elems) { oob.hit("in", gi, in_elems); continue; }
              float val = ok ? in[gi] : 0.0f;
              if (cell.lds < 0 || cell.lds >= p.plane) oob.hit("B lds", cell.lds, p.plane);
              else Bs[(long long)j * p.plane + cell.lds] = val;
            }
          }
        } else if (flat) {
          // flat pointwise staging: one cell per thread, planes kl0, kl0 + PSTEP, ...; the
          // range check sees only the end of the tensor, planes past the last channel are
          // zeroed after the store
          const int kl0 = tid / CPP, e = tid - kl0 * CPP;
          BCell cell = b_cell(p, t, e, Sk, STR);
          const bool cell_ok = (unsigned)cell.ih0 < (unsigned)p.H;
          for (int j = 0; j < KR / PSTEP; ++j) {
            const int kl = kl0 + j * PSTEP;
            const bool sok = (kk0 + j * PSTEP) < p.CRrows;     // the scalar part of the test
            for (int u = 0; u < p.bv; ++u) {
              long long gi = (long long)cell.goff + (long long)(kk0 + kl) * p.HW + u;
              const bool ok = cell_ok && sok && gi + (p.bv - 1 - u) < in_elems;
              if (ok && (gi < 0 || gi >= in_elems)) { oob.hit("in", gi, in_elems); continue; }
              if (p.bv == 4 && u == 0 && ok && (gi % 4) != 0) oob.hit("in alignment", gi, 4);
              float val = ok ? in[gi] : 0.0f;
              if (kk0 + kl >= p.CRrows) val = 0.0f;           // tail cleanup
              long long li = (long long)kl * p.plane + cell.lds + u;
              if (cell.lds + u < 0 || cell.lds + u >= p.plane || kl >= KR) oob.hit("B lds", cell.lds + u, p.plane);
              else Bs[li] = val;
            }
          }
        } else {
        int c = kk0 / Rk, r = kk0 - c * Rk;
        for (int kl = 0; kl < KR; ++kl) {
          const bool rowok = (kk0 + kl) < p.CRrows;
          const int koff = c * p.HW + r * p.W;
          for (int i = 0; i < EPT; ++i) {
            int e = tid + i * NTHR;
            if (e * p.bv >= ncell) continue;
            BCell cell = b_cell(p, t, e, Sk, STR);
            bool ok = rowok && ((unsigned)(cell.ih0 + r) < (unsigned)p.H);
            if (v.BV == kModeSlotsNoPad) {
              // scalar addressing: a cell that ever loads, loads for every kernel row; the
              // row must then be inside the image (the kernel has no per-row mask)
              ok = rowok && cell.ih0 != kNeverValid;
              if (ok && !((unsigned)(cell.ih0 + r) < (unsigned)p.H)) oob.hit("unmasked row", cell.ih0 + r, p.H);
            }
            for (int u = 0; u < p.bv; ++u) {
              long long gi = ok ? (long long)cell.goff + koff + u : 0;
              if (p.bv == 4 && u == 0 && ok && (gi % 4) != 0) oob.hit("in alignment", gi, 4);
              if (gi < 0 || gi >= in_elems) { oob.hit("in", gi, in_elems); continue; }
              float val = ok ? in[gi] : 0.0f;
              long long li = (long long)kl * p.plane + cell.lds + u;
              if (cell.lds + u < 0 || cell.lds + u >= p.plane) oob.hit("B lds", cell.lds + u, p.plane);
              else Bs[li] = val;
            }
          }
          if (++r == Rk) { r = 0; ++c; }
        }
        }
      }
      // compute: every wave, every (j, s) step
      for (int wave = 0; wave < NW * KS; ++wave) {
        const int kgrp = wave / NW, wv = wave % NW;
        const int wm = wv / v.WN, wn = wv % v.WN;
        float* accg = acc.data() + (size_t)kgrp * BM * BN;
        const int MS = v.MS, KSL = v.KSL();
        const int NPAIR = KR / KSL / KS, HALF = (KR / KSL) * Sk, RUN = NPAIR * Sk;
        for (int j = 0; j < NPAIR; ++j)
        for (int s = 0; s < Sk; ++s) {
          const int aoff = j * Sk + s;
          const int boff = (p.halo ? (j / p.R) * p.plane + (j % p.R) * p.rowst : j * p.plane) +
                           tap_off(s, STR, p.phst);
          for (int mt = 0; mt < v.MT; ++mt)
          for (int nt = 0; nt < v.NT; ++nt) {
            float a[64], b[64];
            for (int lane = 0; lane < 64; ++lane) {
              const int l32 = lane % MS, h = lane / MS;
              const int laneA = (wm * v.MT * MS + l32) * p.ast + h * HALF + kgrp * RUN;
              BLane bl = p.halo ? h_lane(p, t, ht, (wn * v.NT + nt) * MS + l32)
                                : b_lane(p, t, (wn * v.NT + nt) * MS + l32);
              const int hk = h * (KR / KSL) + kgrp * NPAIR;
              const int laneB = bl.ldsbase + (p.halo ? hk / p.R : hk) * p.plane;
              long long ai = (long long)laneA + mt * MS * p.ast + aoff;
              long long bi = (long long)laneB + boff;
              if (ai < 0 || ai >= abuf) { oob.hit("A read", ai, abuf); a[lane] = 0; } else a[lane] = As[ai];
              if (bi < 0 || bi >= bbuf) { oob.hit("B read", bi, bbuf); b[lane] = 0; } else b[lane] = Bs[bi];
            }
            for (int i = 0; i < MS; ++i)
              for (int jn = 0; jn < MS; ++jn) {
                float d = accg[(size_t)((wm * v.MT + mt) * MS + i) * BN + (wn * v.NT + nt) * MS + jn];
                for (int k = 0; k < KSL; ++k) d = std::fmaf(a[k * MS + i], b[k * MS + jn], d);
                accg[(size_t)((wm * v.MT + mt) * MS + i) * BN + (wn * v.NT + nt) * MS + jn] = d;
              }
          }
        }
      }
    }
    // reduction groups summed in group order, as the kernel does through LDS
    if ((size_t)BM * BN * 4 > pl.lds_bytes && KS > 1) oob.hit("reduction scratch", (long long)BM * BN * 4, (long long)pl.lds_bytes);
    for (int g = 1; g < KS; ++g)
      for (size_t i = 0; i < (size_t)BM * BN; ++i) acc[i] += acc[(size_t)g * BM * BN + i];
    // epilogue through the lane/register map
    for (int wave = 0; wave < v.WM * v.WN; ++wave) {
      const int wm = wave / v.WN, wn = wave % v.WN;
      for (int lane = 0; lane < 64; ++lane)
      for (int mt = 0; mt < v.MT; ++mt)
      for (int i = 0; i < v.MS * v.MS / 64; ++i) {
        const int row = (wm * v.MT + mt) * v.MS + acc_row(lane, i, v.MS);
        const int k = m0 + row;
        if (k >= p.K) continue;
        for (int nt = 0; nt < v.NT; ++nt) {
          const int col = (wn * v.NT + nt) * v.MS + lane % v.MS;
          BLane bl = p.halo ? h_lane(p, t, ht, col) : b_lane(p, t, col);
          if (!bl.valid) continue;
          long long oi = (long long)bl.outoff + (long long)k * p.PQ;
          if (oi < 0 || oi >= p.out_elems) { oob.hit("out", oi, p.out_elems); continue; }
          partial[(size_t)bz * p.out_elems + oi] = acc[(size_t)row * BN + col];
        }
      }
    }
  }
  const int PQ = p.PQ;
  for (int i = 0; i < p.out_elems; ++i) {
    float val = 0.0f;
    for (int z = 0; z < p.nsplit; ++z) val += partial[(size_t)z * p.out_elems + i];
    if (bias) val += bias[(i / PQ) % p.K];
    if (relu) val = val > 0.0f ? val : 0.0f;
    out[i] = val;
  }
  return oob.count ? 2 + oob.count : 0;
}

// fd_div(n, make_fastdiv(d)) for each pair; returns the index of the first quotient that
// differs from n / d, or -1.
extern "C" long long emu_fastdiv_check(const int* n, const int* d, long long count) {
  for (long long i = 0; i < count; ++i)
    if (fd_div(n[i], make_fastdiv((unsigned)d[i])) != n[i] / d[i]) return i;
  return -1;
}

extern "C" void emu_xcd_tile(unsigned lin, unsigned gx, unsigned gy, unsigned gz, int filter_major, int* x,
                             int* y, int* z) {
  bconv::BlockTile b = bconv::xcd_tile(lin, gx, gy, gz, filter_major);
  *x = b.x; *y = b.y; *z = b.z;
}
