// Index arithmetic of the tiled MFMA convolution kernel, usable from device code
// and from plain host C++ (the host-side bounds audit walks exactly these
// functions for every workgroup, thread and reduction chunk before a shape /
// variant pair is ever launched).
//
// Problem view (paper Section III, convolution as a matrix product, with the
// roles fixed by the NCHW / KCRS layouts):
//     out_n[K x PQ] = filt[K x (C*R*S)] . rows_of(in_n)[(C*R*S) x PQ]
// Rows of the left operand are filters, columns of the right operand are output
// pixels.  The reduction index is split as (kk, s) with kk = c*R + r a
// "reduction row" (one input channel, one kernel row) and s the kernel column.
//
// Workgroup tile: BM filters x BN consecutive flattened output pixels
// g = (img*P + p)*Q + q.  The pixels of a tile lie on at most `nrows` output
// rows rho = img*P + p ("row slots").  For one reduction row kk = (c, r) and
// one slot the kernel stages the piece of input row (img, c, p*stride-pad+r)
// that the slot's pixels read -- the paper's tiled-convolution idea (Section VI:
// load whole X tiles of the input per workgroup, unroll over the kernel's X
// extent) -- so the S taps of a pixel are S shifted reads of one staged row.
// For stride > 1 a staged row is split into `stride` phase planes so that
// consecutive pixels read consecutive LDS words for every tap.
#pragma once

#if defined(__HIPCC__)
#define BCONV_HD __host__ __device__ __forceinline__
#else
#define BCONV_HD inline
#endif

namespace bconv {

// Division of a non-negative 31-bit number by a divisor fixed per launch, as a multiply
// and a shift (the round-up method for unsigned division by an invariant integer): the
// host derives (mul, shift) once, the kernel's prologue then spends three instructions
// per quotient instead of the ~30 of a run-time integer division.
struct FastDiv {
  unsigned mul, shift;
};

inline FastDiv make_fastdiv(unsigned d) {
  if (d == 0) d = 1;
  unsigned s = 0;
  while ((1u << s) < d) ++s;                                    // ceil(log2 d)
  const unsigned long long m = ((1ull << 32) * ((1ull << s) - d)) / d + 1;   // < 2^32 for d < 2^31
  return FastDiv{(unsigned)m, s};
}

// floor(n / d) for 0 <= n < 2^31 and the d that f was made for.
BCONV_HD int fd_div(int n, FastDiv f) {
#if defined(__HIP_DEVICE_COMPILE__)
  const unsigned hi = __umulhi((unsigned)n, f.mul);
#else
  const unsigned hi = (unsigned)(((unsigned long long)(unsigned)n * f.mul) >> 32);
#endif
  return (int)((hi + (unsigned)n) >> f.shift);
}

// Kernel argument block of the tiled MFMA kernel (plain data).
struct TconvParams {
  const float* in;
  const float* filt;
  const float* bias;    // may be null
  float* out;
  float* partial;       // split-K partial sums [nsplit][N*K*P*Q], null when nsplit == 1
  int N, C, H, W, K, R, S, stride, pad, P, Q;
  int relu;
  int PQ, NPQ, HW, CHW, CRS, CRrows;   // CRrows = C*R reduction rows
  int nrows, phst, rowst, plane;       // staged-input geometry, plane = nrows*rowst
  int compact;                         // S == 1 and stride == 1: one staged cell per bv tile pixels
  int bv;                              // pixels per staged cell in compact mode (1 or 4)
  int halo;                            // input staged as whole padded rows per channel (see h_cell)
  int hp, wt, vr;                      // halo mode: padded height, padded width, staged rows per channel
  int gbias;                           // pad*W + pad: most negative cell offset, see the kernel's loads
  int ast;                             // LDS stride between filter rows (odd)
  int nchunks, chunks_per_split, nsplit;
  int out_elems;                       // N*K*P*Q
  int filter_major;                    // order of the block-to-tile map, see xcd_tile
  FastDiv fdQ, fdP, fdRowst, fdHp;     // divisions by Q, P, rowst and hp (hp: halo mode)
};

// Which tile a workgroup computes, from its position in dispatch order (x fastest, then
// y, then z).  Consecutive workgroups go to the eight accelerator dies in turn, and each
// die has its own L2; this map hands each die one contiguous run of the tile list, so that
// workgroups that share an operand tile meet in one L2 instead of every die fetching it.
// The list is ordered (reduction split, pixel tile, filter tile) when the input is the
// larger operand (filter_major = 0: a die's run shares few input tiles and reads all the
// filters, which are small) and (reduction split, filter tile, pixel tile) when the filters
// are (filter_major = 1, the small batches: each die then reads an eighth of the filters
// and the whole, small, input).  With a run at least one row of the list long, the bytes
// the eight L2s fetch are 8 F + I in the first order and F + 8 I in the second (F, I the
// filter and input bytes), so the larger operand decides.  It is a bijection on the grid.
struct BlockTile {
  int x, y, z;        // pixel tile, filter tile, reduction split
};

BCONV_HD BlockTile xcd_tile(unsigned lin, unsigned gx, unsigned gy, unsigned gz, int filter_major) {
  const unsigned kDies = 8;
  const unsigned total = gx * gy * gz;
  const unsigned die = lin % kDies, slot = lin / kDies;
  const unsigned q = total / kDies, r = total % kDies;
  const unsigned n = die * q + (die < r ? die : r) + slot;   // position in the tile list
  BlockTile b;
  if (filter_major) {
    b.x = (int)(n % gx);
    b.y = (int)((n / gx) % gy);
  } else {
    b.y = (int)(n % gy);
    b.x = (int)((n / gy) % gx);
  }
  b.z = (int)(n / (gx * gy));
  return b;
}

struct PixTile {
  int g0, cnt;        // first flattened pixel and number of valid pixels
  int rho0, q00;      // output row / column of the first pixel
  int rho1, qlast;    // output row / column of the last valid pixel
};

BCONV_HD PixTile pix_tile(int tile_idx, int BN, int NPQ, int Q, FastDiv fdQ) {
  PixTile t;
  t.g0 = tile_idx * BN;
  int rem = NPQ - t.g0;
  t.cnt = rem < BN ? rem : BN;
  t.rho0 = fd_div(t.g0, fdQ);
  t.q00 = t.g0 - t.rho0 * Q;
  int gl = t.g0 + t.cnt - 1;
  t.rho1 = fd_div(gl, fdQ);
  t.qlast = gl - t.rho1 * Q;
  return t;
}

// Upper bound on the row slots a tile of BN consecutive pixels can touch.
BCONV_HD int tile_nrows(int BN, int Q, int total_rows) {
  int n = (BN - 1) / Q + 2;
  return n < total_rows ? n : total_rows;
}

// Words per phase plane of one staged row.
BCONV_HD int tile_phst(int BN, int Q, int S, int stride) {
  return (Q < BN ? Q : BN) + (S - 1) / stride;
}

constexpr int kNeverValid = -(1 << 24);

// One staged-input cell: where it lives in a B plane, which input word it takes
// for reduction row (c=0, r=0), and the input row index for r = 0.  A cell that
// never loads (outside the tile's need, or in the zero padding columns) has
// ih0 = kNeverValid so that the per-row test (unsigned)(ih0 + r) < H fails.
struct BCell {
  int lds;
  int goff;
  int ih0;
};

BCONV_HD BCell b_cell(const TconvParams& p, const PixTile& t, int e, int S, int STR) {
  BCell c;
  if (p.compact) {
    // kernel width 1 at stride 1: cell e covers the input words under tile pixels
    // bv*e .. bv*e + bv - 1 (bv = 4 only where a cell never straddles an image row)
    int col = e * p.bv;
    bool ok = col < t.cnt;
    int g = t.g0 + (ok ? col : 0);
    int rho = fd_div(g, p.fdQ);
    int q = g - rho * p.Q;
    int img = fd_div(rho, p.fdP);
    int pp = rho - img * p.P;
    int iw = q - p.pad;
    ok = ok && (iw >= 0) && (iw < p.W);
    int ih0 = pp - p.pad;
    c.lds = col;
    c.goff = img * p.CHW + ih0 * p.W + iw;
    c.ih0 = ok ? ih0 : kNeverValid;
    return c;
  }
  int slot = fd_div(e, p.fdRowst);
  int xrel = e - slot * p.rowst;
  int rho = t.rho0 + slot;
  bool ok = (slot < p.nrows) && (rho <= t.rho1);
  int img = fd_div(rho, p.fdP);
  int pp = rho - img * p.P;
  int qlo = (slot == 0) ? t.q00 : 0;
  int qhi = (rho == t.rho1) ? t.qlast : p.Q - 1;
  int width = (qhi - qlo) * STR + S;
  ok = ok && (xrel < width);
  int iw = qlo * STR + xrel - p.pad;
  ok = ok && (iw >= 0) && (iw < p.W);
  int ih0 = pp * STR - p.pad;
  int ph = xrel % STR;
  c.lds = slot * p.rowst + ph * p.phst + xrel / STR;
  c.goff = img * p.CHW + ih0 * p.W + iw;
  c.ih0 = ok ? ih0 : kNeverValid;
  return c;
}

// One output column of the tile as a lane sees it.
struct BLane {
  int ldsbase;   // slot*rowst + (q - qlo(slot)): add tap_off(s) and kl*plane
  int outoff;    // img*K*PQ + p*Q + q: add k*PQ
  int valid;
};

BCONV_HD BLane b_lane(const TconvParams& p, const PixTile& t, int col) {
  BLane l;
  l.valid = col < t.cnt;
  int cc = l.valid ? col : t.cnt - 1;   // ragged tail: alias the last valid pixel
  int g = t.g0 + cc;
  int rho = fd_div(g, p.fdQ);
  int q = g - rho * p.Q;
  int slot = rho - t.rho0;
  int qlo = (slot == 0) ? t.q00 : 0;
  int img = fd_div(rho, p.fdP);
  int pp = rho - img * p.P;
  l.ldsbase = p.compact ? cc : slot * p.rowst + (q - qlo);
  l.outoff = img * p.K * p.PQ + pp * p.Q + q;
  return l;
}

// ---- halo staging -------------------------------------------------------------
// Instead of one copy of an input row per kernel row that reads it, the tile's
// input is staged once: for each channel of the chunk the padded input rows
// u_first .. u_first + vr - 1, where u = img*(H + 2*pad) + (ih + pad) numbers the
// padded rows of all images consecutively (rows of zeros separate the images).
// An output pixel (img, p, q) then reads kernel row r, column s at
//   (u(img, p*stride) - u_first + r) * rowst + tap_off(s) + q
// so both kernel offsets are uniform over the lanes.  Whole padded rows are
// staged (phase-split for stride > 1 exactly like the row-slot scheme).
struct HaloTile {
  int u_first, vr;
};

BCONV_HD HaloTile halo_tile(const TconvParams& p, const PixTile& t) {
  HaloTile h;
  int img0 = fd_div(t.rho0, p.fdP), p0 = t.rho0 - img0 * p.P;
  int img1 = fd_div(t.rho1, p.fdP), p1 = t.rho1 - img1 * p.P;
  h.u_first = img0 * p.hp + p0 * p.stride;
  h.vr = img1 * p.hp + p1 * p.stride + p.R - h.u_first;
  return h;
}

// Staged cell e of one channel plane: row e / rowst of the tile's halo, padded
// column e % rowst.  goff is the input word for channel 0; ih0 = 0 marks a cell
// that loads, kNeverValid one that holds padding (or lies outside the halo).
BCONV_HD BCell h_cell(const TconvParams& p, const HaloTile& ht, int e, int STR) {
  BCell c;
  int v = fd_div(e, p.fdRowst);
  int xp = e - v * p.rowst;
  bool ok = (v < ht.vr) && (xp < p.wt);
  int u = ht.u_first + v;
  int img = fd_div(u, p.fdHp);
  int ih = u - img * p.hp - p.pad;
  int iw = xp - p.pad;
  ok = ok && (img < p.N) && (ih >= 0) && (ih < p.H) && (iw >= 0) && (iw < p.W);
  c.lds = v * p.rowst + (xp % STR) * p.phst + xp / STR;
  c.goff = img * p.CHW + ih * p.W + iw;
  c.ih0 = ok ? 0 : kNeverValid;
  return c;
}

BCONV_HD BLane h_lane(const TconvParams& p, const PixTile& t, const HaloTile& ht, int col) {
  BLane l;
  l.valid = col < t.cnt;
  int cc = l.valid ? col : t.cnt - 1;
  int g = t.g0 + cc;
  int rho = fd_div(g, p.fdQ);
  int q = g - rho * p.Q;
  int img = fd_div(rho, p.fdP);
  int pp = rho - img * p.P;
  l.ldsbase = (img * p.hp + pp * p.stride - ht.u_first) * p.rowst + q;
  l.outoff = img * p.K * p.PQ + pp * p.Q + q;
  return l;
}

// LDS word offset of kernel column s relative to a lane's ldsbase.
BCONV_HD int tap_off(int s, int STR, int phst) {
  return (s % STR) * phst + s / STR;
}

// Words per LDS read of a lane's filter run.  One MFMA consumes KSL reduction rows (2 for
// 32x32x2, 4 for 16x16x4), lane slice h taking its row from the h-th of KSL equal parts of
// the chunk; the run of reduction group g inside part h starts at word
// h*(KR/KSL)*S + g*(KR/KSL/KS)*S of a filter row, so the read width is limited by the
// alignment of both terms.  Run-time S (S = 0): 1.
BCONV_HD constexpr int a_read_width(int KR, int S, int KS, int KSL) {
  return S <= 0 ? 1
         : ((((KR / KSL) * S) % 4 == 0 && ((KR / KSL / KS) * S) % 4 == 0) ? 4
            : ((((KR / KSL) * S) % 2 == 0 && ((KR / KSL / KS) * S) % 2 == 0) ? 2 : 1));
}

// LDS stride (words) between filter rows holding KRS words each: a multiple of
// the read width whose quotient is odd, which spreads rows over all banks for
// 4-, 8- and 16-byte reads alike.
BCONV_HD constexpr int a_row_stride(int KRS, int vw) {
  return (((KRS + vw - 1) / vw) | 1) * vw;
}

// Row of a 32x32 MFMA accumulator tile held by (lane, register i), i in [0,16).
BCONV_HD int acc_row_32(int lane, int i) {
  return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
}

// Row of an MS x MS accumulator tile held by (lane, register i): the 32x32x2 map above, or
// for 16x16x4 (four registers per lane) row 4*(lane/16) + i; the column is lane % MS in both.
BCONV_HD int acc_row(int lane, int i, int MS) {
  return MS == 32 ? acc_row_32(lane, i) : 4 * (lane >> 4) + i;
}

}  // namespace bconv
