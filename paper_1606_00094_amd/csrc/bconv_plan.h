// Launch planning of the tiled MFMA kernel: plain host C++ (no HIP types) so that
// the library and the host-side emulation used by the CPU tests derive the
// argument block and grid from the same code.
#pragma once
#include <cstddef>
#include <cstring>

#include "bconv_geom.h"

namespace bconv {

struct Shape {
  int N, C, H, W, K, R, S, stride, pad, P, Q;
};

constexpr size_t kLdsLimitBytes = 160 * 1024;
constexpr int kSmaxGeneric = 16;   // widest kernel the run-time generic tiles take
// input staging mode of a tile (last column of variants.def)
constexpr int kModeSlots = 1;      // one copy of an input row per kernel row and output row (or compact cells)
constexpr int kModeCompact4 = 4;   // compact cells of four pixels, 16-byte loads (flattened pointwise)
constexpr int kModeHalo = 2;       // whole padded rows per channel, staged once
constexpr int kModeSlotsNoPad = 3; // kModeSlots for layers without padding (every staged row is inside the image)
// kModeHalo for tiles whose halo has far fewer cells than the workgroup has threads: the
// threads form EPT groups, group g staging planes g, g + EPT, ... of a chunk, one cell per
// thread (the EPT column of variants.def is the number of groups here), so that few lanes
// issue masked loads
constexpr int kModeHaloFlat = 5;
constexpr int kLdsTrashWords = 16; // LDS words (in front of the filter buffers, behind each input buffer) that absorb masked stores

// One row of variants.def.
struct TileDesc {
  const char* name;
  int R, S, STR;            // 0 = run-time value
  int WM, WN, MT, NT, KR, EPT, AV, KS, BV;
  int PD;                   // register sets of the software pipeline (chunks in flight + 1)
  int WPE;                  // waves per SIMD the compiler is asked to make room for (1: no demand)
  int MS;                   // edge of one MFMA accumulator tile: 32 (32x32x2) or 16 (16x16x4)
  int BM() const { return WM * MT * MS; }
  int BN() const { return WN * NT * MS; }
  int NTHR() const { return WM * WN * KS * 64; }
  int KSL() const { return 64 / MS; }                 // reduction rows one MFMA consumes
  bool halo() const { return BV == kModeHalo || BV == kModeHaloFlat; }
  // input cells of one LDS plane that the workgroup's threads can stage
  long long cell_capacity(int bv) const {
    return BV == kModeHaloFlat ? NTHR() / EPT : (long long)EPT * NTHR() * bv;
  }
};

static const TileDesc kTileDescs[] = {
#define X(name, R, S, STR, WM, WN, MT, NT, KR, EPT, AV, KS, BV, PD, WPE, MS) \
  {#name, R, S, STR, WM, WN, MT, NT, KR, EPT, AV, KS, BV, PD, WPE, MS},
#include "variants.def"
#undef X
};
constexpr int kNumTiles = (int)(sizeof(kTileDescs) / sizeof(kTileDescs[0]));

struct Plan {
  TconvParams p;
  unsigned gx, gy, gz;
  size_t lds_bytes;
  size_t ws_bytes;
};

// Fills the argument block (pointers left null) and launch geometry of tile v
// for shape s0, or returns false if the tile cannot run the shape.
inline bool plan_tconv(const Shape& s0, const TileDesc& v, int nsplit, Plan* pl) {
  Shape s = s0;
  if ((v.R && v.R != s.R) || (v.S && v.S != s.S) || (v.STR && v.STR != s.stride)) return false;
  if (!v.S && s.S > kSmaxGeneric) return false;
  if (v.AV == 4 && ((long long)s.C * s.R * s.S) % 4 != 0) return false;
  const long long i31 = (1LL << 31) - 1;
  // the kernel addresses both inputs through 32-bit byte offsets below 2 GiB
  const long long gbias = (long long)s.pad * s.W + s.pad;
  if (((long long)s.N * s.C * s.H * s.W + gbias) * 4 > i31 || (long long)s.K * s.C * s.R * s.S * 4 > i31)
    return false;
  if ((long long)s.N * s.C * s.H * s.W > i31 || (long long)s.K * s.C * s.R * s.S > i31 ||
      (long long)s.N * s.K * s.P * s.Q > i31)
    return false;
  // A pointwise layer reads each image as one long row (per-image im2col is the
  // identity, paper Section VI k1conv).
  const bool flat = (s.R == 1 && s.S == 1 && s.stride == 1 && s.pad == 0);
  if (flat) {
    s.W = s.H * s.W;
    s.H = 1;
    s.Q = s.P * s.Q;
    s.P = 1;
  }
  // 16-byte input loads: only for flattened pointwise layers whose images are a
  // multiple of four pixels long, so that no group of four pixels straddles images
  if (v.BV == kModeCompact4 && !(flat && s.W % 4 == 0)) return false;
  // the no-padding form of slot staging: nothing to mask per kernel row (and no pointwise cells)
  if (v.BV == kModeSlotsNoPad && (s.pad != 0 || (s.S == 1 && s.stride == 1))) return false;
  // halo staging needs kernel sizes fixed at compile time, a kernel wider than one
  // column or a stride, and half-chunks / reduction groups made of whole channels
  if (v.halo() &&
      !(v.R > 0 && v.S > 0 && v.STR > 0 && !(s.S == 1 && s.stride == 1) && (v.KR / v.KSL()) % v.R == 0 &&
        (v.KR / v.KSL() / v.KS) % v.R == 0))
    return false;
  if (v.BV == kModeHaloFlat && !(v.NTHR() % v.EPT == 0 && (v.KR / v.R) % v.EPT == 0)) return false;
  TconvParams& p = pl->p;
  std::memset(&p, 0, sizeof(p));
  p.N = s.N; p.C = s.C; p.H = s.H; p.W = s.W; p.K = s.K; p.R = s.R; p.S = s.S;
  p.stride = s.stride; p.pad = s.pad; p.P = s.P; p.Q = s.Q;
  p.PQ = s.P * s.Q;
  p.NPQ = s.N * p.PQ;
  p.HW = s.H * s.W;
  p.CHW = s.C * p.HW;
  p.CRS = s.C * s.R * s.S;
  p.CRrows = s.C * s.R;
  p.out_elems = s.N * s.K * p.PQ;
  p.filter_major = (long long)s.K * s.C * s.R * s.S > (long long)s.N * s.C * s.H * s.W ? 1 : 0;
  p.fdQ = make_fastdiv((unsigned)p.Q);
  p.fdP = make_fastdiv((unsigned)p.P);
  const int BN = v.BN(), BM = v.BM();
  long long total_rows = (long long)s.N * s.P;
  p.gbias = s.pad * s.W + s.pad;
  p.compact = (s.S == 1 && s.stride == 1) ? 1 : 0;
  p.bv = (p.compact && v.BV == kModeCompact4) ? 4 : 1;
  p.halo = v.halo() ? 1 : 0;
  int planes = v.KR;                 // LDS planes per input buffer
  if (p.halo) {
    p.hp = s.H + 2 * s.pad;
    p.wt = s.W + 2 * s.pad;
    p.phst = (p.wt + s.stride - 1) / s.stride;
    p.rowst = s.stride * p.phst;
    p.fdHp = make_fastdiv((unsigned)p.hp);
    p.nrows = 0;
    p.vr = 0;
    const int ntiles = (p.NPQ + BN - 1) / BN;
    for (int ti = 0; ti < ntiles; ++ti) {
      HaloTile ht = halo_tile(p, pix_tile(ti, BN, p.NPQ, p.Q, p.fdQ));
      if (ht.vr > p.vr) p.vr = ht.vr;
    }
    p.nrows = p.vr;
    planes = v.KR / s.R;
  } else if (p.compact) {
    p.nrows = 1;
    p.phst = BN;
    p.rowst = BN;
  } else {
    p.nrows = tile_nrows(BN, s.Q, total_rows > i31 ? (int)i31 : (int)total_rows);
    p.phst = tile_phst(BN, s.Q, s.S, s.stride);
    p.rowst = s.stride * p.phst;
  }
  p.plane = p.nrows * p.rowst;
  p.fdRowst = make_fastdiv((unsigned)p.rowst);
  if (!p.halo) p.fdHp = make_fastdiv(1);
  if ((long long)p.nrows * p.rowst > v.cell_capacity(p.bv)) return false;
  p.ast = a_row_stride(v.KR * s.S, a_read_width(v.KR, v.S, v.KS, v.KSL()));
  size_t lds = (size_t)(2 * BM * p.ast + 2 * (planes * p.plane + kLdsTrashWords) + kLdsTrashWords) * sizeof(float);
  if (v.KS > 1 && lds < (size_t)BM * BN * sizeof(float)) lds = (size_t)BM * BN * sizeof(float);
  if (lds > kLdsLimitBytes) return false;
  p.nchunks = (p.CRrows + v.KR - 1) / v.KR;
  if (nsplit < 1 || nsplit > p.nchunks) return false;
  p.chunks_per_split = (p.nchunks + nsplit - 1) / nsplit;
  // no empty split: the request must be reproduced by its own chunk count
  if ((p.nchunks + p.chunks_per_split - 1) / p.chunks_per_split != nsplit) return false;
  p.nsplit = nsplit;
  long long gx = (p.NPQ + BN - 1) / BN, gy = (s.K + BM - 1) / BM;
  if (gx > i31 || gy > 65535 || nsplit > 65535) return false;
  pl->gx = (unsigned)gx;
  pl->gy = (unsigned)gy;
  pl->gz = (unsigned)nsplit;
  pl->lds_bytes = lds;
  pl->ws_bytes = nsplit > 1 ? (size_t)nsplit * (size_t)p.out_elems * sizeof(float) : 0;
  return true;
}

}  // namespace bconv
