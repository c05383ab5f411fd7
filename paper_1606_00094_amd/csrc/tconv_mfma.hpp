// Tiled MFMA forward convolution for gfx950 (CDNA4), fp32 arithmetic; tensors stored as
// fp32 or, with T = _Float16, as half floats widened on their way into LDS.
//
// One workgroup computes BM filters x BN consecutive output pixels.  The main
// loop has the shape of the paper's SGEMM template (Section V: barrier,
// cooperative global->local loads, barrier, unrolled local->register loads and
// multiply-adds) with the register-tile FMAs replaced by
// v_mfma_f32_32x32x2_f32 and the right-hand operand never materialised: as in
// the paper's tiled-convolution variant (Section VI) whole pieces of input rows
// are staged in LDS and the S kernel columns are S shifted LDS reads of the
// same staged row, so global traffic for the input is not multiplied by S.
// A 1x1 layer (the paper's k1conv case) is the same kernel with R = S = 1, the
// host having flattened each image to one row of H*W pixels.
//
// Reduction order inside a chunk of KR reduction rows kk = c*R + r: row i of the
// first half of the chunk and row KR/2 + i of the second half feed the two
// k-slices of one MFMA (lanes 0-31 carry the first, lanes 32-63 the second),
// kernel column s innermost.  With this pairing the filter words one lane needs
// during a chunk are contiguous both in HBM and in LDS, so they are fetched with
// 16-byte global loads, stored with 16-byte LDS writes and read back with
// 16-byte LDS reads.
//
// The matrix pipe is the only unit with real work; what limits the kernel is the
// number of other instructions a wave has to issue per MFMA.  Hence: buffer loads
// whose out-of-range lanes return zero (no selects for padding and tails), wide
// LDS accesses for the filter operand, tap offsets as immediates, (c, r) of a
// reduction row resolved at compile time where the chunk holds whole channels,
// scalar addressing of the loads (per-lane offsets fixed before the loop), and a
// hand-made software pipeline: while chunk i is consumed from one LDS buffer, the
// global loads of chunk i+PD are issued between the MFMAs of the first steps and
// the LDS stores of chunk i+1 (into the other buffer) between the MFMAs of the
// last steps; one barrier per chunk.  BV selects how the input is staged (row
// slots, one cell per pixel for S = 1 stride 1, or halo: each input row of a
// channel once, shared by all kernel rows); PD is the number of register sets.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "bconv_plan.h"

namespace bconv {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

template <int VW> struct VecOf;
template <> struct VecOf<1> { typedef float type; };
template <> struct VecOf<2> { typedef floatx2 type; };
template <> struct VecOf<4> { typedef floatx4 type; };

// Calls f(std::integral_constant<int, I>{}) for I = BEGIN .. END-1, each call its own
// instantiation.
template <int BEGIN, int END, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (BEGIN < END) {
    f(std::integral_constant<int, BEGIN>{});
    static_for<BEGIN + 1, END>(static_cast<F&&>(f));
  }
}
constexpr int cdiv_c(int a, int b) { return (a + b - 1) / b; }

// R_/S_/STR_ > 0: compile-time kernel height / width / stride (tap offsets become
// instruction immediates); 0: taken from the argument block at run time, with
// S <= kSmaxGeneric.  AV = 4: filter rows are fetched with 16-byte loads (the host
// guarantees CRS % 4 == 0 and a 16-byte aligned filter pointer; KR*S % 4 == 0
// holds by construction); AV = 1: 4-byte loads, no alignment demand.
//
// WPE > 1 asks the compiler to fit the kernel's registers for that many waves per
// SIMD (a first-layer tile that just misses three waves otherwise runs its
// workgroups in one and a half rounds).
//
// KS > 1 splits the reduction inside the workgroup: KS groups of WM*WN waves share
// the staged tiles, group g consuming row pairs [g*NPAIR, (g+1)*NPAIR) of every
// chunk, and their accumulators are summed through LDS before the epilogue.
//
// T is the storage type of input, filters and output (float, or _Float16: the paper's
// Section VII outlook of half-precision storage with the arithmetic left in fp32).  Half
// elements are loaded with 2- and 8-byte accesses in place of 4 and 16, kept as raw bits
// in the staging registers and widened when they are stored to LDS; LDS, the MFMAs and
// the partial sums of a split reduction are fp32 either way; the result is rounded to
// T (to nearest even) once, after bias and ReLU.
//
// MS is the edge of one accumulator tile: 32 (v_mfma_f32_32x32x2_f32, two reduction rows per
// instruction) or 16 (v_mfma_f32_16x16x4_f32, four).  Both run at the same rate; the small
// tile quarters the work of one wave-tile, so that a layer with few output points (batch 1)
// still cuts into enough workgroups to fill the chip in ONE kernel, the reduction split over
// the KS wave groups of a workgroup instead of over the grid with partial sums in HBM.
// Everywhere below "pair" means the KSL = 64 / MS reduction rows one MFMA consumes: lane slice
// h = lane / MS takes row h * (KR / KSL) + i of the chunk.
template <int R_, int S_, int STR_, int WM, int WN, int MT, int NT, int KR, int EPT, int AV, int KS, int BV, int PD, int WPE,
          int MS = 32, typename T = float>
__global__ __launch_bounds__(WM * WN * KS * 64, WPE)
void tconv_mfma_kernel(const TconvParams p) {
  constexpr int NW = WM * WN;              // waves per reduction group
  constexpr int NTHR = NW * KS * 64;
  static_assert(MS == 32 || MS == 16, "accumulator tiles are 32x32 or 16x16");
  constexpr int KSL = 64 / MS;             // reduction rows per MFMA
  constexpr int ACCN = MS * MS / 64;       // accumulator registers per tile and lane
  static_assert(KR % KSL == 0, "reduction rows are consumed KSL at a time");
  static_assert((KR / KSL) % KS == 0, "row groups of a chunk must divide among the reduction groups");
  constexpr int NPAIR = KR / KSL / KS;     // row groups per chunk and reduction group
  constexpr int BM = WM * MT * MS, BN = WN * NT * MS;
  constexpr int SP = S_ > 0 ? S_ : kSmaxGeneric;   // filter columns per reduction row (bound)
  constexpr int KRSP = KR * SP;
  static_assert(AV == 1 || (AV == 4 && S_ > 0 && KRSP % 4 == 0), "vector filter loads need KR*S % 4 == 0");
  constexpr int AGRP = KRSP / AV;                      // load groups per filter row
  constexpr int NA = (BM * AGRP + NTHR - 1) / NTHR;    // filter load items per thread
  // BV is the input staging mode: kModeSlots, kModeSlotsNoPad, kModeCompact4, kModeHalo or
  // kModeHaloFlat
  constexpr bool HFLAT = (BV == kModeHaloFlat);
  constexpr bool HALO = (BV == kModeHalo) || HFLAT;
  constexpr int BVW = (BV == kModeCompact4) ? 4 : 1;   // words per input load
  static_assert(BV == kModeSlots || BV == kModeSlotsNoPad || BV == kModeCompact4 || HALO,
                "unknown staging mode");
  static_assert(BV != kModeCompact4 || (S_ == 1 && STR_ == 1), "16-byte input loads are for pointwise tiles");
  static_assert(!HALO || (R_ > 0 && S_ > 0 && STR_ > 0 && (KR / KSL) % (R_ > 0 ? R_ : 1) == 0 &&
                          (KR / KSL / KS) % (R_ > 0 ? R_ : 1) == 0),
                "halo staging needs whole channels per chunk part and reduction group");
  constexpr int RDIV = R_ > 0 ? R_ : 1;
  constexpr int NPL = HALO ? KR / RDIV : KR;           // LDS planes per input buffer
  // Flat staging (pointwise tiles whose pixel tile has fewer cells than the workgroup
  // has threads): every thread owns one cell and stages it for the planes
  // kl0, kl0 + PSTEP, ... with kl0 = tid / CPP, so that no thread issues masked loads.
  constexpr int CPP = BN / BVW;                        // cells per plane of a pointwise tile
  constexpr bool PFLAT = !HALO && R_ == 1 && S_ == 1 && STR_ == 1 && CPP < NTHR && NTHR % CPP == 0 &&
                         KR % (NTHR / CPP) == 0;
  // The same for a halo tile with few cells per channel plane (kModeHaloFlat): EPT thread
  // groups of NTHR / EPT threads, group g staging planes g, g + EPT, ... of the chunk.
  static_assert(!HFLAT || (NTHR % EPT == 0 && NPL % EPT == 0), "plane groups must divide threads and planes");
  constexpr bool FLAT = PFLAT || HFLAT;
  constexpr int PSTEP = PFLAT ? NTHR / CPP : (HFLAT ? EPT : 1);
  constexpr int FCELLS = PFLAT ? CPP : (HFLAT ? NTHR / EPT : 1);   // cells per plane under flat staging
  constexpr int NCELL = FLAT ? 1 : EPT;                // staged cells per thread and plane
  constexpr int NB = FLAT ? NPL / PSTEP : NPL * EPT;   // input load items per thread (BVW words each)
  constexpr int NL = NA + NB;
  constexpr int VW = a_read_width(KR, S_, KS, KSL);    // words per LDS read of the filter operand
  constexpr int SW = (AV == 4) ? VW : 1;               // words per LDS store of the filter operand
  constexpr bool WHOLE_CH = R_ > 0 && (KR % (R_ > 0 ? R_ : 1)) == 0;   // chunks hold whole channels
  // Scalar addressing: a load's per-lane offset is a register computed once before the
  // loop, and everything that changes from chunk to chunk (channel, kernel row, "past
  // the end") goes into the scalar offset and the descriptor's size.  No vector
  // instruction then writes a register that a load also writes, so the compiler needs
  // no wait on loads in flight before it issues the next ones.
  constexpr bool A_SCALAR = NA <= 12;                  // one offset register per filter item
  // (slot staging qualifies when the layer has no padding: a cell that loads at all loads for
  // every kernel row, so its validity does not change from chunk to chunk)
  constexpr bool B_SCALAR = HALO || (R_ == 1 && S_ == 1 && STR_ == 1) || BV == kModeSlotsNoPad;
  typedef typename VecOf<VW>::type avec_t;
  typedef typename VecOf<SW>::type svec_t;
  static_assert(sizeof(T) == 4 || sizeof(T) == 2, "fp32 or fp16 storage");
  constexpr int ESZ = sizeof(T);                       // bytes per stored element
  constexpr bool F16 = ESZ == 2;
  constexpr int AVR = F16 ? (AV + 1) / 2 : AV;         // 32-bit registers per filter load item
  constexpr int BVR = F16 ? (BVW + 1) / 2 : BVW;       // and per input load item

  const int R = R_ > 0 ? R_ : p.R;
  const int S = S_ > 0 ? S_ : p.S;
  const int STR = STR_ > 0 ? STR_ : p.stride;
  const int KRS = KR * S;            // valid filter words per row per chunk
  const int HALF = (KR / KSL) * S;   // words of one lane slice's part of a filter row
  const int RUN = NPAIR * S;         // words of this group's run inside a half-chunk
  const int ast = S_ > 0 ? a_row_stride(KR * (S_ > 0 ? S_ : 1), VW) : p.ast;
  const int plane = p.plane;
  const int phst = p.phst;

  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int abuf = BM * ast;
  const int bbuf = NPL * plane + kLdsTrashWords;   // each input buffer ends in its own trash words
  float* const trash = smem;                       // kLdsTrashWords words nobody reads
  float* const As = smem + kLdsTrashWords;         // [2][BM][ast]
  float* const Bs = As + 2 * abuf;                 // [2][KR][nrows][rowst] (+ trash)

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int kgrp = wave / NW;
  const int wv = wave - kgrp * NW;
  const int wm = wv / WN, wn = wv % WN;
  const int l32 = lane & (MS - 1), h = lane / MS;     // row / column inside the tile, lane slice

  const BlockTile bt = xcd_tile(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), gridDim.x,
                                gridDim.y, gridDim.z, p.filter_major);
  const PixTile t = pix_tile(bt.x, BN, p.NPQ, p.Q, p.fdQ);
  const HaloTile ht = HALO ? halo_tile(p, t) : HaloTile{0, 0};
  const int m0 = bt.y * BM;

  // ---- per-thread staging cells of the input tile (fixed for the whole loop)
  int c_lds[NCELL], c_pl[NCELL], c_goff[NCELL], c_ih0[NCELL];
  const int ncell = p.nrows * p.rowst;
  const int kl0 = FLAT ? tid / FCELLS : 0;
#pragma unroll
  for (int i = 0; i < NCELL; ++i) {
    int e = FLAT ? tid - kl0 * FCELLS : tid + i * NTHR;
    const bool in_tile = e * BVW < ncell;
    BCell c = HALO ? h_cell(p, ht, in_tile ? e : 0, STR) : b_cell(p, t, in_tile ? e : 0, S, STR);
    // LDS word offset from Bs of the cell in plane 0 and the plane stride to add per
    // reduction row; a cell outside the tile writes to the trash words (stride 0)
    c_lds[i] = in_tile ? c.lds : NPL * plane;
    c_pl[i] = in_tile ? plane : 0;
    c_ih0[i] = in_tile ? c.ih0 : kNeverValid;
    // byte offset from the biased descriptor base; in halo mode a cell's validity
    // does not depend on the kernel row, so it is folded into the offset here
    const bool never = HALO ? (c_ih0[i] == kNeverValid)
                            : (B_SCALAR && (unsigned)c_ih0[i] >= (unsigned)p.H);
    c_goff[i] = never ? (int)0x80000000u : (c.goff + p.gbias) * ESZ;
    if constexpr (FLAT) {
      // this thread's first plane folded into both offsets (the marker stays out of range)
      c_goff[i] += kl0 * p.HW * ESZ;
      c_lds[i] += kl0 * c_pl[i];
    }
  }

  // ---- per-lane operand bases
  int laneB[NT], outoff[NT], colvalid[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    BLane bl = HALO ? h_lane(p, t, ht, (wn * NT + nt) * MS + l32) : b_lane(p, t, (wn * NT + nt) * MS + l32);
    laneB[nt] = bl.ldsbase + (HALO ? (h * (KR / KSL) + kgrp * NPAIR) / RDIV : h * (KR / KSL) + kgrp * NPAIR) * plane;
    outoff[nt] = bl.outoff;
    colvalid[nt] = bl.valid;
  }
  const int laneA = (wm * MT * MS + l32) * ast + h * HALF + kgrp * RUN;

  typedef float acc_t __attribute__((ext_vector_type(ACCN)));
  acc_t acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int i = 0; i < ACCN; ++i) acc[mt][nt][i] = 0.0f;

  const bool split = p.nsplit > 1;
  // bias through a buffer descriptor that is empty when there is none to add (no bias,
  // or partial sums): out-of-range loads return 0, so nothing is selected afterwards.
  // A tile with one accumulator tile per wave fetches its 16 values here, ahead of the
  // main loop, so that a workgroup that runs alone (small batches) does not end on an
  // exposed memory round trip; larger tiles keep the registers free and load at the end
  // (64x128 tiles lost 5 % to the 16 extra registers).
  constexpr bool BIAS_EARLY = (MT * NT == 1);
  const __amdgpu_buffer_rsrc_t rsrc_bias = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(p.bias), 0, (!split && p.bias) ? p.K * 4 : 0, 0x00020000);
  float bvals[MT][ACCN];
  auto load_bias = [&]() {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < ACCN; ++i) {
        const int k = m0 + (wm * MT + mt) * MS + acc_row(lane, i, MS);
        bvals[mt][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_bias, k * 4, 0, 0));
      }
  };
  if constexpr (BIAS_EARLY) load_bias();

  const int z = bt.z;
  const int ch_begin = z * p.chunks_per_split;
  int ch_end = ch_begin + p.chunks_per_split;
  if (ch_end > p.nchunks) ch_end = p.nchunks;

  // PD register sets: the words of chunks i+2 .. i+PD are in flight while those of
  // chunk i+1 are being stored to LDS and chunk i is consumed
  static_assert(PD == 2 || PD == 4, "prefetch depth");
  // (half elements stay packed, two to a register, until they are stored to LDS)
  float ra[PD][NA * AVR];
  float rb[PD][NB * BVR];

  // Global loads go through raw buffer descriptors: a load whose offset is out of
  // range returns 0, so zero padding, ragged tails and masked lanes need no select
  // after the load (the loaded registers are not touched until they are stored to
  // LDS, which keeps the memory latency off the wave's critical path).  The input
  // descriptor starts gbias words before the tensor so that cell offsets, which may
  // point above the first image row, are never negative.
  constexpr unsigned kOob = 0x80000000u;
  // sc0 | sc1: the loads are served by L2.  Every word is fetched once per workgroup
  // and goes straight to LDS, so the vector L1 has nothing to reuse, and its in-order
  // handling of requests that hit a line still in flight (neighbouring kernel rows of
  // one channel, filter rows that straddle lines) only stalls the other loads.
  constexpr int kLoadPolicy = 17;
  T* const in_base = reinterpret_cast<T*>(const_cast<float*>(p.in)) - p.gbias;
  T* const filt_base = reinterpret_cast<T*>(const_cast<float*>(p.filt));
  const __amdgpu_buffer_rsrc_t rsrc_in = __builtin_amdgcn_make_buffer_rsrc(
      in_base, 0, (p.N * p.CHW + p.gbias) * ESZ, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_filt = __builtin_amdgcn_make_buffer_rsrc(
      filt_base, 0, p.K * p.CRS * ESZ, 0x00020000);

  // per-lane byte offsets of the filter load items (out-of-range marker where the
  // item lies outside the tile, the filter count or the chunk's row width)
  unsigned a_voff[A_SCALAR ? NA : 1];
  if constexpr (A_SCALAR) {
#pragma unroll
    for (int q = 0; q < NA; ++q) {
      const int e = tid + q * NTHR;
      const int m = e / AGRP;
      const int j = (e - m * AGRP) * AV;
      const bool ok = (((q + 1) * NTHR <= BM * AGRP) || (m < BM)) && (S_ > 0 || j < KRS) && (m0 + m < p.K);
      a_voff[q] = ok ? (unsigned)(((m0 + m) * p.CRS + j) * ESZ) : kOob;
    }
  }
  const unsigned filt_bytes = (unsigned)(p.K * p.CRS * ESZ);
  const unsigned in_bytes = (unsigned)((p.N * p.CHW + p.gbias) * ESZ);
  // the last chunk of the reduction may be narrower than KR rows: its filter words
  // past the end of the row are zeroed in LDS after they are stored
  const bool has_tail = p.nchunks * KR * S > p.CRS;

  // (c, r) of reduction row kl of chunk ch: compile-time r when a chunk holds
  // whole channels, one conditional wrap when a chunk is shorter than a channel.
  auto row_cr = [&](int ch, int kl, int c0, int r0, int& c, int& r) {
    if constexpr (WHOLE_CH) {
      c = ch * (KR / (R_ > 0 ? R_ : 1)) + kl / (R_ > 0 ? R_ : 1);
      r = kl % (R_ > 0 ? R_ : 1);
    } else if constexpr (R_ > 0 && KR <= R_) {
      const bool wrap = (r0 + kl) >= R_;
      c = c0 + (wrap ? 1 : 0);
      r = r0 + kl - (wrap ? R_ : 0);
    } else {
      const int kk = ch * KR + kl;
      c = kk / R;
      r = kk - c * R;
    }
  };

  // Load item q of chunk ch: q < NA is a group of AV filter words, otherwise the
  // input cell (kl, i) = ((q - NA) / EPT, (q - NA) % EPT).
  auto load_item = [&](auto set_tag, int ch, int q, int c0, int r0) {
    constexpr int SET = decltype(set_tag)::value;
    const bool chok = ch < ch_end;      // chunks past this workgroup's range load zeros
    const int kk0 = ch * KR;
    if (q < NA) {
      const int col0 = kk0 * S;
      const int e = tid + q * NTHR;
      const int m = e / AGRP;
      const int j = (e - m * AGRP) * AV;
      // (q + 1) * NTHR <= BM * AGRP folds to true for all but a ragged last item
      const bool inside = ((q + 1) * NTHR <= BM * AGRP) || (m < BM);
      const bool ok = chok && inside && (S_ > 0 || j < KRS) && (m0 + m < p.K) && (col0 + j < p.CRS);
      unsigned voff;
      __amdgpu_buffer_rsrc_t rsrc_a;
      if constexpr (A_SCALAR) {
        voff = a_voff[q];
        // (the range check covers per-lane plus scalar offset, so a lane of the last
        // filter row that would run past the tensor reads 0)
        rsrc_a = __builtin_amdgcn_make_buffer_rsrc(filt_base, 0, chok ? filt_bytes : 0u, 0x00020000);
      } else {
        voff = ok ? (unsigned)(((m0 + m) * p.CRS + j) * ESZ) : kOob;
        rsrc_a = rsrc_filt;
      }
      if constexpr (F16 && AV == 4) {
        floatx2 v = __builtin_bit_cast(
            floatx2, __builtin_amdgcn_raw_buffer_load_b64(rsrc_a, voff, col0 * ESZ, kLoadPolicy));
        ra[SET][q * 2] = v[0];
        ra[SET][q * 2 + 1] = v[1];
      } else if constexpr (F16) {
        ra[SET][q] = __builtin_bit_cast(
            float, (unsigned)(unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rsrc_a, voff, col0 * ESZ, kLoadPolicy));
      } else if constexpr (AV == 4) {
        floatx4 v = __builtin_bit_cast(
            floatx4, __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, voff, col0 * 4, kLoadPolicy));
#pragma unroll
        for (int u = 0; u < 4; ++u) ra[SET][q * 4 + u] = v[u];
      } else {
        ra[SET][q] = __builtin_bit_cast(float,
                                   __builtin_amdgcn_raw_buffer_load_b32(rsrc_a, voff, col0 * 4, kLoadPolicy));
      }
    } else {
      const int kl = FLAT ? (q - NA) * PSTEP : (q - NA) / EPT, i = FLAT ? 0 : (q - NA) % EPT;
      int c, r;
      bool ok;
      if constexpr (HALO) {
        // plane kl is channel ch*NPL + kl; the cell offset already encodes padding.  (Flat
        // halo staging: the thread's own plane kl0 is folded into its offsets and may carry
        // it past the last channel in the last chunk; those cells are zeroed in LDS after
        // the store, as under flat pointwise staging.)
        c = ch * NPL + kl;
        r = 0;
        ok = chok && (c < p.C);
      } else {
        row_cr(ch, kl, c0, r0, c, r);
        ok = chok && (kk0 + kl < p.CRrows) && ((unsigned)(c_ih0[i] + r) < (unsigned)p.H);
      }
      unsigned voff;
      __amdgpu_buffer_rsrc_t rsrc_b;
      if constexpr (B_SCALAR) {
        // what is left of ok is the same for every lane: switch the descriptor off
        // (flat staging: the thread's own plane offset may carry it past the last
        // channel in the last chunk; those cells are zeroed in LDS after the store)
        const bool sok = HALO ? ok : (chok && (kk0 + kl < p.CRrows));
        voff = (unsigned)c_goff[i];
        rsrc_b = __builtin_amdgcn_make_buffer_rsrc(in_base, 0, sok ? in_bytes : 0u, 0x00020000);
      } else {
        voff = ok ? (unsigned)c_goff[i] : kOob;
        rsrc_b = rsrc_in;
      }
      if constexpr (F16 && BVW == 4) {
        floatx2 v = __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(
                                                    rsrc_b, voff, (c * p.HW + r * p.W) * ESZ, kLoadPolicy));
        rb[SET][(q - NA) * 2] = v[0];
        rb[SET][(q - NA) * 2 + 1] = v[1];
      } else if constexpr (F16) {
        rb[SET][q - NA] = __builtin_bit_cast(
            float, (unsigned)(unsigned short)__builtin_amdgcn_raw_buffer_load_b16(
                       rsrc_b, voff, (c * p.HW + r * p.W) * ESZ, kLoadPolicy));
      } else if constexpr (BVW == 4) {
        floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(
                                                    rsrc_b, voff, (c * p.HW + r * p.W) * 4, kLoadPolicy));
#pragma unroll
        for (int u = 0; u < 4; ++u) rb[SET][(q - NA) * 4 + u] = v[u];
      } else {
        rb[SET][q - NA] = __builtin_bit_cast(
            float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_b, voff, (c * p.HW + r * p.W) * 4, kLoadPolicy));
      }
    }
  };

  // element u of the load item whose first register is regs[base]: the fp32 word itself,
  // or half u of the packed pairs widened to fp32 (exact)
  auto element = [&](const auto& regs, int base, int u) -> float {
    if constexpr (F16) {
      const unsigned bits = __builtin_bit_cast(unsigned, regs[base + (u >> 1)]) >> ((u & 1) * 16);
      return (float)__builtin_bit_cast(_Float16, (unsigned short)bits);
    } else {
      return regs[base + u];
    }
  };

  auto store_item = [&](auto set_tag, int buf, int q) {
    constexpr int SET = decltype(set_tag)::value;
    if (q < NA) {
      float* A = As + buf * abuf;
      const int e = tid + q * NTHR;
      const int m = e / AGRP;
      const int j = (e - m * AGRP) * AV;
      // words outside the tile go to the trash words in front of the buffers, so
      // that the store needs no branch
      const bool ok = (((q + 1) * NTHR <= BM * AGRP) || (m < BM)) && (S_ > 0 || j < KRS);
      float* dst = ok ? A + m * ast + j : trash;
#pragma unroll
      for (int u = 0; u < AV; u += SW) {
        svec_t v;
        if constexpr (SW == 1) {
          v = element(ra[SET], q * AVR, u);
        } else {
#pragma unroll
          for (int w = 0; w < SW; ++w) v[w] = element(ra[SET], q * AVR, u + w);
        }
        *reinterpret_cast<svec_t*>(dst + u) = v;
      }
    } else {
      float* B = Bs + buf * bbuf;
      const int kl = FLAT ? (q - NA) * PSTEP : (q - NA) / EPT, i = FLAT ? 0 : (q - NA) % EPT;
      if constexpr (BVW == 4) {
        floatx4 v;
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = element(rb[SET], (q - NA) * BVR, u);
        *reinterpret_cast<floatx4*>(B + kl * c_pl[i] + c_lds[i]) = v;
      } else {
        B[kl * c_pl[i] + c_lds[i]] = element(rb[SET], q - NA, 0);
      }
    }
  };

  // zero the filter words of chunk ch in LDS buffer buf that lie past the end of the
  // filter row (scalar addressing loads them from the next row)
  auto zero_tail = [&](int buf, int ch) {
    if constexpr (FLAT) {
      // flat staging: planes past the last channel were loaded from the next image
      float* B = Bs + buf * bbuf;
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        if (HFLAT ? (ch * NPL + kl0 + j * PSTEP >= p.C) : (ch * KR + kl0 + j * PSTEP >= p.CRrows)) {
#pragma unroll
          for (int u = 0; u < BVW; ++u) B[j * PSTEP * c_pl[0] + c_lds[0] + u] = 0.0f;
        }
      }
    }
    if constexpr (A_SCALAR) {
      float* A = As + buf * abuf;
      const int col0 = ch * KR * S;
#pragma unroll
      for (int q = 0; q < NA; ++q) {
        const int e = tid + q * NTHR;
        const int m = e / AGRP;
        const int j = (e - m * AGRP) * AV;
        const bool ok = (((q + 1) * NTHR <= BM * AGRP) || (m < BM)) && (S_ > 0 || j < KRS);
        if (ok && col0 + j >= p.CRS) {
#pragma unroll
          for (int u = 0; u < AV; ++u) A[m * ast + j + u] = 0.0f;
        }
      }
    }
  };

  // Waves with one accumulator tile raise their priority while they issue a step's MFMA:
  // with several short-step waves per SIMD the matrix pipe then goes to the wave that has
  // its operands rather than to one that is about to stall on staging (1.5-4 % on the 1x1
  // layers and small matrix products, 0-3 % on the other single-tile waves).  Tiles whose
  // waves hold several accumulator tiles run one or two waves per SIMD, have nobody to take
  // priority from, and lost 1-2 % to the two extra instructions.
  constexpr bool MFMA_PRIO = (MT * NT == 1);
  auto mfma_tile = [&](const float (&a)[MT], const float (&b)[NT]) {
    if constexpr (MFMA_PRIO) __builtin_amdgcn_s_setprio(2);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        if constexpr (MS == 32)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
        else
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
    if constexpr (MFMA_PRIO) __builtin_amdgcn_s_setprio(0);
  };

  // One pipeline stage, J = (ch - ch_begin) % PD: consumes chunk ch from LDS buffer
  // J % 2; between its MFMAs the global loads of chunk ch + PD are issued into
  // register set J (free since the previous stage) and register set J + 1 (chunk
  // ch + 1, loaded PD - 1 stages ago) is stored to the other LDS buffer.  Staging
  // work is spread evenly over the steps and needs no conditions: chunks past the
  // end load zeros and are stored to a buffer nobody reads.
  auto stage = [&](auto par_tag, int ch) {
    constexpr int J = decltype(par_tag)::value;
    constexpr int P = J % 2;
    typedef std::integral_constant<int, J> SetLoad;
    typedef std::integral_constant<int, (J + 1) % PD> SetStore;
    const float* A = As + P * abuf;
    const float* B = Bs + P * bbuf;
    const int next = ch + PD;
    int c0 = 0, r0 = 0;
    if constexpr (!WHOLE_CH) {
      c0 = (next * KR) / R;
      r0 = next * KR - c0 * R;
    }
    if constexpr (S_ > 0 && STR_ > 0) {
      constexpr int NSTEPS = NPAIR * (S_ > 0 ? S_ : 1);
      constexpr int LSTEPS = NSTEPS > 1 ? NSTEPS / 2 : 0;   // steps that issue global loads
      // this lane's filter words are read VW at a time, one read ahead of their use
      constexpr int NGRP = (NSTEPS + VW - 1) / VW;
      float areg[2][MT][VW];
      auto read_a = [&](int g, float (&dst)[MT][VW]) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          avec_t v = *reinterpret_cast<const avec_t*>(A + laneA + mt * MS * ast + g * VW);
          if constexpr (VW == 1) {
            dst[mt][0] = v;
          } else {
#pragma unroll
            for (int u = 0; u < VW; ++u) dst[mt][u] = v[u];
          }
        }
      };
      read_a(0, areg[0]);
      // input operands of step st+1 are read from LDS before the MFMAs of step st issue
      float b[2][NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) b[0][nt] = B[laneB[nt]];
      // The steps are instantiated one by one (not a loop the compiler may decline to
      // unroll), so that every register array index and every staging item of a step
      // is a compile-time constant.
      static_for<0, NSTEPS>([&](auto st_tag) {
        constexpr int st = decltype(st_tag)::value;
        if constexpr (st + 1 < NSTEPS) {
          constexpr int i = (st + 1) / (S_ > 0 ? S_ : 1), s = (st + 1) % (S_ > 0 ? S_ : 1);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            b[(st + 1) & 1][nt] =
                B[laneB[nt] + (HALO ? (i / RDIV) * plane + (i % RDIV) * p.rowst : i * plane) +
                  (s % (STR_ > 0 ? STR_ : 1)) * phst + s / (STR_ > 0 ? STR_ : 1)];
        }
        if constexpr (st % VW == 0 && st / VW + 1 < NGRP) read_a(st / VW + 1, areg[(st / VW + 1) & 1]);
        float a[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[mt] = areg[(st / VW) & 1][mt][st % VW];
        mfma_tile(a, b[st & 1]);
        // loads in the first half of the steps, stores in the second half, both spread
        // evenly: the memory counter retires loads in order, so a store waits for every
        // load issued before it except this stage's own; this way those are at least
        // PD - 1 stages old
        constexpr int D = NSTEPS - LSTEPS;
        constexpr int lq0 = LSTEPS ? (st < LSTEPS ? cdiv_c(st * NL, LSTEPS) : NL) : (st == 0 ? 0 : NL);
        constexpr int lq1 = LSTEPS ? (st < LSTEPS ? cdiv_c((st + 1) * NL, LSTEPS) : NL) : NL;
        constexpr int sq0 = st >= LSTEPS ? cdiv_c((st - LSTEPS) * NL, D) : NL;
        constexpr int sq1 = st >= LSTEPS ? cdiv_c((st - LSTEPS + 1) * NL, D) : NL;
        static_for<lq0, lq1>([&](auto q_tag) { load_item(SetLoad{}, next, decltype(q_tag)::value, c0, r0); });
        static_for<sq0, sq1>([&](auto q_tag) { store_item(SetStore{}, 1 - P, decltype(q_tag)::value); });
        // keep the compiler from regrouping the staging work of different steps
        __builtin_amdgcn_sched_barrier(0);
      });
    } else {
#pragma unroll
      for (int q = 0; q < NL; ++q) load_item(SetLoad{}, next, q, c0, r0);
      for (int i = 0; i < NPAIR; ++i) {
        int ph = 0, xq = 0;
        for (int s = 0; s < S; ++s) {
          float a[MT], b[NT];
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) a[mt] = A[laneA + mt * MS * ast + i * S + s];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) b[nt] = B[laneB[nt] + i * plane + ph * phst + xq];
          mfma_tile(a, b);
          if (++ph == STR) { ph = 0; ++xq; }
        }
      }
#pragma unroll
      for (int q = 0; q < NL; ++q) store_item(SetStore{}, 1 - P, q);
    }
    if (has_tail && ch + 1 == p.nchunks - 1) zero_tail(1 - P, ch + 1);
  };

  typedef std::integral_constant<int, 0> Zero;
  auto prologue_load = [&](auto set_tag) {
    constexpr int J = decltype(set_tag)::value;
    const int c0 = ((ch_begin + J) * KR) / R;
    const int r0 = (ch_begin + J) * KR - c0 * R;
#pragma unroll
    for (int q = 0; q < NL; ++q) load_item(set_tag, ch_begin + J, q, c0, r0);
  };
  // prologue: chunks 0 .. PD-1 into the register sets, chunk 0 on into buffer 0
  prologue_load(Zero{});
  prologue_load(std::integral_constant<int, 1>{});
  if constexpr (PD == 4) {
    prologue_load(std::integral_constant<int, 2>{});
    prologue_load(std::integral_constant<int, 3>{});
  }
#pragma unroll
  for (int q = 0; q < NL; ++q) store_item(Zero{}, 0, q);
  if (has_tail && ch_begin == p.nchunks - 1) zero_tail(0, ch_begin);
  __syncthreads();
  // The loop body runs PD stages unconditionally and the remaining 0 .. PD-1 stages
  // follow it.  (A stage guarded by a condition inside the loop would add a path to
  // the control flow graph that skips it and re-enters the loop; that path never
  // runs, but on it a register set would still have loads in flight when the next
  // stage reuses it, and the compiler would make every stage wait for them.)
  {
    const int nst = ch_end - ch_begin;
    int ch = ch_begin;
    for (int it = nst / PD; it > 0; --it, ch += PD) {
      stage(Zero{}, ch);
      __syncthreads();
      stage(std::integral_constant<int, 1>{}, ch + 1);
      __syncthreads();
      if constexpr (PD == 4) {
        stage(std::integral_constant<int, 2>{}, ch + 2);
        __syncthreads();
        stage(std::integral_constant<int, 3>{}, ch + 3);
        __syncthreads();
      }
    }
    const int rem = nst % PD;
    if (rem >= 1) {
      stage(Zero{}, ch);
      __syncthreads();
    }
    if constexpr (PD == 4) {
      if (rem >= 2) {
        stage(std::integral_constant<int, 1>{}, ch + 1);
        __syncthreads();
      }
      if (rem >= 3) {
        stage(std::integral_constant<int, 2>{}, ch + 2);
        __syncthreads();
      }
    }
  }

  // ---- sum the reduction groups' accumulators through LDS (staging buffers are free now)
  if constexpr (KS > 1) {
    float* const red = smem;
    for (int g = 1; g < KS; ++g) {
      __syncthreads();
      if (kgrp == g) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < ACCN; ++i)
              red[(((wv * MT + mt) * NT + nt) * ACCN + i) * 64 + lane] = acc[mt][nt][i];
      }
      __syncthreads();
      if (kgrp == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < ACCN; ++i)
              acc[mt][nt][i] += red[(((wv * MT + mt) * NT + nt) * ACCN + i) * 64 + lane];
      }
    }
  }
  if (KS > 1 && kgrp != 0) return;

  // ---- epilogue: bias + optional ReLU + store (or raw partial sums for split-K;
  // partial tiles are summed by a second kernel: exchanging them inside this one
  // would need a device-scope release/acquire per workgroup, which on this part
  // means writing back and invalidating a whole L2 slice each time)
  if constexpr (!BIAS_EARLY) load_bias();
  // dst: fp32 partial sums of this split, or the output tensor in its storage type
  auto emit = [&](auto* dst) {
    typedef std::remove_pointer_t<decltype(dst)> out_t;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int i = 0; i < ACCN; ++i) {
        const int k = m0 + (wm * MT + mt) * MS + acc_row(lane, i, MS);
        if (k < p.K) {
          const float bv = bvals[mt][i];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            if (colvalid[nt]) {
              float v = acc[mt][nt][i] + bv;
              if (!split && p.relu) v = v > 0.0f ? v : 0.0f;
              dst[outoff[nt] + k * p.PQ] = (out_t)v;
            }
          }
        }
      }
    }
  };
  float* const part = p.partial + (split ? (size_t)z * (size_t)p.out_elems : (size_t)0);
  if constexpr (F16) {
    if (split) emit(part);
    else emit(reinterpret_cast<T*>(p.out));
  } else {
    emit(split ? part : p.out);
  }
}

}  // namespace bconv
