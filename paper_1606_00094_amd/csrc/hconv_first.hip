// Half-precision first layers on the fp16 matrix cores: few input channels (C <= 3), a kernel
// several times wider than its stride (11x11 step 4, 7x7 step 2) -- the shape class the paper's
// Section VI gives its tiled-convolution variant (kernel sizes 2 .. ~11, whole rows of the input
// tile held locally, the kernel's X extent unrolled).  With three channels there are no channel
// octets to feed v_mfma_f32_32x32x16_f16, so here the MFMA's 16 reduction slots run along the
// KERNEL ROW: a step is one (channel, kernel row) with the S columns in slots 0..S-1 and zeros
// in the rest (S > 8), or two (channel, kernel row) pairs of S <= 8 columns each, one per lane
// half.  A lane's B operand for pixel (p, q) is then 8 consecutive input elements of one image
// row starting at column q*stride (+8 for the upper lane half when S > 8): contiguous in a
// row-major tile, at an alignment of 2*stride bytes.
//
//   * Input: NCHW rows are 2-byte aligned at best (odd widths), and 2-byte loads are what made
//     the NCHW staging of the other fp16 tiles slow.  A small kernel first writes a padded copy
//     [N][C][H+2pad][WP] (zero borders, row pitch WP a multiple of eight elements and long enough
//     for the last pixel's 16 slots): the paper's "input transformation ... to improve memory
//     access patterns".  The main kernel stages whole rows of that copy with 16-byte loads.
//   * Filters: re-laid into lane order [32-filter block][step][lane][8], zeros in unused slots.
//     A wave keeps the operands of ITS 32 filters for all steps in registers (33 steps x 4
//     registers for 11x11x3) for the whole launch, so LDS serves only the input operand.
//   * A workgroup is one wave per 32 filters (up to four); it walks pixel tiles of NT*32 pixels
//     of one image (persistent: grid-stride over the tile list), staging the next tile's rows
//     into the other LDS buffer while it multiplies the current one.
// Arithmetic as in the other fp16 tiles: exact fp16 x fp16 products, fp32 sums, bias and ReLU
// in fp32, one rounding.  Output NCHW, or octet-interleaved (C8) for a chain that continues on
// the channel-octet tiles; the 2-byte stores of the NCHW form are what limits it (a plane of
// odd size allows nothing wider), the C8 form stores 8 bytes per lane.
#include <atomic>
#include <cstdint>
#include <cstring>

#include "bconv_internal.h"

namespace bconv {

typedef _Float16 fl_half8 __attribute__((ext_vector_type(8)));
typedef float fl_acc __attribute__((ext_vector_type(16)));
typedef unsigned fl_quad __attribute__((ext_vector_type(4)));
typedef unsigned fl_pair __attribute__((ext_vector_type(2)));

#ifndef HFL_PF
#define HFL_PF 2
#endif
constexpr int kFlCmax = 3;       // channels the unrolled step list covers
constexpr int kFlUnits = 12;     // 16-byte staging units per thread and tile, at most

struct HflParams {
  const _Float16* xpad;    // padded copy [N][C][HP][WP]
  const _Float16* apack;   // [K32][STEPS][64][8]
  const float* bias;       // may be null
  _Float16* out;           // N x K x P x Q
  int N, C, K, P, Q, PQ, HP, WP, NR;
  int tiles_per_img, ntiles, units;   // units: 16-byte units of one staged tile, C*NR*WP/8
  int relu;
  unsigned xpad_bytes, apack_bytes;
  FastDiv fdQ, fdTpi, fdRowUnits, fdNR;
};

// LDS byte offset of (channel, kernel row) = flattened index cr in a staged tile
template <int R_>
__device__ __forceinline__ int fl_row_off(int cr, int nr, int wp) {
  const int c = cr / R_, r = cr % R_;
  return (c * nr + r) * wp * 2;
}

// FULLC: the layer has all kFlCmax channels, so every step of the unrolled list is used and the
// step loop has no branches (with them each step is a basic block of its own and the waits on
// the LDS operands can no longer be counted past the block's end).
template <int R_, int S_, int STR_, int NT, bool C8O, bool FULLC>
__global__ __launch_bounds__(256)
void hfl_kernel(const HflParams p) {
  static_assert(S_ <= 16 && STR_ >= 2 && (STR_ & (STR_ - 1)) == 0, "slots along the kernel row");
  constexpr bool WIDE = S_ > 8;                         // one (c, r) per step, two octets
  constexpr int CR = kFlCmax * R_;
  constexpr int STEPS = WIDE ? CR : (CR + 1) / 2;
  constexpr int BN = NT * 32;
  extern __shared__ __attribute__((aligned(16))) fl_quad fsm[];   // [2][units]
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nwave = nthr >> 6;
  const int l32 = lane & 31, gq = lane >> 5;
  const int k32 = blockIdx.y * nwave + wave;            // this wave's block of 32 filters
  const int cr_used = FULLC ? kFlCmax * R_ : p.C * R_;

  const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<_Float16*>(p.apack), 0, p.apack_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<_Float16*>(p.xpad), 0, p.xpad_bytes, 0x00020000);

  // ---- this wave's filter operands, all steps, for the whole launch
  fl_half8 a[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s)
    a[s] = __builtin_bit_cast(fl_half8, __builtin_amdgcn_raw_buffer_load_b128(
                                            rsrc_a, (unsigned)(((k32 * STEPS + s) * 64 + lane) * 16), 0, 0));
  float bv[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int k = k32 * 32 + acc_row_32(lane, i);
    bv[i] = (p.bias && k < p.K) ? p.bias[k] : 0.0f;
  }

  // ---- staging items of this thread: unit -> (offset inside a tile of the padded copy, LDS slot)
  int src_rel[kFlUnits];
#pragma unroll
  for (int i = 0; i < kFlUnits; ++i) {
    const int e = tid + i * nthr;
    const int crow = fd_div(e, p.fdRowUnits);            // c * NR + row
    const int u = e - crow * (p.WP >> 3);
    const int c = fd_div(crow, p.fdNR);
    const int row = crow - c * p.NR;
    src_rel[i] = e < p.units ? ((c * p.HP + row) * p.WP + u * 8) * 2 : -1;
  }

  fl_quad rs[kFlUnits];
  auto tile_origin = [&](int t, int* n, int* g0) {
    *n = fd_div(t, p.fdTpi);
    *g0 = (t - *n * p.tiles_per_img) * BN;
  };
  auto load_tile = [&](int t) {
    int n, g0;
    tile_origin(t, &n, &g0);
    const int p0 = fd_div(g0, p.fdQ);
    const unsigned origin = (unsigned)((n * p.C * p.HP + p0 * STR_) * p.WP * 2);   // bytes
#pragma unroll
    for (int i = 0; i < kFlUnits; ++i)
      rs[i] = __builtin_bit_cast(fl_quad, __builtin_amdgcn_raw_buffer_load_b128(
                                              rsrc_x, src_rel[i] >= 0 ? (unsigned)src_rel[i] : 0x80000000u, origin, 0));
  };
  auto store_tile = [&](int buf) {
    fl_quad* B = fsm + buf * p.units;
#pragma unroll
    for (int i = 0; i < kFlUnits; ++i)
      if (src_rel[i] >= 0) B[tid + i * nthr] = rs[i];
  };

  const int t0 = blockIdx.x;
  if (t0 < p.ntiles) {
    load_tile(t0);
    store_tile(0);
  }
  __syncthreads();
  int buf = 0;
  for (int t = t0; t < p.ntiles; t += gridDim.x, buf ^= 1) {
    const int tn = t + gridDim.x;
    const bool more = tn < p.ntiles;
    if (more) load_tile(tn);
    __builtin_amdgcn_sched_barrier(0);

    // ---- this tile: lane pixel offsets
    int n, g0;
    tile_origin(t, &n, &g0);
    const int p0 = fd_div(g0, p.fdQ);
    int lbase[NT], g[NT];
    bool valid[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int gg = g0 + nt * 32 + l32;
      valid[nt] = gg < p.PQ;
      g[nt] = valid[nt] ? gg : p.PQ - 1;
      const int pp = fd_div(g[nt], p.fdQ), q = g[nt] - pp * p.Q;
      lbase[nt] = ((pp - p0) * STR_ * p.WP + q * STR_) * 2 + (WIDE ? gq * 16 : 0);
    }
    const char* B = reinterpret_cast<const char*>(fsm + buf * p.units);

    fl_acc acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[nt][i] = 0.0f;

    // the 16 bytes of an operand in pieces the alignment allows (8 bytes at stride 4, 4 at 2).
    // Slots past the kernel's width hold input columns that belong to the NEXT pixels' windows;
    // their filter slots are zero, but 0 x Inf is NaN, so they are cleared here as well and
    // a non-finite input element reaches exactly the outputs whose window contains it.
    auto read_b = [&](int off) {
      fl_quad v;
      if constexpr (STR_ >= 4) {
        const fl_pair lo = *reinterpret_cast<const fl_pair*>(B + off);
        const fl_pair hi = *reinterpret_cast<const fl_pair*>(B + off + 8);
        v[0] = lo[0]; v[1] = lo[1]; v[2] = hi[0]; v[3] = hi[1];
      } else {
#pragma unroll
        for (int w = 0; w < 4; ++w) v[w] = *reinterpret_cast<const unsigned*>(B + off + 4 * w);
      }
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        // slots 2w, 2w+1 of this lane's octet are columns base + 2w, base + 2w + 1
        const int lo0 = 2 * w, lo1 = (WIDE ? 8 : 0) + 2 * w;       // first column, lane half 0 / 1
        const unsigned m0 = lo0 + 1 < S_ ? 0xffffffffu : (lo0 < S_ ? 0x0000ffffu : 0u);
        const unsigned m1 = lo1 + 1 < S_ ? 0xffffffffu : (lo1 < S_ ? 0x0000ffffu : 0u);
        if (m0 != 0xffffffffu || m1 != 0xffffffffu) v[w] &= (gq ? m1 : m0);
      }
      return __builtin_bit_cast(fl_half8, v);
    };
    constexpr int PF = HFL_PF;
    constexpr int NS = PF + 1;
    fl_half8 b[NS][NT];
    auto read_step = [&](int s, int slot) {
      int roff;
      if constexpr (WIDE) {
        roff = fl_row_off<R_>(s, p.NR, p.WP);
      } else {
        // lane half gq takes (channel, row) pair 2s + gq; past the last pair the filters are zero
        const int cr1 = 2 * s + 1 < CR ? 2 * s + 1 : 2 * s;
        const int o0 = fl_row_off<R_>(2 * s, p.NR, p.WP), o1 = fl_row_off<R_>(cr1, p.NR, p.WP);
        roff = gq ? o1 : o0;
        if (2 * s + 1 >= cr_used) roff = o0;            // a row of a channel that is not staged
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) b[slot][nt] = read_b(lbase[nt] + roff);
    };
    // steps whose (channel, row) pairs all lie past the last channel are skipped (uniformly)
    auto step_used = [&](int s) { return FULLC || (WIDE ? s : 2 * s) < cr_used; };
#pragma unroll
    for (int s = 0; s < PF && s < STEPS; ++s)
      if (step_used(s)) read_step(s, s % NS);
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      if (s + PF < STEPS && step_used(s + PF)) read_step(s + PF, (s + PF) % NS);
      if (step_used(s)) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[s], b[s % NS][nt], acc[nt], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    if (more) store_tile(buf ^ 1);
    // ---- epilogue of this tile
    if constexpr (C8O) {
      // octet-interleaved output [N][K/8][P*Q][8]: registers 4j..4j+3 of a lane are four
      // consecutive filters of one pixel, one 8-byte store; the lane halves complete the octet
      typedef _Float16 half4 __attribute__((ext_vector_type(4)));
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = k32 * 32 + j * 8 + gq * 4;
        if (k < p.K) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            if (valid[nt]) {
              half4 h;
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                float v = acc[nt][4 * j + u] + bv[4 * j + u];
                if (p.relu) v = v > 0.0f ? v : 0.0f;
                h[u] = (_Float16)v;
              }
              *reinterpret_cast<half4*>(p.out + ((size_t)n * p.K + (k - gq * 4)) * p.PQ + (size_t)g[nt] * 8 + gq * 4) = h;
            }
          }
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int k = k32 * 32 + acc_row_32(lane, i);
        if (k < p.K) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            if (valid[nt]) {
              float v = acc[nt][i] + bv[i];
              if (p.relu) v = v > 0.0f ? v : 0.0f;
              p.out[((size_t)n * p.K + k) * p.PQ + g[nt]] = (_Float16)v;
            }
          }
        }
      }
    }
    __syncthreads();
  }
}

// The two re-layouts of a call in one launch (each dependent launch costs about as much as
// either of them).
//
// Blocks below pad_blocks: in NCHW fp16 -> padded copy [N*C][HP][WP], zero borders.  A wave takes
// one padded row at a time: lane i loads elements i, i + 64, ... of the source row (consecutive
// lanes, consecutive 2-byte elements: whole cache lines per load), the row goes through LDS, and
// lanes write it out as 16-byte units.
//
// The other blocks: filt KCRS fp16 -> [K32][STEPS][64 lanes][8]: lane (l32, gq) of a step holds,
// for filter 32*block + l32, columns 8*gq .. 8*gq+7 of (channel, row) pair `step` (S > 8), or
// columns 0..7 of pair 2*step + gq (S <= 8); zeros for columns >= S, pairs >= C*R and filters
// >= K.
struct HflPrepParams {
  const _Float16* in;
  fl_quad* xpad;
  const _Float16* filt;
  _Float16* apack;
  int H, W, HP, WP, pad;
  long long rows;            // N * C * HP
  int K, C, R, S, steps;
  long long pack_total;      // elements of apack
  unsigned pad_blocks;
};

__global__ __launch_bounds__(256)
void hfl_prepare_kernel(const HflPrepParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned short prow[];   // [4 waves][WP]
  if (blockIdx.x >= p.pad_blocks) {
    const bool wide = p.S > 8;
    const long long nthreads = (long long)(gridDim.x - p.pad_blocks) * 256;
    for (long long idx = (long long)(blockIdx.x - p.pad_blocks) * 256 + threadIdx.x; idx < p.pack_total;
         idx += nthreads) {
      const int j = (int)(idx & 7);
      const int lane = (int)((idx >> 3) & 63);
      long long r = idx >> 9;
      const int step = (int)(r % p.steps);
      const int kb = (int)(r / p.steps);
      const int k = kb * 32 + (lane & 31), gq = lane >> 5;
      const int cr = wide ? step : 2 * step + gq;
      const int s = wide ? gq * 8 + j : j;
      _Float16 v = (_Float16)0.0f;
      if (k < p.K && cr < p.C * p.R && s < p.S) v = p.filt[((long long)k * p.C * p.R + cr) * p.S + s];
      p.apack[idx] = v;
    }
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned short* mine = prow + wave * p.WP;
  const int wpu = p.WP >> 3;
  for (long long row = (long long)blockIdx.x * 4 + wave; row < p.rows; row += (long long)p.pad_blocks * 4) {
    const int y = (int)(row % p.HP);
    const long long nc = row / p.HP;
    const int iy = y - p.pad;
    const bool rowok = iy >= 0 && iy < p.H;
    const unsigned short* src = reinterpret_cast<const unsigned short*>(p.in) + (nc * p.H + (rowok ? iy : 0)) * p.W;
    for (int x = lane; x < p.WP; x += 64) {
      const int ix = x - p.pad;
      mine[x] = (rowok && ix >= 0 && ix < p.W) ? src[ix] : (unsigned short)0;
    }
    // (a wave reads back only what it wrote itself, and a wave's LDS operations execute in
    // program order: no workgroup barrier)
    __builtin_amdgcn_wave_barrier();
    for (int u = lane; u < wpu; u += 64)
      p.xpad[row * wpu + u] = *reinterpret_cast<const fl_quad*>(mine + u * 8);
    __builtin_amdgcn_wave_barrier();
  }
}

// ------------------------------------------------------------------ catalogue and planning
struct FlTile {
  const char* name;
  int R, S, STR, NT;
};
#define HFL_TILES(X)             \
  X(h16k11s4_p128, 11, 11, 4, 4) \
  X(h16k11s4_p64, 11, 11, 4, 2)  \
  X(h16k11s4_p32, 11, 11, 4, 1)  \
  X(h16k7s2_p128, 7, 7, 2, 4)    \
  X(h16k7s2_p64, 7, 7, 2, 2)     \
  X(h16k7s2_p32, 7, 7, 2, 1)
static const FlTile kFlTiles[] = {
#define X(name, R, S, STR, NT) {#name, R, S, STR, NT},
    HFL_TILES(X)
#undef X
};
constexpr int kNumFlTiles = (int)(sizeof(kFlTiles) / sizeof(kFlTiles[0]));

struct FlPlan {
  HflParams p;
  unsigned gx, gy, nthr;
  size_t lds_bytes, apack_bytes, xpad_bytes;
  int steps;
};

static bool plan_hfl(int which, const Shape& s, FlPlan* pl) {
  if (which < 0 || which >= kNumFlTiles) return false;
  const FlTile& v = kFlTiles[which];
  if (s.R != v.R || s.S != v.S || s.stride != v.STR || s.C > kFlCmax) return false;
  const long long i31 = (1LL << 31) - 1;
  std::memset(pl, 0, sizeof(*pl));
  HflParams& p = pl->p;
  const int BN = v.NT * 32;
  p.N = s.N; p.C = s.C; p.K = s.K; p.P = s.P; p.Q = s.Q; p.PQ = s.P * s.Q;
  p.HP = s.H + 2 * s.pad;
  // a row must hold the 16 slots of the last pixel; the pitch is a whole number of 16-byte units
  int wp = s.W + 2 * s.pad;
  if (wp < (s.Q - 1) * v.STR + 16) wp = (s.Q - 1) * v.STR + 16;
  p.WP = (wp + 7) / 8 * 8;
  p.tiles_per_img = (p.PQ + BN - 1) / BN;
  const long long ntiles = (long long)p.tiles_per_img * s.N;
  if (ntiles > i31) return false;
  p.ntiles = (int)ntiles;
  // output rows a tile can span, hence input rows staged per channel
  int span = 1;
  for (int t = 0; t < p.tiles_per_img; ++t) {
    const int g0 = t * BN, g1 = (g0 + BN < p.PQ ? g0 + BN : p.PQ) - 1;
    const int sp = g1 / s.Q - g0 / s.Q + 1;
    if (sp > span) span = sp;
  }
  p.NR = (span - 1) * v.STR + v.R;
  const long long units = (long long)s.C * p.NR * (p.WP / 8);
  const int nwave = s.K >= 128 ? 4 : (s.K + 31) / 32;
  pl->nthr = (unsigned)nwave * 64;
  if (units > (long long)kFlUnits * pl->nthr) return false;
  p.units = (int)units;
  pl->lds_bytes = (size_t)2 * units * 16;
  if (pl->lds_bytes > kLdsLimitBytes) return false;
  const bool wide = v.S > 8;
  pl->steps = wide ? kFlCmax * v.R : (kFlCmax * v.R + 1) / 2;
  const int k32 = (s.K + 31) / 32;
  const int gy = (k32 + nwave - 1) / nwave;
  if (gy > 65535) return false;
  pl->apack_bytes = (size_t)gy * nwave * pl->steps * 64 * 16;
  const long long xb = (long long)s.N * s.C * p.HP * p.WP * 2;
  // (a tile's origin plus its last unit must stay a 32-bit byte offset)
  if (xb + (long long)kFlCmax * p.HP * p.WP * 2 > i31 || (long long)s.N * s.K * p.PQ > i31) return false;
  pl->xpad_bytes = (size_t)xb;
  p.xpad_bytes = (unsigned)xb;
  p.apack_bytes = (unsigned)pl->apack_bytes;
  p.fdQ = make_fastdiv((unsigned)s.Q);
  p.fdTpi = make_fastdiv((unsigned)p.tiles_per_img);
  p.fdRowUnits = make_fastdiv((unsigned)(p.WP / 8));
  p.fdNR = make_fastdiv((unsigned)p.NR);
  // persistent workgroups: one per compute unit (a wave holds most of a register file's worth
  // of filters, so no second workgroup fits beside it)
  int per_cu = 1;
  long long gx = 256LL * per_cu / gy;
  if (gx < 1) gx = 1;
  if (gx > ntiles) gx = ntiles;
  pl->gx = (unsigned)gx;
  pl->gy = (unsigned)gy;
  return true;
}

static size_t fl_align(size_t b) { return (b + 255) & ~(size_t)255; }

int hfl_num_variants() { return kNumFlTiles; }
const char* hfl_variant_name(int which) { return kFlTiles[which].name; }
bool hfl_applicable(int which, const Shape& s) {
  FlPlan pl;
  return plan_hfl(which, s, &pl);
}
size_t hfl_workspace_bytes(int which, const Shape& s) {
  FlPlan pl;
  return plan_hfl(which, s, &pl) ? fl_align(pl.apack_bytes) + pl.xpad_bytes : 0;
}

long long hfl_tiles(int which, const Shape& s) {
  FlPlan pl;
  return plan_hfl(which, s, &pl) ? pl.p.ntiles : 0;
}

template <typename KernelT>
static hipError_t fl_launch(KernelT kernel, const FlPlan& pl, hipStream_t st, std::atomic<size_t>* allowed) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (pl.lds_bytes > 32768 && pl.lds_bytes > allowed[dev].load(std::memory_order_relaxed)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)pl.lds_bytes);
    if (e != hipSuccess) { (void)hipGetLastError(); return e; }
    allowed[dev].store(pl.lds_bytes, std::memory_order_relaxed);
  }
  return launch_kernel(kernel, dim3(pl.gx, pl.gy), dim3(pl.nthr), pl.lds_bytes, st, pl.p);
}

#define X(name, R, S, STR, NT)                                                             \
  static hipError_t fl_launch_##name(const FlPlan& pl, int out_c8, hipStream_t st) {       \
    static std::atomic<size_t> allowed[4][64];                                             \
    if (pl.p.C == kFlCmax)                                                                 \
      return out_c8 ? fl_launch(hfl_kernel<R, S, STR, NT, true, true>, pl, st, allowed[1])   \
                    : fl_launch(hfl_kernel<R, S, STR, NT, false, true>, pl, st, allowed[0]); \
    return out_c8 ? fl_launch(hfl_kernel<R, S, STR, NT, true, false>, pl, st, allowed[3])  \
                  : fl_launch(hfl_kernel<R, S, STR, NT, false, false>, pl, st, allowed[2]); \
  }
HFL_TILES(X)
#undef X
typedef hipError_t (*FlLaunchFn)(const FlPlan&, int, hipStream_t);
static FlLaunchFn fl_table(int which) {
  static const FlLaunchFn table[] = {
#define X(name, R, S, STR, NT) fl_launch_##name,
      HFL_TILES(X)
#undef X
  };
  return table[which];
}

hipError_t launch_hfl(int which, const void* in, const void* filt, const float* bias, void* out, const Shape& s,
                      int relu, int out_c8, void* ws, hipStream_t st) {
  FlPlan pl;
  if (!plan_hfl(which, s, &pl)) return hipErrorInvalidValue;
  if (out_c8 && s.K % 8 != 0) return hipErrorInvalidValue;
  _Float16* apack = static_cast<_Float16*>(ws);
  fl_quad* xpad = reinterpret_cast<fl_quad*>(static_cast<char*>(ws) + fl_align(pl.apack_bytes));
  {
    HflPrepParams pp;
    pp.in = static_cast<const _Float16*>(in);
    pp.xpad = xpad;
    pp.filt = static_cast<const _Float16*>(filt);
    pp.apack = apack;
    pp.H = s.H; pp.W = s.W; pp.HP = pl.p.HP; pp.WP = pl.p.WP; pp.pad = s.pad;
    pp.rows = (long long)s.N * s.C * pl.p.HP;
    pp.K = s.K; pp.C = s.C; pp.R = s.R; pp.S = s.S; pp.steps = pl.steps;
    pp.pack_total = (long long)(pl.apack_bytes / 2);
    long long pad_blocks = (pp.rows + 3) / 4;
    if (pad_blocks > 8192) pad_blocks = 8192;
    long long pack_blocks = (pp.pack_total + 255) / 256;
    if (pack_blocks > 256) pack_blocks = 256;
    pp.pad_blocks = (unsigned)pad_blocks;
    hipError_t e = launch_kernel(hfl_prepare_kernel, dim3((unsigned)(pad_blocks + pack_blocks)), dim3(256),
                                 (size_t)4 * pl.p.WP * 2, st, pp);
    if (e != hipSuccess) return e;
  }
  pl.p.xpad = reinterpret_cast<const _Float16*>(xpad);
  pl.p.apack = apack;
  pl.p.bias = bias;
  pl.p.out = static_cast<_Float16*>(out);
  pl.p.relu = relu;
  return fl_table(which)(pl, out_c8, st);
}

}  // namespace bconv
