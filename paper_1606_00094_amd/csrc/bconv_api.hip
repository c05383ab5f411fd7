// C ABI of libbconv: argument validation, the variant catalogue, launch planning,
// the per-shape selection (paper Section V: operation -> variant -> blocking
// constants) and the host-only bounds audit.  No arithmetic of the convolution
// is done on the host.
#include <cstdint>
#include <cstdio>
#include <cmath>
#include <cstring>
#include <mutex>
#include <type_traits>
#include <unordered_map>

#include "../../include/bconv.h"
#include "bconv_internal.h"

namespace bconv {

// ------------------------------------------------------------------ catalogue
static const TileLaunchFn kLaunch[] = {
#define X(name, R, S, STR, WM, WN, MT, NT, KR, EPT, AV, KS, BV, PD, WPE, MS) launch_##name,
#include "variants.def"
#undef X
};
// the same tiles for tensors stored in half precision
static const TileLaunchFn kLaunchF16[] = {
#define X(name, R, S, STR, WM, WN, MT, NT, KR, EPT, AV, KS, BV, PD, WPE, MS) launch_f16_##name,
#include "variants.def"
#undef X
};
static const TileDesc* const kTiles = kTileDescs;

// Reduction splits offered for every tile variant.
static const int kSplits[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32};
constexpr int kNumSplits = (int)(sizeof(kSplits) / sizeof(kSplits[0]));

// variant id 0 = direct kernel; 1 + tile*kNumSplits + split_index for the MFMA tiles; the
// vector-FMA first-layer kernels follow them.
constexpr int kNumTileVariants = 1 + kNumTiles * kNumSplits;
static int num_variants() { return kNumTileVariants + fma_num_variants() + hconv_num_variants(); }

// Index into the FMA catalogue, or -1.
static int fma_index(int id) {
  return (id >= kNumTileVariants && id < kNumTileVariants + fma_num_variants()) ? id - kNumTileVariants : -1;
}

// Index into the catalogue of the fp16-matrix-core kernels (half-precision storage only), or -1.
static int hconv_index(int id) {
  const int first = kNumTileVariants + fma_num_variants();
  return (id >= first && id < num_variants()) ? id - first : -1;
}

// What the half-precision entry points run when asked to choose: an fp16-matrix-core tile
// where one applies and the launch is large enough to fill the chip with it, else the
// choice of the fp32 entry points (the same tiles, widening on the way into LDS).
static int select_variant(const Shape& s, bool filt_aligned16, bool in_aligned16);
static int f16_table_lookup(const Shape& s);
static int select_variant_f16(const Shape& s, bool filt_aligned, bool in_aligned) {
  const int listed = f16_table_lookup(s);
  if (listed > 0) return listed;
  const int h = hconv_select(s);
  if (h >= 0) return kNumTileVariants + fma_num_variants() + h;
  return select_variant(s, filt_aligned, in_aligned);
}

static bool decode_variant(int id, int* tile, int* nsplit) {
  if (id < 1 || id >= kNumTileVariants) return false;
  *tile = (id - 1) / kNumSplits;
  *nsplit = kSplits[(id - 1) % kNumSplits];
  return true;
}

// ------------------------------------------------------------------ validation
static int make_shape(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                      Shape* s) {
  if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 ||
      pad < 0)
    return BCONV_EINVAL;
  if ((long long)H + 2LL * pad < R || (long long)W + 2LL * pad < S) return BCONV_ESHAPE;
  long long P = ((long long)H + 2LL * pad - R) / stride + 1;
  long long Q = ((long long)W + 2LL * pad - S) / stride + 1;
  const long long lim = (1LL << 40);
  if ((long long)N * C * H * W >= lim || (long long)K * C * R * S >= lim ||
      (long long)N * K * P * Q >= lim || P > (1 << 30) || Q > (1 << 30))
    return BCONV_ESHAPE;
  *s = Shape{N, C, H, W, K, R, S, stride, pad, (int)P, (int)Q};
  return BCONV_OK;
}

// ------------------------------------------------------------------ batch runs
// One launch of a tiled kernel addresses its input through 32-bit byte offsets and its
// output through 31-bit element offsets.  The images of a batch are independent
// (Section II), so a larger batch is computed as consecutive launches over runs of whole
// images, every run but the last of the size returned here (near-equal runs); s.N when
// one launch takes the whole batch.  When not even one image fits, the whole batch is
// one run again: no tile applies to it and the direct kernel (64-bit indexing) takes it.
static int images_per_launch(const Shape& s) {
  const long long i31 = (1LL << 31) - 1;
  const long long in_img = (long long)s.C * s.H * s.W, out_img = (long long)s.K * s.P * s.Q;
  long long n = (i31 / 4 - ((long long)s.pad * s.W + s.pad)) / in_img;
  if (i31 / out_img < n) n = i31 / out_img;
  if (n >= s.N || n < 1) return s.N;
  const long long launches = (s.N + n - 1) / n;
  return (int)((s.N + launches - 1) / launches);
}

static Shape batch_of(const Shape& s, int n) {
  Shape c = s;
  c.N = n;
  return c;
}

// The (at most two) distinct run shapes of a batch: every full run, and the shorter last one.
static int run_shapes(const Shape& s, Shape out[2]) {
  const int per = images_per_launch(s);
  out[0] = batch_of(s, per);
  if (s.N % per == 0) return 1;
  out[1] = batch_of(s, s.N % per);
  return 2;
}

template <typename P>
static P* byte_offset(P* ptr, size_t bytes) {
  typedef std::conditional_t<std::is_const<P>::value, const char, char> byte_t;
  return reinterpret_cast<P*>(reinterpret_cast<byte_t*>(ptr) + bytes);
}

// ------------------------------------------------------------------ selection
struct TableRow {
  int N, C, H, W, K, R, S, stride, pad;
  const char* tile;
  int nsplit;
};
static const TableRow kTable[] = {
#include "selection_table.inc"
    {0, 0, 0, 0, 0, 0, 0, 0, 0, nullptr, 0}};
// Choices for convolution + 3x3 / step-2 max pooling in one call, where the best one differs
// from the convolution's own (a split variant carries the pooling in its reduction kernel).
static const TableRow kPoolTable[] = {
#include "pool_selection_table.inc"
    {0, 0, 0, 0, 0, 0, 0, 0, 0, nullptr, 0}};

// Measured choices of the half-precision entry points (fp16-matrix-core tiles), where they beat
// what those entry points would otherwise run.
static const TableRow kF16Table[] = {
#include "f16_selection_table.inc"
    {0, 0, 0, 0, 0, 0, 0, 0, 0, nullptr, 0}};

// Measured choices among those tiles for octet-interleaved (C8) activations.
static const TableRow kF16C8Table[] = {
#include "f16_c8_selection_table.inc"
    {0, 0, 0, 0, 0, 0, 0, 0, 0, nullptr, 0}};

static int find_variant(const char* tile, int nsplit) {
  for (int f = 0; f < fma_num_variants(); ++f)
    if (nsplit == 1 && std::strcmp(fma_variant_name(f), tile) == 0) return kNumTileVariants + f;
  for (int h = 0; h < hconv_num_variants(); ++h)
    if (nsplit == hconv_variant_split(h) && std::strcmp(hconv_variant_name(h), tile) == 0)
      return kNumTileVariants + fma_num_variants() + h;
  for (int t = 0; t < kNumTiles; ++t)
    if (std::strcmp(kTiles[t].name, tile) == 0)
      for (int i = 0; i < kNumSplits; ++i)
        if (kSplits[i] == nsplit) return 1 + t * kNumSplits + i;
  return -1;
}

// Time model (in clock cycles) used for shapes the table does not list.  The busiest
// compute unit runs ceil(tiles / 256) workgroups, `resident` of them at a time, in
// rounds.  The workgroups of a round advance chunk by chunk together: a chunk takes
// the longer of its barrier-to-barrier latency and the MFMAs of the waves that share
// one matrix pipe (64 cycles each; a lone wave cannot overlap its own operand reads),
// plus the issue slots of its staging instructions.  The epilogue costs per
// accumulator tile, and per tile and extra wave group when the reduction is split
// inside the workgroup.  A reduction split over the grid pays a second launch and the
// round trip of the partial sums.  The constants were fitted to the tuning sweeps of
// the benchmark layers, the square matrix products and a set of shapes kept out of
// the table (two-fold cross-validated between the listed and the unlisted shapes).
static double model_cost(const TileDesc& v, const Plan& pl) {
  const TconvParams& p = pl.p;
  const int nw = v.WM * v.WN * v.KS;
  const int S = p.S;
  const double steps = (double)(v.KR / v.KSL() / v.KS) * S;           // MFMA steps per chunk and wave
  const double tile_frac = v.MS * v.MS / 1024.0;                      // a 16x16 tile is a quarter of a 32x32 one
  const double chunk_mfma = steps * v.MT * v.NT * (v.MS == 32 ? 64.0 : 32.0);
  const double tiles = (double)pl.gx * pl.gy * pl.gz;
  // residency: LDS, wave slots, registers (accumulators + PD staging sets + addressing)
  const int agrp = v.KR * (v.S ? v.S : kSmaxGeneric) / v.AV;
  const int na = (v.BM() * agrp + v.NTHR() - 1) / v.NTHR();
  const int npl = p.halo ? v.KR / p.R : v.KR;
  const int nb = v.BV == kModeHaloFlat ? npl / v.EPT : npl * v.EPT;   // input load items per thread
  const int regs = v.MT * v.NT * (v.MS * v.MS / 64) + v.PD * (na * v.AV + nb) + 72;
  int resident = (int)(kLdsLimitBytes / pl.lds_bytes);
  const int by_regs = (512 / regs) * 4 / nw, by_waves = 32 / nw;
  if (by_regs < resident) resident = by_regs;
  if (by_waves < resident) resident = by_waves;
  if (resident < 1) resident = 1;
  const double per_cu = std::ceil(tiles / 256.0);                     // workgroups of the busiest unit
  const double conc = std::min((double)resident, per_cu);             // of them, running together
  const double rounds = std::ceil(per_cu / resident);
  const double pipe_waves = std::ceil(conc * nw / 4.0);               // waves sharing a matrix pipe
  const double eff = pipe_waves >= 2.0 ? 1.0 : 0.78;
  // staging instructions per thread and chunk: filter loads of AV words, input cells
  const double in_words = p.halo ? (double)npl * p.plane : (double)v.KR * p.plane;
  // (input loads that keep per-load address selects -- slot staging of a padded layer --
  // count one and a half times)
  const bool scalar_in = p.halo || v.BV == kModeSlotsNoPad || (v.R == 1 && v.S == 1 && v.STR == 1);
  // (flat halo staging: a thread's load count does not depend on how full the planes are)
  const double in_instr = v.BV == kModeHaloFlat ? (double)nb
                                                : in_words / v.NTHR() / (v.BV == kModeCompact4 ? 4.0 : 1.0);
  const double stage_instr = (double)v.BM() * v.KR * S / v.NTHR() / v.AV + in_instr * (scalar_in ? 1.0 : 1.5);
  const double chunk_time = std::max(300.0, pipe_waves * chunk_mfma / eff) + 80.0 * stage_instr * pipe_waves;
  const double wg_time = p.chunks_per_split * chunk_time + 1200.0 * v.MT * v.NT * tile_frac +
                         1170.0 * (v.KS - 1) * v.MT * v.NT * tile_frac;
  double t = 6000.0 + rounds * wg_time;
  if (p.nsplit > 1) t += 3900.0 + 730.0 * p.nsplit + (double)(2 * p.nsplit + 2) * p.out_elems * 4.0 / 2000.0;
  return t;
}

static double variant_cost(const TileDesc& v, const Plan& pl) {
  double c = model_cost(v, pl);
  if (!v.S) c *= 3.0;                                   // a tile compiled for this kernel size beats the generic one
  return c;
}

static int select_variant_uncached(const Shape& s, bool filt_aligned16, bool in_aligned16);

// The choice depends only on the shape and the two alignment flags; the heuristic
// plans every tile and split for a shape the table does not list (about a
// millisecond for a halo family), so the answers are remembered.
struct SelectKey {
  int v[11];
  bool operator==(const SelectKey& o) const { return std::memcmp(v, o.v, sizeof(v)) == 0; }
};
struct SelectKeyHash {
  size_t operator()(const SelectKey& k) const {
    uint64_t h = 1469598103934665603ull;
    for (int i = 0; i < 11; ++i) h = (h ^ (uint32_t)k.v[i]) * 1099511628211ull;
    return (size_t)h;
  }
};
static std::unordered_map<SelectKey, int, SelectKeyHash> g_select_cache;
static std::mutex g_select_mutex;

static int select_variant(const Shape& s, bool filt_aligned16 = true, bool in_aligned16 = true) {
  const SelectKey key = {{s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, filt_aligned16 ? 1 : 0,
                          in_aligned16 ? 1 : 0}};
  {
    std::lock_guard<std::mutex> lock(g_select_mutex);
    auto it = g_select_cache.find(key);
    if (it != g_select_cache.end()) return it->second;
  }
  const int id = select_variant_uncached(s, filt_aligned16, in_aligned16);
  std::lock_guard<std::mutex> lock(g_select_mutex);
  if (g_select_cache.size() > 4096) g_select_cache.clear();
  g_select_cache[key] = id;
  return id;
}

// The table's variant for this exact shape if the pointers allow its loads, else -1.
static int table_lookup(const TableRow* table, const Shape& s, bool filt_aligned16, bool in_aligned16) {
  for (const TableRow* r = table; r->tile; ++r) {
    if (r->N == s.N && r->C == s.C && r->H == s.H && r->W == s.W && r->K == s.K && r->R == s.R &&
        r->S == s.S && r->stride == s.stride && r->pad == s.pad) {
      int id = find_variant(r->tile, r->nsplit);
      int t, ns;
      Plan pl;
      if (fma_index(id) >= 0 && fma_conv_applicable(fma_index(id), s)) return id;
      if (id > 0 && decode_variant(id, &t, &ns) && (filt_aligned16 || kTiles[t].AV == 1) &&
          (in_aligned16 || kTiles[t].BV != kModeCompact4) &&
          plan_tconv(s, kTiles[t], ns, &pl))
        return id;
    }
  }
  return -1;
}

// A half-precision table's fp16-matrix-core tile for this exact shape, or -1.
static int f16_rows_lookup(const TableRow* rows, const Shape& s);
static int f16_table_lookup(const Shape& s) { return f16_rows_lookup(kF16Table, s); }
static int f16_rows_lookup(const TableRow* rows, const Shape& s) {
  for (const TableRow* r = rows; r->tile; ++r) {
    if (r->N == s.N && r->C == s.C && r->H == s.H && r->W == s.W && r->K == s.K && r->R == s.R &&
        r->S == s.S && r->stride == s.stride && r->pad == s.pad) {
      const int id = find_variant(r->tile, r->nsplit);
      if (hconv_index(id) >= 0 && hconv_applicable(hconv_index(id), s)) return id;
    }
  }
  return -1;
}

// Convolution + pooling in one call: the pooled table covers windows of 3 with step 2
// (the pooling of the benchmark stack); everything else takes the convolution's choice.
static int select_pool_variant(const Shape& s, int ksz, int pstride, bool filt_aligned16,
                               bool in_aligned16) {
  if (ksz == 3 && pstride == 2) {
    const int id = table_lookup(kPoolTable, s, filt_aligned16, in_aligned16);
    if (id > 0) return id;
  }
  return select_variant(s, filt_aligned16, in_aligned16);
}

static int select_variant_uncached(const Shape& s, bool filt_aligned16, bool in_aligned16) {
  const int listed = table_lookup(kTable, s, filt_aligned16, in_aligned16);
  if (listed > 0) return listed;
  int best = 0;
  double best_cost = 0.0;
  for (int t = 0; t < kNumTiles; ++t) {
    if (!filt_aligned16 && kTiles[t].AV != 1) continue;
    if (!in_aligned16 && kTiles[t].BV == kModeCompact4) continue;
    for (int i = 0; i < kNumSplits; ++i) {
      Plan pl;
      if (!plan_tconv(s, kTiles[t], kSplits[i], &pl)) continue;
      double c = variant_cost(kTiles[t], pl);
      if (best == 0 || c < best_cost) {
        best = 1 + t * kNumSplits + i;
        best_cost = c;
      }
    }
  }
  return best;   // 0 = direct kernel when no tile applies
}

// ------------------------------------------------------------------ workspace
struct DeviceWorkspace {
  void* ptr = nullptr;
  size_t bytes = 0;
};
static DeviceWorkspace g_ws[64];
static std::mutex g_ws_mutex;
static std::mutex g_own_ws_call_mutex;   // held by a call from workspace lookup to its last launch

static int internal_workspace(size_t need, void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return BCONV_ELAUNCH;
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  DeviceWorkspace& w = g_ws[dev];
  if (w.bytes < need) {
    if (w.ptr) {
      if (hipDeviceSynchronize() != hipSuccess) return BCONV_ELAUNCH;
      (void)hipFree(w.ptr);
      w.ptr = nullptr;
      w.bytes = 0;
    }
    size_t want = need < (size_t)(32u << 20) ? (size_t)(32u << 20) : need;
    if (hipMalloc(&w.ptr, want) != hipSuccess) {
      w.ptr = nullptr;
      (void)hipGetLastError();
      return BCONV_ELAUNCH;
    }
    w.bytes = want;
  }
  *out = w.ptr;
  return BCONV_OK;
}

// ------------------------------------------------------------------ static scratch
// Device memory for the partial sums of conv_fwd_noalloc: part of the library's code object,
// so every GPU that loads the library holds its own copy until the process ends and no call
// ever allocates.  In host code the array's name is only a handle for the runtime's symbol
// lookup, never an address: the per-device address comes from hipGetSymbolAddress, once per
// device with that device current, and that pointer is what kernels are given.
constexpr size_t kStaticScratchBytes = BCONV_NOALLOC_MAX_WORKSPACE_BYTES;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];
static void* g_scratch_ptr[64];
static std::mutex g_scratch_mutex;

static int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return BCONV_ELAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return BCONV_ELAUNCH;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return BCONV_OK;
}

// ------------------------------------------------------------------ run
// f16: in, filt and out hold _Float16 elements (passed through float pointers); the
// tiles' 4-element loads then need 8-byte instead of 16-byte alignment.
// One launch (plus its reduction kernel) over a batch that a single launch can address.
// dry: resolve the variant and check everything a launch would, store the workspace need
// in *need_out, and return before allocating or launching anything.
static int run_conv_launch(const float* in, const float* filt, const float* bias, float* out,
                           const Shape& s, int relu, void* ws, size_t ws_bytes, bool own_ws,
                           hipStream_t st, int variant_id, bool f16, bool dry, size_t* need_out) {
  const uintptr_t vec_mask = f16 ? 7u : 15u;
  const bool aligned16 = (reinterpret_cast<uintptr_t>(filt) & vec_mask) == 0;
  const bool in_aligned16 = (reinterpret_cast<uintptr_t>(in) & vec_mask) == 0;
  if (variant_id < 0)
    variant_id = f16 ? select_variant_f16(s, aligned16, in_aligned16) : select_variant(s, aligned16, in_aligned16);
  if (need_out) *need_out = 0;
  if (hconv_index(variant_id) >= 0) {
    const int h = hconv_index(variant_id);
    if (!f16 || !hconv_applicable(h, s)) return BCONV_EVARIANT;
    const size_t need = hconv_workspace_bytes(h, s);
    if (need_out) *need_out = need;
    if (own_ws) {
      if (!dry) {
        int rc = internal_workspace(need, &ws);
        if (rc != BCONV_OK) return rc;
      }
    } else if (!ws || ws_bytes < need) {
      return BCONV_EWORKSPACE;
    }
    if (dry) return BCONV_OK;
    return launch_hconv(h, in, filt, bias, out, s, relu, 0, 0, ws, st) == hipSuccess ? BCONV_OK : BCONV_ELAUNCH;
  }
  if (variant_id == 0) {
    if (dry) return BCONV_OK;
    return launch_direct_conv(in, filt, bias, out, s, relu, f16, st) == hipSuccess ? BCONV_OK
                                                                                   : BCONV_ELAUNCH;
  }
  if (fma_index(variant_id) >= 0) {
    if (f16 || !fma_conv_applicable(fma_index(variant_id), s)) return BCONV_EVARIANT;
    if (dry) return BCONV_OK;
    return launch_fma_conv(fma_index(variant_id), in, filt, bias, out, s, relu, st) == hipSuccess
               ? BCONV_OK
               : BCONV_ELAUNCH;
  }
  int t, nsplit;
  if (!decode_variant(variant_id, &t, &nsplit)) return BCONV_EVARIANT;
  Plan pl;
  if (!plan_tconv(s, kTiles[t], nsplit, &pl)) return BCONV_EVARIANT;
  if (kTiles[t].AV == 4 && !aligned16) return BCONV_EVARIANT;
  if (kTiles[t].BV == kModeCompact4 && !in_aligned16) return BCONV_EVARIANT;
  if (need_out) *need_out = pl.ws_bytes;
  if (pl.ws_bytes) {
    if (own_ws) {
      if (!dry) {
        int rc = internal_workspace(pl.ws_bytes, &ws);
        if (rc != BCONV_OK) return rc;
      }
    } else if (!ws || ws_bytes < pl.ws_bytes) {
      return BCONV_EWORKSPACE;
    }
  }
  if (dry) return BCONV_OK;
  pl.p.in = in;
  pl.p.filt = filt;
  pl.p.bias = bias;
  pl.p.out = out;
  pl.p.partial = pl.ws_bytes ? static_cast<float*>(ws) : nullptr;
  pl.p.relu = relu;
  if ((f16 ? kLaunchF16 : kLaunch)[t](pl.p, dim3(pl.gx, pl.gy, pl.gz), pl.lds_bytes, st) != hipSuccess)
    return BCONV_ELAUNCH;
  if (nsplit > 1) {
    if (launch_splitk_reduce(pl.p.partial, bias, out, nsplit, pl.p.out_elems, s.K, s.P * s.Q, relu,
                             f16, false, st) != hipSuccess)
      return BCONV_ELAUNCH;
  }
  return BCONV_OK;
}

// The whole batch: one launch, or consecutive launches over runs of images when the
// tensors are beyond what one launch addresses.  All runs are checked before the first
// is launched, so that an error leaves nothing enqueued.
static int run_conv(const float* in, const float* filt, const float* bias, float* out,
                    const Shape& s, int relu, void* ws, size_t ws_bytes, bool own_ws,
                    hipStream_t st, int variant_id, bool f16 = false) {
  // The library's own workspace may be regrown (synchronise, free, allocate) by another host
  // thread: growing and enqueueing the kernels that use it are one critical section.
  std::unique_lock<std::mutex> own_ws_lock(g_own_ws_call_mutex, std::defer_lock);
  if (own_ws) own_ws_lock.lock();
  const int per = images_per_launch(s);
  if (per >= s.N)
    return run_conv_launch(in, filt, bias, out, s, relu, ws, ws_bytes, own_ws, st, variant_id, f16,
                           false, nullptr);
  const size_t esz = f16 ? 2 : 4;
  const size_t in_img = (size_t)s.C * s.H * s.W * esz, out_img = (size_t)s.K * s.P * s.Q * esz;
  size_t need = 0;
  for (int pass = 0; pass < 2; ++pass) {
    for (int n0 = 0; n0 < s.N; n0 += per) {
      const Shape run = batch_of(s, s.N - n0 < per ? s.N - n0 : per);
      size_t n = 0;
      int rc = run_conv_launch(byte_offset(in, n0 * in_img), filt, bias, byte_offset(out, n0 * out_img),
                               run, relu, ws, ws_bytes, own_ws, st, variant_id, f16, pass == 0, &n);
      if (rc != BCONV_OK) return rc;
      if (n > need) need = n;
    }
    if (pass == 0 && own_ws && need) {        // one allocation that serves every run
      int rc = internal_workspace(need, &ws);
      if (rc != BCONV_OK) return rc;
      ws_bytes = need;
      own_ws = false;
    }
  }
  return BCONV_OK;
}

// Convolution + bias + ReLU followed by max pooling (window ksz, step pstride, no padding)
// in one call, fp32.  Workspace need of a variant: the partial sums when it splits the
// reduction (the pooling is then folded into the reduction kernel), else the unpooled
// convolution output (pooled by a second kernel).
static size_t conv_pool_need(const Shape& s, int variant_id) {
  const size_t conv_bytes = (size_t)s.N * s.K * s.P * s.Q * sizeof(float);
  int t, nsplit;
  Plan pl;
  if (variant_id == 0) return conv_bytes;
  if (fma_index(variant_id) >= 0) return fma_conv_applicable(fma_index(variant_id), s) ? conv_bytes : 0;
  if (!decode_variant(variant_id, &t, &nsplit) || !plan_tconv(s, kTiles[t], nsplit, &pl)) return 0;
  return nsplit > 1 ? pl.ws_bytes : conv_bytes;
}

static int run_conv_pool_launch(const float* in, const float* filt, const float* bias, float* out,
                                const Shape& s, int relu, int ksz, int pstride, void* ws,
                                size_t ws_bytes, hipStream_t st, int variant_id, bool dry) {
  const bool aligned16 = (reinterpret_cast<uintptr_t>(filt) & 15u) == 0;
  const bool in_aligned16 = (reinterpret_cast<uintptr_t>(in) & 15u) == 0;
  if (variant_id < 0) variant_id = select_pool_variant(s, ksz, pstride, aligned16, in_aligned16);
  const size_t need = conv_pool_need(s, variant_id);
  if (need == 0) return BCONV_EVARIANT;
  if (!ws || ws_bytes < need) return BCONV_EWORKSPACE;
  int t = 0, nsplit = 1;
  if (variant_id > 0 && fma_index(variant_id) < 0 && !decode_variant(variant_id, &t, &nsplit))
    return BCONV_EVARIANT;
  float* const scratch = static_cast<float*>(ws);
  if (variant_id == 0 || nsplit == 1) {
    // unpooled output into the workspace (a variant without split needs none of its own)
    int rc = run_conv_launch(in, filt, bias, scratch, s, relu, nullptr, 0, false, st, variant_id, false,
                             dry, nullptr);
    if (rc != BCONV_OK || dry) return rc;
    return launch_maxpool(scratch, out, s.N, s.K, s.P, s.Q, ksz, pstride, (s.P - ksz) / pstride + 1,
                          (s.Q - ksz) / pstride + 1, st) == hipSuccess
               ? BCONV_OK
               : BCONV_ELAUNCH;
  }
  Plan pl;
  if (!plan_tconv(s, kTiles[t], nsplit, &pl)) return BCONV_EVARIANT;
  if (kTiles[t].AV == 4 && !aligned16) return BCONV_EVARIANT;
  if (kTiles[t].BV == kModeCompact4 && !in_aligned16) return BCONV_EVARIANT;
  if (dry) return BCONV_OK;
  pl.p.in = in;
  pl.p.filt = filt;
  pl.p.bias = bias;
  pl.p.out = nullptr;          // a split launch writes partial sums only
  pl.p.partial = scratch;
  pl.p.relu = relu;
  if (kLaunch[t](pl.p, dim3(pl.gx, pl.gy, pl.gz), pl.lds_bytes, st) != hipSuccess) return BCONV_ELAUNCH;
  return launch_splitk_reduce_pool(scratch, bias, out, nsplit, pl.p.out_elems, s.N, s.K, s.P, s.Q, ksz,
                                   pstride, relu, st) == hipSuccess
             ? BCONV_OK
             : BCONV_ELAUNCH;
}

static int run_conv_pool(const float* in, const float* filt, const float* bias, float* out,
                         const Shape& s, int relu, int ksz, int pstride, void* ws, size_t ws_bytes,
                         hipStream_t st, int variant_id) {
  const int per = images_per_launch(s);
  if (per >= s.N)
    return run_conv_pool_launch(in, filt, bias, out, s, relu, ksz, pstride, ws, ws_bytes, st, variant_id,
                                false);
  const size_t in_img = (size_t)s.C * s.H * s.W * sizeof(float);
  const size_t out_img = (size_t)s.K * ((s.P - ksz) / pstride + 1) * ((s.Q - ksz) / pstride + 1) * sizeof(float);
  for (int pass = 0; pass < 2; ++pass)
    for (int n0 = 0; n0 < s.N; n0 += per) {
      const Shape run = batch_of(s, s.N - n0 < per ? s.N - n0 : per);
      int rc = run_conv_pool_launch(byte_offset(in, n0 * in_img), filt, bias, byte_offset(out, n0 * out_img),
                                    run, relu, ksz, pstride, ws, ws_bytes, st, variant_id, pass == 0);
      if (rc != BCONV_OK) return rc;
    }
  return BCONV_OK;
}

// ------------------------------------------------------------------ audit
static long long audit(const Shape& s, const TileDesc& v, const Plan& pl) {
  const TconvParams& p = pl.p;
  long long bad = 0;
  const int BN = v.BN(), BM = v.BM(), NTHR = v.NTHR();
  const long long in_elems = (long long)p.N * p.CHW;
  const int ncell = p.nrows * p.rowst;
  const int planes = p.halo ? v.KR / p.R : v.KR;
  if (p.ast < v.KR * p.S) ++bad;
  if ((size_t)(2 * BM * p.ast + 2 * (planes * p.plane + kLdsTrashWords) + kLdsTrashWords) * 4 >
      pl.lds_bytes)
    ++bad;
  if (v.KS > 1 && (size_t)BM * BN * 4 > pl.lds_bytes) ++bad;
  if ((long long)ncell > v.cell_capacity(p.bv)) ++bad;
  for (unsigned bx = 0; bx < pl.gx; ++bx) {
    PixTile t = pix_tile((int)bx, BN, p.NPQ, p.Q, p.fdQ);
    if (t.cnt < 1 || t.cnt > BN) ++bad;
    if (p.halo) {
      HaloTile ht = halo_tile(p, t);
      if (ht.vr < 1 || ht.vr > p.vr) ++bad;
      for (int e = 0; e < ncell; ++e) {
        BCell c = h_cell(p, ht, e, p.stride);
        if (c.lds < 0 || c.lds >= p.plane) ++bad;
        if (c.ih0 == kNeverValid) continue;
        long long lo = c.goff, hi = (long long)c.goff + (long long)(p.C - 1) * p.HW;
        if (lo < 0 || hi >= in_elems) ++bad;
      }
      for (int col = 0; col < BN; ++col) {
        BLane l = h_lane(p, t, ht, col);
        for (int r = 0; r < p.R; ++r)
          for (int ss = 0; ss < p.S; ++ss) {
            int a = l.ldsbase + r * p.rowst + tap_off(ss, p.stride, p.phst);
            if (a < 0 || a >= p.plane) ++bad;
          }
        if (l.valid) {
          long long lo = l.outoff, hi = (long long)l.outoff + (long long)(p.K - 1) * p.PQ;
          if (lo < 0 || hi >= p.out_elems) ++bad;
        }
      }
      continue;
    }
    if (!p.compact && t.rho1 - t.rho0 + 1 > p.nrows) ++bad;
    // staged cells: each LDS word of a plane is written by exactly one cell
    for (int e = 0; e < v.EPT * NTHR; ++e) {
      if (e * p.bv >= ncell) continue;
      BCell c = b_cell(p, t, e, p.S, p.stride);
      if (c.lds < 0 || c.lds >= p.plane) ++bad;
      if (c.ih0 == kNeverValid) continue;
      for (int ci = 0; ci < 2; ++ci) {
        int cc = ci ? p.C - 1 : 0;
        for (int r = 0; r < p.R; ++r) {
          if ((unsigned)(c.ih0 + r) >= (unsigned)p.H) continue;
          long long off = (long long)c.goff + (long long)cc * p.HW + (long long)r * p.W;
          if (off < 0 || off >= in_elems) ++bad;
        }
      }
    }
    // lanes: every tap read stays inside the plane; stores inside out
    for (int col = 0; col < BN; ++col) {
      BLane l = b_lane(p, t, col);
      for (int ss = 0; ss < p.S; ++ss) {
        int a = l.ldsbase + tap_off(ss, p.stride, p.phst);
        if (a < 0 || a >= p.plane) ++bad;
      }
      if (l.valid) {
        long long lo = l.outoff, hi = (long long)l.outoff + (long long)(p.K - 1) * p.PQ;
        if (lo < 0 || hi >= p.out_elems) ++bad;
      }
    }
  }
  // Input reads of the last chunk under flat staging: a thread's own plane offset can carry it up
  // to one chunk of planes past the last channel -- into the next image, or past the tensor for
  // the last image, where the range check returns zero; the kernel zeroes those cells in LDS by
  // the same predicate that would have masked the load.  What the host has to guarantee is that
  // the byte offset of such a read cannot wrap around 2^32 back into the tensor.
  if (((long long)in_elems + p.gbias + (long long)planes * p.HW + 4) * 4 > (1LL << 32)) ++bad;
  // Filter reads.  A staged item is AV consecutive words of one filter row, at the chunk's
  // column offset col0 = chunk * KR * S plus the item's column j.  Only the last chunk can
  // reach past the end of its row (every earlier one ends at or before (nchunks-1)*KR*S <
  // C*R*S); there a word past the row's end comes from the next filter row, or, in the last
  // row, from beyond the tensor, where the kernel relies on the buffer range check (which
  // covers per-lane plus scalar offset) to return zero.  Either way the kernel zeroes the
  // item in LDS afterwards, which it decides per item from col0 + j >= C*R*S: so every word
  // past the row's end must belong to an item that starts past it, and the byte offset of a
  // read beyond the tensor must not wrap around 2^32 back into it.
  {
    const int SP = v.S ? v.S : kSmaxGeneric;
    const int agrp = v.KR * SP / v.AV;
    const int krs = v.KR * p.S;
    const long long col0 = (long long)(p.nchunks - 1) * v.KR * p.S;
    const long long filt_words = (long long)p.K * p.CRS;
    for (unsigned by = 0; by < pl.gy; ++by) {
      for (int m = 0; m < BM && (long long)by * BM + m < p.K; ++m) {
        const long long row = ((long long)by * BM + m) * p.CRS;
        for (int g = 0; g < agrp; ++g) {
          const int j = g * v.AV;
          if (!v.S && j >= krs) continue;
          for (int u = 0; u < v.AV; ++u) {
            const long long w = col0 + j + u;
            if (w < p.CRS) continue;
            if (col0 + j < p.CRS) ++bad;                                   // straddles the row's end: not zeroed
            if (row + w >= filt_words && (row + w + 1) * 4 > (1LL << 32)) ++bad;    // would wrap into the tensor
          }
        }
      }
    }
  }
  for (unsigned by = 0; by < pl.gy; ++by) {
    int m0 = (int)by * BM;
    if (m0 >= p.K) ++bad;
  }
  if ((long long)p.nchunks * v.KR < p.CRrows) ++bad;
  if ((long long)p.chunks_per_split * p.nsplit < p.nchunks) ++bad;
  (void)s;
  return bad;
}

static const char* status_text(int st) {
  switch (st) {
    case BCONV_OK: return "ok";
    case BCONV_EINVAL: return "invalid argument (dimension, stride, pad or relu flag)";
    case BCONV_ENULL: return "required pointer is NULL";
    case BCONV_ESHAPE: return "shape has no output point or a tensor is too large";
    case BCONV_EWORKSPACE: return "workspace missing or too small";
    case BCONV_ELAUNCH: return "HIP runtime refused an allocation or a kernel launch";
    case BCONV_EVARIANT: return "variant id out of range or not applicable to this shape";
    default: return "unknown status";
  }
}

}  // namespace bconv

using namespace bconv;

extern "C" {

int conv_out_dims(int H, int W, int R, int S, int stride, int pad, int* P, int* Q) {
  if (!P || !Q) return BCONV_ENULL;
  Shape s;
  int rc = make_shape(1, 1, H, W, 1, R, S, stride, pad, &s);
  if (rc != BCONV_OK) return rc;
  *P = s.P;
  *Q = s.Q;
  return BCONV_OK;
}

// Argument checks shared by the four convolution entry points (elem_bytes: 4 for
// fp32 tensors, 2 for half precision, whose pointers must be 2-byte aligned).
static int check_conv_args(const void* in, const void* filt, const void* out, int N, int C, int H,
                           int W, int K, int R, int S, int stride, int pad, int relu,
                           int elem_bytes, Shape* s) {
  int rc = make_shape(N, C, H, W, K, R, S, stride, pad, s);
  if (rc != BCONV_OK) return rc;
  if (relu != 0 && relu != 1) return BCONV_EINVAL;
  if (!in || !filt || !out) return BCONV_ENULL;
  if (elem_bytes == 2 &&
      ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(filt) |
        reinterpret_cast<uintptr_t>(out)) & 1u) != 0)
    return BCONV_EINVAL;
  return BCONV_OK;
}

int conv_fwd_ex(const float* in, const float* filt, const float* bias, float* out, int N, int C,
                int H, int W, int K, int R, int S, int stride, int pad, int relu, void* workspace,
                size_t workspace_bytes, void* hip_stream, int variant_id) {
  Shape s;
  int rc = check_conv_args(in, filt, out, N, C, H, W, K, R, S, stride, pad, relu, 4, &s);
  if (rc != BCONV_OK) return rc;
  if (variant_id < -1 || variant_id >= num_variants()) return BCONV_EVARIANT;
  return run_conv(in, filt, bias, out, s, relu, workspace, workspace_bytes, false,
                  static_cast<hipStream_t>(hip_stream), variant_id);
}

int conv_fwd(const float* in, const float* filt, const float* bias, float* out, int N, int C,
             int H, int W, int K, int R, int S, int stride, int pad, int relu) {
  Shape s;
  int rc = check_conv_args(in, filt, out, N, C, H, W, K, R, S, stride, pad, relu, 4, &s);
  if (rc != BCONV_OK) return rc;
  return run_conv(in, filt, bias, out, s, relu, nullptr, 0, true, nullptr, -1);
}

// conv_fwd_ex with the partial sums in the library's static device array; see include/bconv.h.
int conv_fwd_noalloc(const float* in, const float* filt, const float* bias, float* out, int N, int C,
                     int H, int W, int K, int R, int S, int stride, int pad, int relu,
                     void* hip_stream) {
  Shape s;
  int rc = check_conv_args(in, filt, out, N, C, H, W, K, R, S, stride, pad, relu, 4, &s);
  if (rc != BCONV_OK) return rc;
  // the need is known before anything is looked up on the device: beyond the array -> refused
  if (conv_fwd_workspace_bytes(N, C, H, W, K, R, S, stride, pad, -1) > kStaticScratchBytes)
    return BCONV_EWORKSPACE;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != BCONV_OK) return rc;
  return run_conv(in, filt, bias, out, s, relu, ws, kStaticScratchBytes, false,
                  static_cast<hipStream_t>(hip_stream), -1);
}

// Half-precision storage: the same layer with in, filt and out as IEEE binary16.
int conv_fwd_f16_ex(const void* in, const void* filt, const float* bias, void* out, int N, int C,
                    int H, int W, int K, int R, int S, int stride, int pad, int relu,
                    void* workspace, size_t workspace_bytes, void* hip_stream, int variant_id) {
  Shape s;
  int rc = check_conv_args(in, filt, out, N, C, H, W, K, R, S, stride, pad, relu, 2, &s);
  if (rc != BCONV_OK) return rc;
  if (variant_id < -1 || variant_id >= num_variants()) return BCONV_EVARIANT;
  return run_conv(static_cast<const float*>(in), static_cast<const float*>(filt), bias,
                  static_cast<float*>(out), s, relu, workspace, workspace_bytes, false,
                  static_cast<hipStream_t>(hip_stream), variant_id, true);
}

int conv_fwd_f16(const void* in, const void* filt, const float* bias, void* out, int N, int C,
                 int H, int W, int K, int R, int S, int stride, int pad, int relu) {
  Shape s;
  int rc = check_conv_args(in, filt, out, N, C, H, W, K, R, S, stride, pad, relu, 2, &s);
  if (rc != BCONV_OK) return rc;
  return run_conv(static_cast<const float*>(in), static_cast<const float*>(filt), bias,
                  static_cast<float*>(out), s, relu, nullptr, 0, true, nullptr, -1, true);
}

// Convolution + bias + ReLU + max pooling; see include/bconv.h.
int conv_pool_fwd_ex(const float* in, const float* filt, const float* bias, float* out, int N,
                     int C, int H, int W, int K, int R, int S, int stride, int pad, int relu,
                     int pool_ksz, int pool_stride, void* workspace, size_t workspace_bytes,
                     void* hip_stream, int variant_id) {
  Shape s;
  int rc = check_conv_args(in, filt, out, N, C, H, W, K, R, S, stride, pad, relu, 4, &s);
  if (rc != BCONV_OK) return rc;
  if (pool_ksz <= 0 || pool_stride <= 0) return BCONV_EINVAL;
  if (s.P < pool_ksz || s.Q < pool_ksz) return BCONV_ESHAPE;
  if (variant_id < -1 || variant_id >= num_variants()) return BCONV_EVARIANT;
  return run_conv_pool(in, filt, bias, out, s, relu, pool_ksz, pool_stride, workspace,
                       workspace_bytes, static_cast<hipStream_t>(hip_stream), variant_id);
}

// Workspace of one run shape (see run_shapes); 0 when a forced variant cannot run it.
static size_t conv_pool_need_any_alignment(const Shape& s, int variant_id) {
  if (variant_id >= 0) return variant_id < num_variants() ? conv_pool_need(s, variant_id) : 0;
  size_t need = 0;
  for (int mask = 0; mask < 4; ++mask) {     // whichever loads the pointers turn out to allow
    // (the pooling window is not known here: enough for the pooled table's choice too)
    const size_t n = conv_pool_need(s, select_variant(s, (mask & 1) != 0, (mask & 2) != 0));
    const size_t m = conv_pool_need(s, select_pool_variant(s, 3, 2, (mask & 1) != 0, (mask & 2) != 0));
    if (n > need) need = n;
    if (m > need) need = m;
  }
  return need;
}

size_t conv_pool_fwd_workspace_bytes(int N, int C, int H, int W, int K, int R, int S, int stride,
                                     int pad, int variant_id) {
  Shape s, runs[2];
  if (make_shape(N, C, H, W, K, R, S, stride, pad, &s) != BCONV_OK) return 0;
  size_t need = 0;
  for (int i = 0, n = run_shapes(s, runs); i < n; ++i) {
    const size_t b = conv_pool_need_any_alignment(runs[i], variant_id);
    if (b == 0) return 0;                    // (a conv + pool call always needs a workspace)
    if (b > need) need = b;
  }
  return need;
}

int conv_pool_selected_variant(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               int pool_ksz, int pool_stride) {
  Shape s;
  int rc = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
  if (rc != BCONV_OK) return rc;
  if (pool_ksz <= 0 || pool_stride <= 0) return BCONV_EINVAL;
  if (s.P < pool_ksz || s.Q < pool_ksz) return BCONV_ESHAPE;
  return select_pool_variant(batch_of(s, images_per_launch(s)), pool_ksz, pool_stride, true, true);
}

// Workspace of one run shape; *ok = false when a forced variant cannot run it.
static size_t conv_need_any_alignment(const Shape& s, int variant_id, bool* ok) {
  int t, nsplit;
  Plan pl;
  *ok = true;
  if (variant_id < 0) {
    // the choice depends on whether in / filt allow the wide loads, which this call
    // cannot know: enough for whichever of the four cases the pointers turn out to be
    size_t need = 0;
    for (int mask = 0; mask < 4; ++mask) {
      const int id = select_variant(s, (mask & 1) != 0, (mask & 2) != 0);
      if (decode_variant(id, &t, &nsplit) && plan_tconv(s, kTiles[t], nsplit, &pl) && pl.ws_bytes > need)
        need = pl.ws_bytes;
    }
    return need;
  }
  if (variant_id == 0) return 0;
  if (fma_index(variant_id) >= 0) {
    *ok = fma_conv_applicable(fma_index(variant_id), s);
    return 0;
  }
  if (!decode_variant(variant_id, &t, &nsplit) || !plan_tconv(s, kTiles[t], nsplit, &pl)) {
    *ok = false;
    return 0;
  }
  return pl.ws_bytes;
}

size_t conv_fwd_workspace_bytes(int N, int C, int H, int W, int K, int R, int S, int stride,
                                int pad, int variant_id) {
  Shape s, runs[2];
  if (make_shape(N, C, H, W, K, R, S, stride, pad, &s) != BCONV_OK) return 0;
  size_t need = 0;
  for (int i = 0, n = run_shapes(s, runs); i < n; ++i) {
    bool ok;
    const size_t b = conv_need_any_alignment(runs[i], variant_id, &ok);
    if (!ok) return 0;
    if (b > need) need = b;
  }
  return need;
}

// ---- queries of the half-precision entry points (their choice and catalogue include the
// fp16-matrix-core tiles, which the fp32 entry points cannot run)
int conv_fwd_f16_selected_variant(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
  Shape s;
  int rc = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
  if (rc != BCONV_OK) return rc;
  return select_variant_f16(batch_of(s, images_per_launch(s)), true, true);
}

int conv_fwd_f16_variant_applicable(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                    int variant_id) {
  Shape s, runs[2];
  int rc = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
  if (rc != BCONV_OK) return rc;
  if (hconv_index(variant_id) >= 0) {
    for (int i = 0, n = run_shapes(s, runs); i < n; ++i)
      if (!hconv_applicable(hconv_index(variant_id), runs[i])) return 0;
    return 1;
  }
  if (fma_index(variant_id) >= 0) return 0;
  return conv_variant_applicable(N, C, H, W, K, R, S, stride, pad, variant_id);
}

size_t conv_fwd_f16_workspace_bytes(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                    int variant_id) {
  Shape s, runs[2];
  if (make_shape(N, C, H, W, K, R, S, stride, pad, &s) != BCONV_OK) return 0;
  if (variant_id >= 0 && hconv_index(variant_id) < 0)
    return conv_fwd_workspace_bytes(N, C, H, W, K, R, S, stride, pad, variant_id);
  size_t need = variant_id < 0 ? conv_fwd_workspace_bytes(N, C, H, W, K, R, S, stride, pad, -1) : 0;
  for (int i = 0, n = run_shapes(s, runs); i < n; ++i) {
    const int h = variant_id < 0 ? hconv_index(select_variant_f16(runs[i], true, true)) : hconv_index(variant_id);
    if (h < 0) continue;
    if (!hconv_applicable(h, runs[i])) return 0;
    const size_t b = hconv_workspace_bytes(h, runs[i]);
    if (b > need) need = b;
  }
  return need;
}

// ---- filter pre-packing for the fp16-matrix-core tiles (weights are constant in deployment)
// The tile a (shape, variant_id) pair means for the packed calls, or -1.
static int packed_tile(const Shape& s, int variant_id) {
  if (images_per_launch(s) < s.N) return -1;            // one launch only
  const int id = variant_id < 0 ? select_variant_f16(s, true, true) : variant_id;
  const int h = hconv_index(id);
  return (h >= 0 && hconv_packable(h) && hconv_applicable(h, s)) ? h : -1;
}

int conv_fwd_f16_c8_selected_variant(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
  Shape s;
  int rc = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
  if (rc != BCONV_OK) return rc;
  if (images_per_launch(s) < s.N) return BCONV_EVARIANT;
  const int listed = f16_rows_lookup(kF16C8Table, s);
  if (listed > 0) return listed;
  const int h = hconv_select(s, true);
  // (the first-layer tiles read NCHW only)
  return (h < 0 || !hconv_packable(h)) ? BCONV_EVARIANT : kNumTileVariants + fma_num_variants() + h;
}

// The partial sums of a split variant under the packed calls (which take no workspace): the
// library's own per-device buffer, grown on first need like conv_fwd's.
static int packed_scratch(int h, const Shape& s, void** scratch) {
  *scratch = nullptr;
  const size_t need = hconv_partial_bytes(h, s);
  return need ? internal_workspace(need, scratch) : BCONV_OK;
}

size_t conv_f16_packed_filter_bytes(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                    int variant_id) {
  Shape s;
  if (make_shape(N, C, H, W, K, R, S, stride, pad, &s) != BCONV_OK) return 0;
  const int h = packed_tile(s, variant_id);
  return h < 0 ? 0 : hconv_packed_bytes(h, s);
}

int conv_f16_pack_filters(const void* filt, void* packed, size_t packed_bytes, int N, int C, int H, int W,
                          int K, int R, int S, int stride, int pad, void* hip_stream, int variant_id) {
  Shape s;
  int rc = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
  if (rc != BCONV_OK) return rc;
  if (!filt || !packed) return BCONV_ENULL;
  if (((reinterpret_cast<uintptr_t>(filt) & 1u) | (reinterpret_cast<uintptr_t>(packed) & 15u)) != 0) return BCONV_EINVAL;
  const int h = packed_tile(s, variant_id);
  if (h < 0) return BCONV_EVARIANT;
  if (packed_bytes < hconv_packed_bytes(h, s)) return BCONV_EWORKSPACE;
  return launch_hconv_pack(h, filt, packed, s, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? BCONV_OK
                                                                                                  : BCONV_ELAUNCH;
}

int conv_fwd_f16_packed_ex(const void* in, const void* packed, const float* bias, void* out, int N, int C,
                           int H, int W, int K, int R, int S, int stride, int pad, int relu,
                           void* hip_stream, int variant_id) {
  Shape s;
  int rc = check_conv_args(in, packed, out, N, C, H, W, K, R, S, stride, pad, relu, 2, &s);
  if (rc != BCONV_OK) return rc;
  if ((reinterpret_cast<uintptr_t>(packed) & 15u) != 0) return BCONV_EINVAL;
  const int h = packed_tile(s, variant_id);
  if (h < 0) return BCONV_EVARIANT;
  void* scratch = nullptr;
  rc = packed_scratch(h, s, &scratch);
  if (rc != BCONV_OK) return rc;
  return launch_hconv_packed(h, in, packed, bias, out, s, relu, 0, 0, scratch,
                             static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? BCONV_OK
             : BCONV_ELAUNCH;
}

int conv_fwd_f16_packed_layout_ex(const void* in, int in_layout, const void* packed, const float* bias, void* out,
                                  int out_layout, int N, int C, int H, int W, int K, int R, int S, int stride,
                                  int pad, int relu, void* hip_stream, int variant_id) {
  Shape s;
  int rc = check_conv_args(in, packed, out, N, C, H, W, K, R, S, stride, pad, relu, 2, &s);
  if (rc != BCONV_OK) return rc;
  if ((in_layout != BCONV_LAYOUT_NCHW && in_layout != BCONV_LAYOUT_C8) ||
      (out_layout != BCONV_LAYOUT_NCHW && out_layout != BCONV_LAYOUT_C8))
    return BCONV_EINVAL;
  // the octet-interleaved output is written by kernels that read the octet-interleaved input
  if (out_layout == BCONV_LAYOUT_C8 && (in_layout != BCONV_LAYOUT_C8 || K % 8 != 0)) return BCONV_EINVAL;
  if ((reinterpret_cast<uintptr_t>(packed) & 15u) != 0) return BCONV_EINVAL;
  if (in_layout == BCONV_LAYOUT_C8 && (reinterpret_cast<uintptr_t>(in) & 15u) != 0) return BCONV_EINVAL;
  if (out_layout == BCONV_LAYOUT_C8 && (reinterpret_cast<uintptr_t>(out) & 15u) != 0) return BCONV_EINVAL;
  const int h = packed_tile(s, variant_id);
  if (h < 0) return BCONV_EVARIANT;
  void* scratch = nullptr;
  rc = packed_scratch(h, s, &scratch);
  if (rc != BCONV_OK) return rc;
  return launch_hconv_packed(h, in, packed, bias, out, s, relu, in_layout == BCONV_LAYOUT_C8,
                             out_layout == BCONV_LAYOUT_C8, scratch, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? BCONV_OK
             : BCONV_ELAUNCH;
}

int conv_fwd_f16_layout_ex(const void* in, int in_layout, const void* filt, const float* bias, void* out,
                           int out_layout, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           int relu, void* workspace, size_t workspace_bytes, void* hip_stream, int variant_id) {
  if ((in_layout != BCONV_LAYOUT_NCHW && in_layout != BCONV_LAYOUT_C8) ||
      (out_layout != BCONV_LAYOUT_NCHW && out_layout != BCONV_LAYOUT_C8))
    return BCONV_EINVAL;
  if (in_layout == BCONV_LAYOUT_NCHW && out_layout == BCONV_LAYOUT_NCHW)
    return conv_fwd_f16_ex(in, filt, bias, out, N, C, H, W, K, R, S, stride, pad, relu, workspace, workspace_bytes,
                           hip_stream, variant_id);
  Shape s;
  int rc = check_conv_args(in, filt, out, N, C, H, W, K, R, S, stride, pad, relu, 2, &s);
  if (rc != BCONV_OK) return rc;
  if (in_layout == BCONV_LAYOUT_C8 && (C % 8 != 0 || (reinterpret_cast<uintptr_t>(in) & 15u) != 0)) return BCONV_EINVAL;
  if (out_layout == BCONV_LAYOUT_C8 && (K % 8 != 0 || (reinterpret_cast<uintptr_t>(out) & 15u) != 0)) return BCONV_EINVAL;
  if (images_per_launch(s) < s.N) return BCONV_EVARIANT;
  int id = variant_id;
  if (id < 0) {
    id = in_layout == BCONV_LAYOUT_C8 ? conv_fwd_f16_c8_selected_variant(N, C, H, W, K, R, S, stride, pad)
                                      : select_variant_f16(s, true, true);
    if (id < 0) return BCONV_EVARIANT;
  }
  const int h = hconv_index(id);
  if (h < 0 || !hconv_applicable(h, s)) return BCONV_EVARIANT;
  // channel-octet tiles write C8 from C8 input only; the first-layer tiles read NCHW only
  if (hconv_packable(h) ? (in_layout != BCONV_LAYOUT_C8) : (in_layout != BCONV_LAYOUT_NCHW)) return BCONV_EVARIANT;
  const size_t need = hconv_workspace_bytes(h, s);
  if (!workspace || workspace_bytes < need) return BCONV_EWORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 15u) != 0) return BCONV_EINVAL;
  return launch_hconv(h, in, filt, bias, out, s, relu, in_layout == BCONV_LAYOUT_C8, out_layout == BCONV_LAYOUT_C8,
                      workspace, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? BCONV_OK
             : BCONV_ELAUNCH;
}

int f16_layout_convert(const void* in, int in_layout, void* out, int out_layout, int N, int C, int H, int W,
                       void* hip_stream) {
  if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return BCONV_EINVAL;
  if (!in || !out) return BCONV_ENULL;
  if (in == out) return BCONV_EINVAL;
  const bool to_c8 = in_layout == BCONV_LAYOUT_NCHW && out_layout == BCONV_LAYOUT_C8;
  const bool from_c8 = in_layout == BCONV_LAYOUT_C8 && out_layout == BCONV_LAYOUT_NCHW;
  if ((!to_c8 && !from_c8) || C % 8 != 0) return BCONV_EINVAL;
  const void* c8 = to_c8 ? out : in;
  const void* plain = to_c8 ? in : out;
  if ((reinterpret_cast<uintptr_t>(c8) & 15u) != 0 || (reinterpret_cast<uintptr_t>(plain) & 1u) != 0)
    return BCONV_EINVAL;
  if ((long long)H * W > 0x7fffffffLL) return BCONV_ESHAPE;
  return launch_f16_layout(in, out, (long long)N * C, H * W, to_c8 ? 1 : 0, static_cast<hipStream_t>(hip_stream)) ==
                 hipSuccess
             ? BCONV_OK
             : BCONV_ELAUNCH;
}

// C[M x N] = A[M x K] * B[K x N] is the pointwise convolution of one "image" whose
// N columns are the pixels: filters = rows of A, channels = the reduction index.
int sgemm_ex(const float* A, const float* B, float* C, int M, int N, int K, void* workspace,
             size_t workspace_bytes, void* hip_stream, int variant_id) {
  return conv_fwd_ex(B, A, nullptr, C, 1, K, 1, N, M, 1, 1, 1, 0, 0, workspace, workspace_bytes,
                     hip_stream, variant_id);
}

int sgemm(const float* A, const float* B, float* C, int M, int N, int K) {
  return conv_fwd(B, A, nullptr, C, 1, K, 1, N, M, 1, 1, 1, 0, 0);
}

size_t sgemm_workspace_bytes(int M, int N, int K, int variant_id) {
  return conv_fwd_workspace_bytes(1, K, 1, N, M, 1, 1, 1, 0, variant_id);
}

int conv_num_variants(void) { return num_variants(); }

int conv_variant_name(int variant_id, char* buf, size_t buflen) {
  if (!buf || buflen == 0) return BCONV_ENULL;
  if (variant_id == 0) {
    std::snprintf(buf, buflen, "direct");
    return BCONV_OK;
  }
  if (fma_index(variant_id) >= 0) {
    std::snprintf(buf, buflen, "%s/s1", fma_variant_name(fma_index(variant_id)));
    return BCONV_OK;
  }
  if (hconv_index(variant_id) >= 0) {
    std::snprintf(buf, buflen, "%s/s%d", hconv_variant_name(hconv_index(variant_id)),
                  hconv_variant_split(hconv_index(variant_id)));
    return BCONV_OK;
  }
  int t, nsplit;
  if (!decode_variant(variant_id, &t, &nsplit)) return BCONV_EVARIANT;
  std::snprintf(buf, buflen, "%s/s%d", kTiles[t].name, nsplit);
  return BCONV_OK;
}

int conv_selected_variant(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
  Shape s;
  int rc = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
  if (rc != BCONV_OK) return rc;
  return select_variant(batch_of(s, images_per_launch(s)));
}

int conv_variant_applicable(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                            int variant_id) {
  Shape s;
  int rc = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
  if (rc != BCONV_OK) return rc;
  if (variant_id == 0) return 1;
  if (hconv_index(variant_id) >= 0) return 0;   // half-precision entry points only
  int t, nsplit;
  Plan pl;
  Shape runs[2];
  if (fma_index(variant_id) >= 0) {
    for (int i = 0, n = run_shapes(s, runs); i < n; ++i)
      if (!fma_conv_applicable(fma_index(variant_id), runs[i])) return 0;
    return 1;
  }
  if (!decode_variant(variant_id, &t, &nsplit)) return BCONV_EVARIANT;
  for (int i = 0, n = run_shapes(s, runs); i < n; ++i)
    if (!plan_tconv(runs[i], kTiles[t], nsplit, &pl)) return 0;
  return 1;
}

long long bconv_debug_audit(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                            int variant_id) {
  Shape s;
  int rc = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
  if (rc != BCONV_OK) return rc;
  if (variant_id == 0) return 0;
  int t, nsplit;
  Plan pl;
  // (the FMA kernels test every global index against the image bounds themselves)
  if (fma_index(variant_id) >= 0) return fma_conv_applicable(fma_index(variant_id), s) ? 0 : BCONV_EVARIANT;
  if (!decode_variant(variant_id, &t, &nsplit)) return BCONV_EVARIANT;
  Shape runs[2];
  long long bad = 0;
  for (int i = 0, n = run_shapes(s, runs); i < n; ++i) {
    if (!plan_tconv(runs[i], kTiles[t], nsplit, &pl)) return BCONV_EVARIANT;
    bad += audit(runs[i], kTiles[t], pl);
  }
  return bad;
}

double bconv_debug_model_cost(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                              int variant_id) {
  Shape s;
  if (make_shape(N, C, H, W, K, R, S, stride, pad, &s) != BCONV_OK) return -1.0;
  int t, nsplit;
  Plan pl;
  s = batch_of(s, images_per_launch(s));    // the estimate is per launch
  if (hconv_index(variant_id) >= 0) return hconv_model_cost(hconv_index(variant_id), s);
  if (!decode_variant(variant_id, &t, &nsplit) || !plan_tconv(s, kTiles[t], nsplit, &pl)) return -1.0;
  return variant_cost(kTiles[t], pl);
}

int maxpool_fwd(const float* in, float* out, int N, int C, int H, int W, int ksz, int stride,
                void* hip_stream) {
  if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || ksz <= 0 || stride <= 0) return BCONV_EINVAL;
  if (H < ksz || W < ksz) return BCONV_ESHAPE;
  if ((long long)N * C > 0x7fffffffLL || (long long)H * W > 0x7fffffffLL) return BCONV_ESHAPE;
  if (!in || !out) return BCONV_ENULL;
  int P = (H - ksz) / stride + 1, Q = (W - ksz) / stride + 1;
  return launch_maxpool(in, out, N, C, H, W, ksz, stride, P, Q,
                        static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? BCONV_OK
             : BCONV_ELAUNCH;
}

int maxpool_fwd_f16(const void* in, void* out, int layout, int N, int C, int H, int W, int ksz, int stride,
                    void* hip_stream) {
  if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || ksz <= 0 || stride <= 0) return BCONV_EINVAL;
  if (layout != BCONV_LAYOUT_NCHW && layout != BCONV_LAYOUT_C8) return BCONV_EINVAL;
  if (layout == BCONV_LAYOUT_C8 && C % 8 != 0) return BCONV_EINVAL;
  if (H < ksz || W < ksz) return BCONV_ESHAPE;
  if ((long long)N * C > 0x7fffffffLL || (long long)H * W > 0x7fffffffLL) return BCONV_ESHAPE;
  if (!in || !out) return BCONV_ENULL;
  const uintptr_t mask = layout == BCONV_LAYOUT_C8 ? 15u : 1u;
  if (((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & mask) != 0) return BCONV_EINVAL;
  const int P = (H - ksz) / stride + 1, Q = (W - ksz) / stride + 1;
  return launch_maxpool_f16(in, out, (long long)N * C, H, W, ksz, stride, P, Q, layout == BCONV_LAYOUT_C8,
                            static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? BCONV_OK
             : BCONV_ELAUNCH;
}

int bconv_debug_mfma_loop(float* out, int workgroups, int iters, void* hip_stream) {
  if (!out) return BCONV_ENULL;
  if (workgroups <= 0 || workgroups > 65536 || iters <= 0) return BCONV_EINVAL;
  return launch_mfma_loop(out, workgroups, iters, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? BCONV_OK
             : BCONV_ELAUNCH;
}

const char* bconv_strerror(int status) { return status_text(status); }

}  // extern "C"
