// Host-side sanitizer driver (CPU tests only): linked against a build of the library whose
// host code is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer, the host
// emulation of the tiled kernel and the C oracle, all instrumented the same way.  It walks
// the host-only entry points (validation, selection, planning, workspace queries, the bounds
// audit, names) over the benchmark shapes, ragged shapes and every variant, and runs a few
// emulated launches against the oracle.  No GPU is touched.  Exit status 0 = nothing found
// (a sanitizer report aborts the process).
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/bconv.h"

extern "C" {
long long emu_tconv(const float*, const float*, const float*, float*, int, int, int, int, int, int, int, int,
                    int, int, int, int);
int emu_num_tiles();
const char* emu_tile_name(int);
int oracle_conv_fwd(const float*, const float*, const float*, float*, int, int, int, int, int, int, int, int,
                    int, int);
int oracle_maxpool_fwd(const float*, float*, int, int, int, int, int, int);
int oracle_sgemm(const float*, const float*, float*, int, int, int);
}

static int fails = 0;
#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "san_driver: %s failed at line %d\n", #c, __LINE__); ++fails; } } while (0)

struct Sh { int N, C, H, W, K, R, S, st, pad; };

int main() {
  const Sh shapes[] = {
      {1, 3, 32, 32, 16, 3, 3, 1, 1},    {1, 3, 227, 227, 96, 11, 11, 4, 0}, {32, 96, 27, 27, 256, 5, 5, 1, 2},
      {1, 256, 13, 13, 384, 3, 3, 1, 1}, {5, 384, 13, 13, 256, 3, 3, 1, 1},  {32, 480, 14, 14, 192, 1, 1, 1, 0},
      {1, 832, 7, 7, 384, 1, 1, 1, 0},   {2, 13, 13, 13, 70, 3, 3, 1, 1},    {1, 5, 30, 31, 129, 1, 7, 1, 3},
      {3, 37, 7, 7, 50, 1, 1, 2, 0},     {2, 3, 37, 41, 70, 7, 7, 2, 3},     {1, 1, 1, 1, 1, 1, 1, 1, 0},
      {1, 2, 3, 3, 2, 3, 3, 1, 3},       {4000, 3, 227, 227, 96, 11, 11, 4, 0}};
  const int nv = conv_num_variants();
  CHECK(nv > 1);
  char name[96], tiny[4];
  for (const Sh& s : shapes) {
    int P = 0, Q = 0;
    CHECK(conv_out_dims(s.H, s.W, s.R, s.S, s.st, s.pad, &P, &Q) == BCONV_OK && P > 0 && Q > 0);
    const int sel = conv_selected_variant(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.st, s.pad);
    CHECK(sel >= 0 && sel < nv);
    CHECK(conv_variant_applicable(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.st, s.pad, sel) == 1);
    (void)conv_fwd_workspace_bytes(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.st, s.pad, -1);
    (void)conv_pool_fwd_workspace_bytes(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.st, s.pad, -1);
    if (P >= 3 && Q >= 3) CHECK(conv_pool_selected_variant(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.st, s.pad, 3, 2) >= 0);
    const bool walk = (long long)s.N * s.K * P * Q < 400000;   // the audit walks every workgroup
    for (int v = 0; v < nv; ++v) {
      const int ok = conv_variant_applicable(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.st, s.pad, v);
      CHECK(ok == 0 || ok == 1);
      if (!ok) continue;
      (void)conv_fwd_workspace_bytes(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.st, s.pad, v);
      (void)bconv_debug_model_cost(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.st, s.pad, v);
      if (walk && v % 7 == 0) CHECK(bconv_debug_audit(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.st, s.pad, v) == 0);
    }
  }
  for (int v = 0; v < nv; v += 11) {
    CHECK(conv_variant_name(v, name, sizeof(name)) == BCONV_OK && std::strlen(name) > 0);
    CHECK(conv_variant_name(v, tiny, sizeof(tiny)) == BCONV_OK && std::strlen(tiny) <= 3);
  }
  // argument errors never reach a launch (null pointers are refused before anything else is read)
  CHECK(conv_fwd(nullptr, nullptr, nullptr, nullptr, 1, 3, 8, 8, 4, 3, 3, 1, 1, 0) == BCONV_ENULL);
  CHECK(conv_fwd_noalloc(nullptr, nullptr, nullptr, nullptr, 1, 3, 8, 8, 4, 3, 3, 1, 1, 0, nullptr) == BCONV_ENULL);
  CHECK(conv_fwd_ex(nullptr, nullptr, nullptr, nullptr, 0, 3, 8, 8, 4, 3, 3, 1, 1, 0, nullptr, 0, nullptr, -1) == BCONV_EINVAL);
  CHECK(conv_variant_name(nv, name, sizeof(name)) == BCONV_EVARIANT);
  CHECK(conv_variant_name(0, nullptr, 0) == BCONV_ENULL);
  CHECK(std::strlen(bconv_strerror(-99)) > 0);

  // a few emulated launches (every LDS and global index bounds-checked by the emulator, every
  // heap access by the sanitizer) against the oracle, small-integer data: bitwise equal
  const struct { const char* tile; Sh s; int split; } cases[] = {
      {"k3_64x64_k12_h", {2, 5, 13, 13, 40, 3, 3, 1, 1}, 1},
      {"k3_16x16m_k96_s8_v4_hf", {2, 44, 13, 13, 50, 3, 3, 1, 1}, 1},
      {"pw_32x32_k32_s4_v4b4", {2, 100, 14, 14, 70, 1, 1, 1, 0}, 1},
      {"pw_16x16m_k64_s4_v4", {1, 200, 7, 7, 20, 1, 1, 1, 0}, 2},
      {"k11s4_32x128_k2_np", {1, 3, 51, 47, 10, 11, 11, 4, 0}, 2},
      {"k5_32x128_k10_h", {1, 6, 14, 14, 33, 5, 5, 1, 2}, 1},
      {"gen_64x64_k2", {2, 3, 9, 10, 7, 2, 4, 2, 1}, 1}};
  for (const auto& c : cases) {
    int tile = -1;
    for (int t = 0; t < emu_num_tiles(); ++t)
      if (std::strcmp(emu_tile_name(t), c.tile) == 0) tile = t;
    CHECK(tile >= 0);
    const Sh& s = c.s;
    int P = 0, Q = 0;
    conv_out_dims(s.H, s.W, s.R, s.S, s.st, s.pad, &P, &Q);
    std::vector<float> x((size_t)s.N * s.C * s.H * s.W), f((size_t)s.K * s.C * s.R * s.S), b(s.K);
    unsigned seed = 12345u + (unsigned)tile;
    auto next = [&]() { seed = seed * 1664525u + 1013904223u; return (float)((int)((seed >> 16) % 5) - 2); };
    for (float& v : x) v = next();
    for (float& v : f) v = next();
    for (float& v : b) v = next();
    std::vector<float> got((size_t)s.N * s.K * P * Q, -7.0f), ref(got.size(), 7.0f);
    const long long rc = emu_tconv(x.data(), f.data(), b.data(), got.data(), s.N, s.C, s.H, s.W, s.K, s.R, s.S,
                                   s.st, s.pad, 1, tile, c.split);
    CHECK(rc == 0);
    CHECK(oracle_conv_fwd(x.data(), f.data(), b.data(), ref.data(), s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.st,
                          s.pad, 1) == 0);
    CHECK(std::memcmp(got.data(), ref.data(), got.size() * sizeof(float)) == 0);
    if (P >= 3 && Q >= 3) {
      std::vector<float> pooled((size_t)s.N * s.K * ((P - 3) / 2 + 1) * ((Q - 3) / 2 + 1));
      CHECK(oracle_maxpool_fwd(ref.data(), pooled.data(), s.N, s.K, P, Q, 3, 2) == 0);
    }
  }
  {
    std::vector<float> a(7 * 5, 1.0f), bm(5 * 3, 2.0f), cm(7 * 3);
    CHECK(oracle_sgemm(a.data(), bm.data(), cm.data(), 7, 3, 5) == 0 && cm[20] == 10.0f);
  }
  if (fails) return 1;
  std::puts("san_driver: ok");
  return 0;
}
