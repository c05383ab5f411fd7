"""CPU checks of the tiled kernel's host logic and indexing.

``tests/host_emu/emu_tconv.cpp`` walks the device kernel's own index functions
and launch plan thread by thread on the CPU (bounds-checked, LDS poisoned) and
models the MFMA by its definition.  Small-integer data makes fp32 exact in any
order, so the emulated result must equal the oracle bit for bit; any staging,
padding, tail or split mistake shows up here before a kernel is launched.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle
import workloads

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "host_emu", "emu_tconv.cpp")
LIB = os.path.join(HERE, "host_emu", "libemu.so")
_f32p = ctypes.POINTER(ctypes.c_float)


@pytest.fixture(scope="module")
def emu():
    csrc = os.path.join(HERE, "..", "paper_1606_00094_amd", "csrc")
    deps = [SRC] + [os.path.join(csrc, f) for f in ("bconv_plan.h", "bconv_geom.h", "variants.def")]
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < max(os.path.getmtime(d) for d in deps):
        subprocess.run(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", LIB, SRC], check=True)
    lib = ctypes.CDLL(LIB)
    lib.emu_tconv.argtypes = [_f32p] * 4 + [ctypes.c_int] * 12
    lib.emu_tconv.restype = ctypes.c_longlong
    lib.emu_num_tiles.restype = ctypes.c_int
    lib.emu_tile_name.restype = ctypes.c_char_p
    lib.emu_tile_name.argtypes = [ctypes.c_int]
    return lib


def _tiles(lib):
    return {lib.emu_tile_name(t).decode(): t for t in range(lib.emu_num_tiles())}


def _run(lib, tile, nsplit, x, f, b, stride, pad, relu):
    N, C, H, W = x.shape
    K, _, R, S = f.shape
    P, Q = oracle.conv_out_dims(H, W, R, S, stride, pad)
    out = np.full((N, K, P, Q), np.nan, np.float32)
    ptr = lambda a: a.ctypes.data_as(_f32p)
    rc = lib.emu_tconv(ptr(x), ptr(f), ptr(b) if b is not None else None, ptr(out),
                       N, C, H, W, K, R, S, stride, pad, int(relu), tile, nsplit)
    return rc, out


# (tile name, N, C, H, W, K, R, S, stride, pad, nsplit)
CASES = [
    ("k3_64x64_k12", 2, 5, 13, 13, 40, 3, 3, 1, 1, 1),
    ("k3_64x64_k12", 3, 13, 13, 13, 70, 3, 3, 1, 1, 2),
    ("k3_128x128_k12", 2, 7, 13, 13, 130, 3, 3, 1, 1, 1),
    ("k3_32x128_k12", 1, 3, 32, 32, 16, 3, 3, 1, 1, 1),
    ("k3_64x64_k12", 1, 6, 9, 200, 33, 3, 3, 1, 0, 1),      # wide rows: Q > BN
    ("k3_64x64_k12", 1, 4, 6, 7, 5, 3, 3, 1, 3, 1),         # pad >= kernel
    ("k5_64x64_k8", 2, 3, 11, 9, 20, 5, 5, 1, 2, 1),
    ("k5_32x128_k8", 1, 16, 28, 28, 32, 5, 5, 1, 2, 2),
    ("pw_64x64_k16", 3, 21, 7, 7, 50, 1, 1, 1, 0, 1),
    ("pw_128x128_k16", 2, 33, 14, 14, 100, 1, 1, 1, 0, 3),
    ("pw_32x128_k16", 1, 5, 28, 28, 9, 1, 1, 1, 0, 1),
    ("k11s4_32x128_k4", 1, 3, 67, 71, 20, 11, 11, 4, 0, 1),
    ("k11s4_96x128_k4", 2, 3, 43, 43, 96, 11, 11, 4, 0, 3),
    ("k11s4_96x64_k4", 1, 3, 51, 47, 10, 11, 11, 4, 2, 1),
    ("k3_64x64_k12_v4", 2, 8, 13, 13, 40, 3, 3, 1, 1, 1),
    ("k3_128x128_k12_v4", 2, 12, 13, 13, 130, 3, 3, 1, 1, 1),
    ("k3_64x128_k12", 2, 5, 13, 13, 40, 3, 3, 1, 1, 1),
    ("k5_128x64_k8_v4", 1, 4, 27, 27, 130, 5, 5, 1, 2, 1),
    ("k5_128x64_k8", 1, 3, 27, 27, 260, 5, 5, 1, 2, 1),
    ("pw_64x256_k16_v4", 2, 20, 14, 14, 70, 1, 1, 1, 0, 1),
    ("pw_64x256_k32_v4", 3, 68, 7, 7, 130, 1, 1, 1, 0, 2),
    ("pw_64x128_k16", 2, 6, 5, 9, 40, 1, 1, 1, 1, 1),           # pointwise with padding
    ("pw_64x128_k16_v4b4", 3, 20, 14, 14, 70, 1, 1, 1, 0, 1),   # 16-byte input loads
    ("k11s4_96x64_k4", 2, 3, 67, 71, 96, 11, 11, 4, 0, 1),
    ("k11s4_32x128_k2", 1, 3, 51, 47, 10, 11, 11, 4, 2, 2),
    ("k3_128x64_k12_s2_v4_h", 2, 12, 13, 13, 130, 3, 3, 1, 1, 1),   # reduction split inside the workgroup
    ("k3_64x64_k12_s2_h", 2, 7, 13, 13, 40, 3, 3, 1, 1, 2),
    ("pw_128x128_k16_s2_v4", 2, 68, 14, 14, 130, 1, 1, 1, 0, 1),
    ("k11s4_32x256_k6_s3", 1, 3, 67, 71, 96, 11, 11, 4, 0, 1),
    ("k3_64x64_k12_h", 2, 5, 13, 13, 40, 3, 3, 1, 1, 1),          # halo staging: one copy of the input rows
    ("k3_64x64_k12_h", 3, 13, 13, 13, 70, 3, 3, 1, 1, 2),
    ("k3_128x128_k12_v4_h", 2, 8, 13, 13, 130, 3, 3, 1, 1, 1),
    ("k3_64x256_k12_h", 3, 5, 13, 13, 40, 3, 3, 1, 1, 1),         # tile spans more than one image
    ("k3_32x128_k12_h", 1, 3, 32, 32, 16, 3, 3, 1, 1, 1),
    ("k3_64x64_k12_h", 1, 4, 6, 7, 5, 3, 3, 1, 3, 1),             # pad >= kernel
    ("k3_64x64_k12_h", 1, 6, 9, 20, 33, 3, 3, 1, 0, 1),
    ("k3_64x128_k12_s2_h", 2, 7, 13, 13, 40, 3, 3, 1, 1, 2),
    ("k3_128x64_k24_s2_v4_h", 2, 12, 13, 13, 130, 3, 3, 1, 1, 1),
    ("k5_64x64_k10_h", 2, 3, 11, 9, 20, 5, 5, 1, 2, 1),
    ("k5_64x128_k20_v4_h", 1, 16, 27, 27, 70, 5, 5, 1, 2, 2),
    ("k5_128x64_k20_s2_v4_h", 1, 4, 27, 27, 130, 5, 5, 1, 2, 1),
    ("pw_64x96w_k16_s2_v4", 2, 68, 14, 14, 70, 1, 1, 1, 0, 1),        # three pixel tiles per wave
    ("pw_64x192w_k16_s2_v4", 3, 132, 7, 7, 100, 1, 1, 1, 0, 1),       # three filter tiles per wave
    ("pw_64x96w_k16_s2", 1, 21, 6, 6, 97, 1, 1, 1, 0, 1),
    ("pw_32x192w_k16_s2_v4", 2, 132, 14, 14, 40, 1, 1, 1, 0, 1),
    ("pw_64x128_k16_v4_p4", 2, 68, 14, 14, 70, 1, 1, 1, 0, 1),        # four register sets
    ("pw_64x128_k16_p4", 2, 137, 9, 9, 200, 1, 1, 1, 0, 3),
    ("k11s4_96x128_k2_p4", 1, 3, 51, 47, 96, 11, 11, 4, 0, 1),
    ("k7s2_64x128_k2", 2, 3, 37, 41, 70, 7, 7, 2, 3, 1),            # 7x7 stride 2 with padding
    ("k7s2_64x256_k2", 1, 3, 64, 64, 64, 7, 7, 2, 3, 2),
    ("k7s2_64x128_k6_s3", 1, 2, 30, 29, 33, 7, 7, 2, 0, 1),
    ("pw_32x32_k32_s4_v4b4", 2, 100, 14, 14, 70, 1, 1, 1, 0, 1),      # fine-grained tiles, reduction split over the waves
    ("pw_32x32_k64_s4_v4", 3, 132, 7, 7, 40, 1, 1, 1, 0, 1),
    ("pw_32x64_k32_s2_v4b4", 2, 68, 14, 14, 70, 1, 1, 1, 0, 2),
    ("pw_64x32_k32_s2", 1, 37, 9, 9, 100, 1, 1, 1, 0, 1),
    ("pw_64x64_k32_s2_v4b4", 2, 68, 14, 14, 130, 1, 1, 1, 0, 1),
    ("pw_32x32_k64_s4_v4b4", 2, 132, 14, 14, 33, 1, 1, 1, 0, 1),
    ("pw_32x32_k128_s8_v4b4", 2, 300, 14, 14, 40, 1, 1, 1, 0, 1),
    ("pw_32x32_k64_s8_v4", 1, 132, 7, 7, 70, 1, 1, 1, 0, 1),
    ("pw_64x32_k64_s4_v4b4", 2, 132, 14, 14, 70, 1, 1, 1, 0, 2),
    ("k3_32x32_k24_s4_v4_h", 2, 20, 13, 13, 70, 3, 3, 1, 1, 1),
    ("k3_32x64_k48_s4_h", 1, 37, 13, 13, 40, 3, 3, 1, 1, 1),
    ("k3_64x32_k24_s4_v4_h", 2, 32, 9, 11, 100, 3, 3, 1, 1, 2),
    ("k3_32x64_k24_s4_v4_h", 1, 24, 28, 28, 70, 3, 3, 1, 1, 1),
    ("k5_32x32_k40_s4_v4_h", 2, 16, 12, 12, 33, 5, 5, 1, 2, 1),
    ("k5_32x64_k40_s4_h", 1, 19, 27, 27, 40, 5, 5, 1, 2, 1),
    ("k5_32x32_k20_s2_h", 2, 7, 14, 10, 20, 5, 5, 1, 2, 1),
    ("k11s4_96x128_k2_np", 2, 3, 51, 47, 70, 11, 11, 4, 0, 1),         # slot staging without padding: scalar addressing
    ("k11s4_32x128_k4_s2_np", 1, 5, 35, 39, 40, 11, 11, 4, 0, 3),
    ("k11s4_96x128_k2_np_w3", 3, 2, 27, 31, 97, 11, 11, 4, 0, 1),
    ("k7s2_64x128_k2_np", 1, 3, 41, 37, 70, 7, 7, 2, 0, 1),
    ("gen_64x64_k2_np", 2, 5, 12, 17, 40, 2, 5, 3, 0, 2),
    ("gen_32x128_k2_np", 1, 4, 9, 30, 33, 1, 4, 1, 0, 1),
    ("pws2_64x128_k16_v4_np", 2, 20, 14, 14, 70, 1, 1, 2, 0, 1),    # the same with scalar addressing
    ("pws2_32x128_k16_np", 1, 37, 28, 27, 40, 1, 1, 2, 0, 2),
    ("k3s2_64x64_k12_v4_np", 2, 20, 15, 13, 70, 3, 3, 2, 0, 1),
    ("k3s2_32x128_k12_np", 1, 7, 27, 27, 33, 3, 3, 2, 0, 1),
    ("pws2_64x128_k16_v4", 2, 20, 14, 14, 70, 1, 1, 2, 0, 1),       # stride-2 pointwise
    ("pws2_32x128_k16", 1, 37, 28, 27, 40, 1, 1, 2, 1, 2),
    ("k3s2_64x64_k12_v4", 2, 12, 27, 27, 70, 3, 3, 2, 0, 1),        # 3x3 stride 2
    ("k3s2_128x128_k12", 1, 7, 28, 30, 130, 3, 3, 2, 1, 1),
    ("k1x7_64x128_k8_v4", 2, 12, 17, 17, 70, 1, 7, 1, 0, 1),        # one-row and one-column kernels
    ("k1x7_32x128_k8", 1, 5, 9, 30, 20, 1, 7, 1, 3, 1),
    ("k7x1_64x64_k14", 2, 12, 17, 17, 70, 7, 1, 1, 0, 1),
    ("k7x1_128x128_k14", 1, 5, 30, 9, 130, 7, 1, 1, 3, 2),
    ("gen_64x64_k2", 2, 3, 9, 10, 7, 2, 4, 2, 1, 1),
    ("gen_64x64_k2", 2, 3, 9, 10, 7, 3, 1, 1, 1, 1),            # S = 1, stride 1, R = 3: compact cells
    ("gen_64x64_k2", 1, 2, 12, 12, 5, 3, 3, 3, 2, 2),
    ("gen_32x128_k2", 1, 4, 8, 8, 6, 1, 1, 2, 0, 1),        # strided pointwise: no flattening
    ("gen_128x128_k2", 1, 3, 20, 17, 9, 7, 7, 2, 3, 1),
    ("gen_64x64_k2", 1, 1, 5, 40, 3, 1, 16, 1, 0, 1),        # widest generic kernel
    # 16x16x4 accumulator tiles (four reduction rows per MFMA), flat halo staging
    ("k3_16x16m_k96_s8_v4_hf", 1, 256, 13, 13, 40, 3, 3, 1, 1, 1),
    ("k3_16x16m_k96_s8_v4_hf", 2, 44, 13, 13, 50, 3, 3, 1, 1, 1),   # ragged channels: planes past the last one
    ("k3_16x16m_k96_s8_hf", 1, 70, 9, 11, 21, 3, 3, 1, 1, 2),
    ("k3_16x16m_k48_s4_v4_hf", 2, 20, 13, 13, 33, 3, 3, 1, 1, 1),
    ("k3_16x32m_k48_s4_v4_hf", 1, 24, 13, 13, 70, 3, 3, 1, 1, 1),
    ("k3_16x32m_k48_s4_hf", 3, 7, 6, 7, 17, 3, 3, 1, 0, 1),
    ("k3_32x16m_k48_s4_v4_hf", 2, 40, 13, 13, 40, 3, 3, 1, 1, 2),
    ("k3_32x32m_k24_s2_v4_hf", 1, 12, 28, 28, 50, 3, 3, 1, 1, 1),
    ("k3_16x32m_k96_s8_v4_hf", 1, 100, 13, 13, 20, 3, 3, 1, 1, 1),
    ("k3_32x32m_k48_s4_v4_hf", 2, 24, 13, 13, 70, 3, 3, 1, 3, 1),   # pad >= kernel
    ("k5_16x16m_k80_s4_v4_hf", 1, 20, 27, 27, 20, 5, 5, 1, 2, 1),
    ("k5_16x32m_k80_s4_v4_hf", 2, 16, 14, 12, 33, 5, 5, 1, 2, 1),
    ("k5_32x32m_k40_s2_v4_hf", 1, 20, 28, 28, 40, 5, 5, 1, 2, 2),
    ("k11s4_16x64m_k4_np", 1, 3, 67, 71, 20, 11, 11, 4, 0, 1),
    ("k11s4_16x128m_k4_np", 2, 3, 51, 47, 40, 11, 11, 4, 0, 1),
    ("k11s4_32x64m_k4_np", 1, 3, 227, 227, 33, 11, 11, 4, 0, 1),
    ("k11s4_16x64m_k8_s2_np", 1, 3, 43, 43, 17, 11, 11, 4, 0, 2),
    ("pw_16x16m_k32_s8_v4", 2, 100, 7, 7, 40, 1, 1, 1, 0, 1),
    ("pw_16x16m_k64_s8_v4", 1, 132, 7, 7, 70, 1, 1, 1, 0, 1),
    ("pw_16x16m_k64_s8", 3, 137, 5, 5, 21, 1, 1, 1, 0, 2),
    ("pw_16x32m_k64_s8_v4", 2, 68, 14, 14, 33, 1, 1, 1, 0, 1),
    ("pw_16x16m_k64_s4_v4", 1, 200, 14, 14, 20, 1, 1, 1, 0, 1),
    ("pw_32x32m_k32_s4_v4", 2, 36, 9, 9, 50, 1, 1, 1, 0, 1),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "%s-N%dC%dH%dW%dK%dR%dS%ds%dp%d-sk%d" % c)
def test_emulated_kernel_matches_oracle_bitwise_on_integers(emu, case):
    name, N, C, H, W, K, R, S, stride, pad, nsplit = case
    tile = _tiles(emu)[name]
    x, f, b = workloads.make_integer_problem(hash(case) % 10000, N, C, H, W, K, R, S)
    for relu in (False, True):
        rc, got = _run(emu, tile, nsplit, x, f, b, stride, pad, relu)
        assert rc == 0, "emulation reported %d (1 = tile not applicable, >1 = bad accesses)" % rc
        ref = oracle.conv_fwd(x, f, b, stride=stride, pad=pad, relu=relu)
        assert np.array_equal(got, ref)


def test_emulated_kernel_float_data_within_tolerance(emu):
    tile = _tiles(emu)["k3_64x64_k12"]
    x, f, b = workloads.make_random_problem(5, 2, 24, 13, 13, 48, 3, 3)
    rc, got = _run(emu, tile, 1, x, f, b, 1, 1, False)
    assert rc == 0
    ref = oracle.conv_fwd(x, f, b, stride=1, pad=1)
    assert np.all(np.abs(got - ref) <= np.maximum(1e-5, 1e-4 * np.abs(ref)))


def test_tile_that_does_not_apply_is_refused(emu):
    tile = _tiles(emu)["k3_64x64_k12"]
    x, f, b = workloads.make_integer_problem(1, 1, 2, 8, 8, 4, 5, 5)
    rc, _ = _run(emu, tile, 1, x, f, b, 1, 2, False)
    assert rc == 1
    # a no-padding tile must refuse a padded layer
    tile = _tiles(emu)["k11s4_32x128_k2_np"]
    x, f, b = workloads.make_integer_problem(2, 1, 3, 40, 40, 8, 11, 11)
    assert _run(emu, tile, 1, x, f, b, 4, 2, False)[0] == 1
    assert _run(emu, tile, 1, x, f, b, 4, 0, False)[0] == 0


def test_fast_division_matches_integer_division(emu):
    """The multiply-and-shift quotient the kernel's index math uses, against n // d: all
    small pairs, divisors around powers of two, the largest dividends, random pairs."""
    rng = np.random.default_rng(77)
    top = 2 ** 31 - 1
    ds = list(range(1, 300)) + [2 ** k + o for k in range(8, 31) for o in (-1, 0, 1)] + [top, top - 1, 3025, 729, 169]
    ns, dd = [], []
    for d in ds:
        d = min(d, top)
        cand = [0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, top, top - 1, top // 2] + \
            [int(x) for x in rng.integers(0, top, size=40)] + [(top // d) * d - 1, (top // d) * d]
        for n in cand:
            if 0 <= n <= top:
                ns.append(n); dd.append(d)
    n_small, d_small = np.meshgrid(np.arange(0, 2000), np.arange(1, 400))
    ns = np.concatenate([np.array(ns, dtype=np.int32), n_small.ravel().astype(np.int32)])
    dd = np.concatenate([np.array(dd, dtype=np.int32), d_small.ravel().astype(np.int32)])
    emu.emu_fastdiv_check.restype = ctypes.c_longlong
    emu.emu_fastdiv_check.argtypes = [ctypes.POINTER(ctypes.c_int)] * 2 + [ctypes.c_longlong]
    ptr = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int))
    bad = emu.emu_fastdiv_check(ptr(ns), ptr(dd), len(ns))
    assert bad == -1, (int(ns[bad]), int(dd[bad]))


@pytest.mark.parametrize("filter_major", [0, 1])
@pytest.mark.parametrize("grid", [(183, 8, 1), (85, 6, 1), (3, 6, 8), (1, 1, 1), (5, 3, 4), (757, 1, 1), (7, 11, 3)])
def test_block_to_tile_map_is_a_bijection_that_groups_tiles_by_die(emu, grid, filter_major):
    """Every tile of the grid is computed exactly once, and the workgroups of one die
    (dispatch position mod 8) cover one contiguous run of the (split, pixel, filter) list, or
    of the (split, filter, pixel) list in the filter-major order."""
    gx, gy, gz = grid
    emu.emu_xcd_tile.argtypes = [ctypes.c_uint] * 4 + [ctypes.c_int] + [ctypes.POINTER(ctypes.c_int)] * 3
    emu.emu_xcd_tile.restype = None
    seen, by_die = set(), {}
    for lin in range(gx * gy * gz):
        x, y, z = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
        emu.emu_xcd_tile(lin, gx, gy, gz, filter_major, ctypes.byref(x), ctypes.byref(y), ctypes.byref(z))
        assert 0 <= x.value < gx and 0 <= y.value < gy and 0 <= z.value < gz
        seen.add((x.value, y.value, z.value))
        pos = (z.value * gy + y.value) * gx + x.value if filter_major else (z.value * gx + x.value) * gy + y.value
        by_die.setdefault(lin % 8, []).append(pos)
    assert len(seen) == gx * gy * gz
    for die, idx in by_die.items():
        assert idx == list(range(idx[0], idx[0] + len(idx)))


def test_emulated_kernel_fuzz_over_tiles_and_shapes(emu):
    """Seeded random (tile, shape, split) draws: whenever the planner accepts the combination
    the emulated kernel must be free of out-of-range accesses and bitwise equal to the oracle."""
    rng = np.random.default_rng(160600094)
    tiles = _tiles(emu)
    names = sorted(tiles)
    fam = {"pw": (1, 1, 1), "k3": (3, 3, 1), "k5": (5, 5, 1), "k11s4": (11, 11, 4), "k7s2": (7, 7, 2),
           "pws2": (1, 1, 2), "k3s2": (3, 3, 2), "k1x7": (1, 7, 1), "k7x1": (7, 1, 1)}
    ran = 0
    for it in range(400):
        name = names[int(rng.integers(len(names)))]
        prefix = name.split("_")[0]
        if prefix == "gen":
            R, S, stride = int(rng.integers(1, 5)), int(rng.integers(1, 5)), int(rng.integers(1, 4))
        else:
            R, S, stride = fam[prefix]
        pad = int(rng.integers(0, R + 1))
        lo = max(1, R - 2 * pad)
        H = int(rng.integers(lo, lo + 12 * stride))
        W = int(rng.integers(max(1, S - 2 * pad), max(1, S - 2 * pad) + 14 * stride))
        N, K = int(rng.integers(1, 4)), int(rng.integers(1, 140))
        C = int(rng.integers(1, 40))
        if "_v4" in name:
            C = 4 * max(1, C // 4)            # 16-byte filter loads need C*R*S % 4 == 0
        nsplit = int(rng.choice([1, 1, 2, 3, 4]))
        x, f, b = workloads.make_integer_problem(it, N, C, H, W, K, R, S)
        rc, got = _run(emu, tiles[name], nsplit, x, f, b, stride, pad, bool(it & 1))
        if rc == 1:
            continue                           # tile does not apply to this shape
        what = "%s N%d C%d H%d W%d K%d R%d S%d s%d p%d split %d" % (name, N, C, H, W, K, R, S, stride, pad, nsplit)
        assert rc == 0, what
        ref = oracle.conv_fwd(x, f, b, stride=stride, pad=pad, relu=bool(it & 1))
        assert np.array_equal(got, ref), what
        ran += 1
    assert ran >= 120
