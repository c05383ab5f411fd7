"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP library.  Each names the passage or the
mathematical fact it rests on.
"""
import os

import numpy as np
import pytest

import oracle
import workloads
from tests import bruteforce

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_kv(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split()
            out[k] = float(v)
    return out


# ---------------------------------------------------------------- P1 / P2 / P10
def test_worked_example_sizes_from_paper():
    """Section II/III running example: 205x205x3, 96 filters 7x7, stride 2."""
    g = _golden_kv("worked_example.txt")
    P, Q = oracle.conv_out_dims(int(g["in_Y"]), int(g["in_X"]), int(g["filts_KSZ"]),
                                int(g["filts_KSZ"]), int(g["stride"]), 0)
    assert (P, Q) == (int(g["out_Y"]), int(g["out_X"]))
    assert int(g["filts_KSZ"]) ** 2 * int(g["in_C"]) == int(g["window_elems"])
    assert P * Q * int(g["filts_OC"]) == int(g["output_points"])
    assert P * Q == int(g["inmat_rows"])
    # the oracle really produces that many points on that shape (one image, 2 filters)
    x = np.zeros((1, 3, 205, 205), np.float32)
    f = np.zeros((2, 3, 7, 7), np.float32)
    assert oracle.conv_fwd(x, f, stride=2).shape == (1, 2, 100, 100)


@pytest.mark.parametrize("H,R,s,p,expect", [
    (227, 11, 4, 0, 55), (27, 5, 1, 2, 27), (13, 3, 1, 1, 13), (32, 3, 1, 1, 32),
    (10, 3, 2, 0, 4),      # not divisible: floor
    (7, 1, 1, 0, 7), (5, 5, 3, 0, 1), (4, 3, 1, 3, 8), (9, 2, 2, 0, 4),
])
def test_out_dims_formula(H, R, s, p, expect):
    assert oracle.conv_out_dims(H, H, R, R, s, p) == (expect, expect)


def test_out_dims_rejects_impossible():
    for args in [(3, 3, 5, 5, 1, 0), (0, 3, 1, 1, 1, 0), (3, 3, 1, 1, 0, 0), (3, 3, 1, 1, 1, -1)]:
        with pytest.raises(ValueError):
            oracle.conv_out_dims(*args)


@pytest.mark.parametrize("R", [1, 3, 5, 7, 11])
def test_same_size_with_half_padding(R):
    """Section II: pad floor(KSZ/2), stride 1 -> same spatial size."""
    x, f, _ = workloads.make_random_problem(R, 1, 2, 12, 17, 2, R, R)
    assert oracle.conv_fwd(x, f, pad=R // 2).shape == (1, 2, 12, 17)


# ---------------------------------------------------------------- hand-computed
def test_hand_computed_2x2_no_flip():
    """Literal numbers: cross-correlation (window times filter, no flip)."""
    x = np.arange(1, 10, dtype=np.float32).reshape(1, 1, 3, 3)
    f = np.array([[1, 2], [3, 4]], np.float32).reshape(1, 1, 2, 2)
    out = oracle.conv_fwd(x, f)
    assert out.reshape(-1).tolist() == [37.0, 47.0, 67.0, 77.0]


def test_hand_computed_stride_pad_bias():
    """3x3 image, 2x2 filter, stride 2, pad 1, bias 0.5: four corner windows."""
    x = np.arange(1, 10, dtype=np.float32).reshape(1, 1, 3, 3)
    f = np.array([[1, 2], [3, 4]], np.float32).reshape(1, 1, 2, 2)
    b = np.array([0.5], np.float32)
    out = oracle.conv_fwd(x, f, b, stride=2, pad=1)
    # windows start at (-1,-1), (-1,1), (1,-1), (1,1)
    expect = [4 * 1 + 0.5, 3 * 2 + 4 * 3 + 0.5, 2 * 4 + 4 * 7 + 0.5,
              1 * 5 + 2 * 6 + 3 * 8 + 4 * 9 + 0.5]
    assert out.shape == (1, 1, 2, 2)
    assert out.reshape(-1).tolist() == expect


def test_hand_computed_two_channels_two_filters():
    x = np.array([[[1, 2]], [[10, 20]]], np.float32).reshape(1, 2, 1, 2)
    f = np.array([[[[1, -1]], [[2, 0]]], [[[0, 3]], [[0, -1]]]], np.float32)  # K=2,C=2,R=1,S=2
    out = oracle.conv_fwd(x, f)
    assert out.reshape(-1).tolist() == [1 - 2 + 20, 6 - 20]


# ---------------------------------------------------------------- P3 / P6
TINY = [
    # N C H  W  K R S s p
    (1, 1, 4, 4, 1, 2, 2, 1, 0),
    (2, 3, 7, 9, 4, 3, 3, 1, 1),
    (1, 2, 9, 6, 3, 3, 2, 2, 0),
    (2, 3, 8, 8, 2, 2, 3, 3, 2),
    (1, 3, 9, 9, 4, 1, 1, 1, 0),
    (1, 2, 5, 7, 3, 5, 3, 1, 2),
    (1, 1, 3, 3, 2, 3, 3, 1, 3),   # pad >= kernel: some windows all padding
    (2, 2, 6, 5, 2, 1, 3, 2, 1),
]


@pytest.mark.parametrize("shape", TINY)
@pytest.mark.parametrize("relu", [False, True])
def test_im2col_matmul_bruteforce_integer_exact(shape, relu):
    """Section III: conv == inmat x filtsmat.  Integer data -> bitwise equal."""
    N, C, H, W, K, R, S, s, p = shape
    x, f, b = workloads.make_integer_problem(sum(shape), N, C, H, W, K, R, S)
    got = oracle.conv_fwd(x, f, b, stride=s, pad=p, relu=relu)
    ref = bruteforce.conv_im2col(x, f, b, stride=s, pad=p, relu=relu, loops=True)
    assert got.shape == ref.shape
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("shape", TINY)
def test_im2col_matmul_bruteforce_float(shape):
    """Same on real-valued data: both accumulate in double in different orders,
    so after the single rounding they agree to at most one fp32 ulp."""
    N, C, H, W, K, R, S, s, p = shape
    x, f, b = workloads.make_random_problem(1000 + sum(shape), N, C, H, W, K, R, S)
    got = oracle.conv_fwd(x, f, b, stride=s, pad=p)
    ref = bruteforce.conv_im2col(x, f, b, stride=s, pad=p, loops=True)
    ulp = np.abs(got.view(np.int32).astype(np.int64) - ref.view(np.int32).astype(np.int64))
    assert ulp.max() <= 1
    assert (ulp == 0).mean() > 0.99


def test_im2col_matmul_medium_library_matmul():
    """A mid-sized case against numpy's float64 matmul (several channels,
    non-square image and kernel, stride 2)."""
    x, f, b = workloads.make_random_problem(7, 2, 5, 19, 23, 6, 4, 3)
    got = oracle.conv_fwd(x, f, b, stride=2, pad=2, relu=True)
    ref = bruteforce.conv_im2col(x, f, b, stride=2, pad=2, relu=True, loops=False)
    np.testing.assert_allclose(got, ref, rtol=3e-7, atol=1e-7)


# ---------------------------------------------------------------- P4
@pytest.mark.parametrize("R", [1, 3, 5])
def test_delta_filter_reproduces_input(R):
    C = 3
    x, _, _ = workloads.make_random_problem(11 + R, 2, C, 9, 11, C, R, R)
    f = np.zeros((C, C, R, R), np.float32)
    for c in range(C):
        f[c, c, R // 2, R // 2] = 1.0
    out = oracle.conv_fwd(x, f, pad=R // 2)
    assert np.array_equal(out, x)


def test_shifted_delta_filter_shifts_input():
    """A one at filter tap (r, s) reads in[y+r-pad, x+s-pad]: direction check."""
    x, _, _ = workloads.make_random_problem(5, 1, 1, 6, 7, 1, 3, 3)
    f = np.zeros((1, 1, 3, 3), np.float32)
    f[0, 0, 0, 2] = 1.0          # r=0 (up), s=2 (right)
    out = oracle.conv_fwd(x, f, pad=1)
    expect = np.zeros_like(x)
    expect[0, 0, 1:, :-1] = x[0, 0, :-1, 1:]
    assert np.array_equal(out, expect)


# ---------------------------------------------------------------- P5
def test_linearity_in_input_and_filter_exact_on_integers():
    xa, f, _ = workloads.make_integer_problem(1, 2, 3, 8, 8, 4, 3, 3, with_bias=False)
    xb, g, _ = workloads.make_integer_problem(2, 2, 3, 8, 8, 4, 3, 3, with_bias=False)
    a, b = np.float32(3.0), np.float32(-2.0)
    lhs = oracle.conv_fwd(a * xa + b * xb, f, pad=1)
    rhs = a * oracle.conv_fwd(xa, f, pad=1) + b * oracle.conv_fwd(xb, f, pad=1)
    assert np.array_equal(lhs, rhs)
    lhs = oracle.conv_fwd(xa, a * f + b * g, pad=1, stride=2)
    rhs = a * oracle.conv_fwd(xa, f, pad=1, stride=2) + b * oracle.conv_fwd(xa, g, pad=1, stride=2)
    assert np.array_equal(lhs, rhs)


def test_linearity_float():
    xa, f, _ = workloads.make_random_problem(3, 1, 4, 10, 10, 5, 3, 3, with_bias=False)
    xb, _, _ = workloads.make_random_problem(4, 1, 4, 10, 10, 5, 3, 3, with_bias=False)
    lhs = oracle.conv_fwd(0.5 * xa + 0.25 * xb, f, pad=1)
    rhs = 0.5 * oracle.conv_fwd(xa, f, pad=1) + 0.25 * oracle.conv_fwd(xb, f, pad=1)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-5, atol=1e-6)


# ---------------------------------------------------------------- P7
@pytest.mark.parametrize("H,W,R,S,s,p", [(7, 9, 3, 3, 1, 1), (8, 8, 5, 3, 2, 2), (6, 5, 2, 4, 1, 3),
                                         (13, 13, 3, 3, 1, 1), (11, 11, 11, 11, 4, 0)])
def test_all_ones_closed_form(H, W, R, S, s, p):
    """in == 1, filt == 1: out = C * (#valid rows of the window) * (#valid cols)."""
    C, K = 3, 2
    x = np.ones((1, C, H, W), np.float32)
    f = np.ones((K, C, R, S), np.float32)
    out = oracle.conv_fwd(x, f, stride=s, pad=p)
    P, Q = out.shape[2:]
    rows = np.array([sum(0 <= pp * s - p + r < H for r in range(R)) for pp in range(P)])
    cols = np.array([sum(0 <= qq * s - p + t < W for t in range(S)) for qq in range(Q)])
    expect = (C * rows[:, None] * cols[None, :]).astype(np.float32)
    for k in range(K):
        assert np.array_equal(out[0, k], expect)


def test_window_entirely_in_padding_yields_bias():
    x = np.ones((1, 1, 2, 2), np.float32)
    f = np.ones((1, 1, 2, 2), np.float32)
    b = np.array([0.25], np.float32)
    out = oracle.conv_fwd(x, f, b, stride=1, pad=2)
    assert out[0, 0, 0, 0] == np.float32(0.25)
    assert out[0, 0, 2, 2] == np.float32(4.25)


# ---------------------------------------------------------------- P8
def test_pointwise_equals_library_gemm():
    """Section VI (k1conv): for KSZ=1 per-image im2col is the identity, so the
    layer is filt[KxC] . in_n[CxHW]."""
    x, f, _ = workloads.make_random_problem(21, 3, 37, 7, 5, 19, 1, 1, with_bias=False)
    out = oracle.conv_fwd(x, f)
    fm = f.reshape(19, 37).astype(np.float64)
    for n in range(3):
        ref = (fm @ x[n].reshape(37, 35).astype(np.float64)).astype(np.float32)
        assert np.array_equal(out[n].reshape(19, 35), ref) or \
            np.abs(out[n].reshape(19, 35) - ref).max() <= 1e-7


def test_pointwise_stride2_subsamples():
    x, f, _ = workloads.make_random_problem(22, 1, 4, 8, 8, 3, 1, 1, with_bias=False)
    full = oracle.conv_fwd(x, f)
    sub = oracle.conv_fwd(x, f, stride=2)
    assert np.array_equal(sub, full[:, :, ::2, ::2])


# ---------------------------------------------------------------- P9
def test_batch_independence_bitwise():
    """Section II: results are independent across image pairs."""
    x, f, b = workloads.make_random_problem(31, 4, 3, 9, 9, 5, 3, 3)
    full = oracle.conv_fwd(x, f, b, pad=1, relu=True)
    for n in range(4):
        one = oracle.conv_fwd(x[n:n + 1], f, b, pad=1, relu=True)
        assert np.array_equal(full[n:n + 1], one)


# ---------------------------------------------------------------- P11
def test_relu_is_max_zero():
    x, f, b = workloads.make_random_problem(41, 2, 3, 10, 10, 6, 3, 3)
    lin = oracle.conv_fwd(x, f, b, pad=1, relu=False)
    act = oracle.conv_fwd(x, f, b, pad=1, relu=True)
    assert (lin < 0).any() and (lin > 0).any()
    assert np.array_equal(act, np.maximum(lin, np.float32(0)))


def test_bias_is_per_output_channel_before_relu():
    x, f, _ = workloads.make_integer_problem(42, 1, 2, 6, 6, 3, 3, 3, with_bias=False)
    b = np.array([-100.0, 0.0, 7.0], np.float32)
    lin = oracle.conv_fwd(x, f, None)
    withb = oracle.conv_fwd(x, f, b)
    for k in range(3):
        assert np.array_equal(withb[:, k], lin[:, k] + b[k])
    act = oracle.conv_fwd(x, f, b, relu=True)
    assert np.array_equal(act, np.maximum(withb, 0))
    assert (act[:, 0] == 0).all()      # -100 bias pushes channel 0 below zero before ReLU


# ---------------------------------------------------------------- P12
def test_translation_equivariance():
    x, f, _ = workloads.make_random_problem(51, 1, 2, 12, 12, 3, 3, 3, with_bias=False)
    dy, dx = 2, 3
    shifted = np.zeros_like(x)
    shifted[:, :, dy:, dx:] = x[:, :, :-dy, :-dx]
    a = oracle.conv_fwd(x, f)
    b = oracle.conv_fwd(shifted, f)
    assert np.array_equal(b[:, :, dy:, dx:], a[:, :, :-dy, :-dx])


# ---------------------------------------------------------------- P14
def test_maxpool_bruteforce_and_closed_form():
    x, _, _ = workloads.make_random_problem(61, 2, 3, 13, 15, 1, 1, 1)
    got = oracle.maxpool_fwd(x, 3, 2)
    assert got.shape == (2, 3, 6, 7)
    assert np.array_equal(got, bruteforce.maxpool_separable(x, 3, 2))
    got = oracle.maxpool_fwd(x, 2, 1)
    assert np.array_equal(got, bruteforce.maxpool_separable(x, 2, 1))
    # monotone data: the max of a window is its bottom-right element
    ramp = np.arange(55 * 55, dtype=np.float32).reshape(1, 1, 55, 55)
    got = oracle.maxpool_fwd(ramp, 3, 2)
    assert got.shape == (1, 1, 27, 27)
    assert np.array_equal(got[0, 0], ramp[0, 0, 2::2, 2::2][:27, :27])


def test_maxpool_negative_values():
    x = -np.ones((1, 1, 5, 5), np.float32)
    x[0, 0, 4, 4] = -0.5
    got = oracle.maxpool_fwd(x, 3, 2)
    assert got.reshape(-1).tolist() == [-1.0, -1.0, -1.0, -0.5]


# ---------------------------------------------------------------- oracle on benchmark toy config
def test_toy_config_against_bruteforce():
    x, f, b = workloads.make_layer_inputs(workloads.TOY, 1)
    got = oracle.conv_fwd(x, f, b, stride=1, pad=1, relu=True)
    ref = bruteforce.conv_im2col(x, f, b, stride=1, pad=1, relu=True, loops=False)
    assert got.shape == (1, 16, 32, 32)
    np.testing.assert_allclose(got, ref, rtol=3e-7, atol=1e-7)


# ------------------------------------------------------------------ sgemm (Section V)
def test_sgemm_hand_computed_rectangular():
    """2x3 times 3x2 worked by hand; a transposed operand or swapped index changes it."""
    a = np.array([[1, 2, 3], [4, 5, 6]], np.float32)
    b = np.array([[7, 8], [9, 10], [11, 12]], np.float32)
    assert oracle.sgemm(a, b).tolist() == [[58.0, 64.0], [139.0, 154.0]]


def test_sgemm_python_loops_on_integers():
    rng = np.random.default_rng(3)
    a = rng.integers(-3, 4, (5, 7)).astype(np.float32)
    b = rng.integers(-3, 4, (7, 4)).astype(np.float32)
    want = [[sum(float(a[i, k]) * float(b[k, j]) for k in range(7)) for j in range(4)] for i in range(5)]
    assert oracle.sgemm(a, b).tolist() == want


def test_sgemm_identity_and_library_product():
    rng = np.random.default_rng(4)
    a = rng.standard_normal((33, 65)).astype(np.float32)
    b = rng.standard_normal((65, 47)).astype(np.float32)
    assert np.array_equal(oracle.sgemm(a, np.eye(65, dtype=np.float32)), a)
    assert np.array_equal(oracle.sgemm(np.eye(65, dtype=np.float32), b), b)
    # float64 library product, rounded once: equal up to the double rounding of a 65-term sum
    want = (a.astype(np.float64) @ b.astype(np.float64)).astype(np.float32)
    got = oracle.sgemm(a, b)
    assert np.all(np.abs(got.astype(np.float64) - want) <= 1e-6 * np.maximum(1.0, np.abs(want)))


def test_sgemm_is_the_pointwise_convolution_of_one_image():
    """C = A*B equals the 1x1 convolution with filters A (M x K) on the image B (K channels,
    1 x N pixels): ties the two oracle functions to each other bit for bit."""
    rng = np.random.default_rng(5)
    a = rng.standard_normal((9, 21)).astype(np.float32)
    b = rng.standard_normal((21, 30)).astype(np.float32)
    conv = oracle.conv_fwd(b.reshape(1, 21, 1, 30), a.reshape(9, 21, 1, 1))
    assert np.array_equal(conv.reshape(9, 30), oracle.sgemm(a, b))


# ---- half-precision storage (Section VII: smaller storage types as the next step)

def test_f16_result_is_rounded_once_from_the_exact_sum():
    # exact sum 1 + 2^-11 + 2^-30 lies just above the midpoint of the fp16 neighbours 1 and
    # 1 + 2^-10: one rounding gives the upper one; rounding to fp32 first would drop the
    # 2^-30, land on the midpoint and round to even, i.e. to 1
    x = np.array([1.0, 2.0 ** -11, 2.0 ** -15], dtype=np.float16).reshape(1, 3, 1, 1)
    f = np.array([1.0, 1.0, 2.0 ** -15], dtype=np.float16).reshape(1, 3, 1, 1)
    out = oracle.conv_fwd_f16(x, f)
    assert out.dtype == np.float16 and out.shape == (1, 1, 1, 1)
    assert float(out[0, 0, 0, 0]) == 1.0 + 2.0 ** -10
    assert float(np.float16(oracle.conv_fwd(x, f)[0, 0, 0, 0])) == 1.0


def test_f16_all_ones_closed_form_and_round_to_even():
    # interior value = number of taps; 2049 taps is a tie between 2048 and 2050 -> 2048
    for C, R, expect in [(3, 11, 363.0), (96, 5, 2400.0), (2049, 1, 2048.0), (2051, 1, 2052.0)]:
        x = np.ones((1, C, R + 2, R + 2), dtype=np.float16)
        f = np.ones((2, C, R, R), dtype=np.float16)
        out = oracle.conv_fwd_f16(x, f)
        assert out.shape == (1, 2, 3, 3) and np.all(out.astype(np.float64) == expect)


def test_f16_matches_fp32_function_where_no_rounding_happens():
    rng = np.random.default_rng(5)
    x = rng.integers(-3, 4, size=(2, 5, 9, 8)).astype(np.float16)
    f = rng.integers(-2, 3, size=(4, 5, 3, 3)).astype(np.float16)
    b = rng.integers(-4, 5, size=4).astype(np.float32)
    for relu in (False, True):
        ref = oracle.conv_fwd(x.astype(np.float32), f.astype(np.float32), b, 2, 1, relu)
        assert np.abs(ref).max() < 2048          # integers this small are exact in fp16
        got = oracle.conv_fwd_f16(x, f, b, 2, 1, relu)
        assert np.array_equal(got.astype(np.float32), ref)


def test_f16_bias_joins_the_sum_before_the_rounding_and_relu_after():
    x = np.ones((1, 1, 1, 1), dtype=np.float16)
    f = np.ones((2, 1, 1, 1), dtype=np.float16)
    # 1 + (2^-11 + 2^-31): above the midpoint only if the bias is added before rounding
    b = np.array([np.float32(2.0 ** -11) * np.float32(1 + 2.0 ** -20), -3.0], dtype=np.float32)
    out = oracle.conv_fwd_f16(x, f, b, 1, 0, False).astype(np.float64).ravel()
    assert out[0] == 1.0 + 2.0 ** -10 and out[1] == -2.0
    out = oracle.conv_fwd_f16(x, f, b, 1, 0, True).astype(np.float64).ravel()
    assert out[0] == 1.0 + 2.0 ** -10 and out[1] == 0.0


def test_f16_float_data_against_float64_im2col():
    rng = np.random.default_rng(6)
    x = rng.uniform(0, 1, size=(2, 7, 10, 9)).astype(np.float16)
    f = (rng.standard_normal((5, 7, 3, 3)) * 0.05).astype(np.float16)
    b = rng.uniform(-0.1, 0.1, size=5).astype(np.float32)
    ref = bruteforce.conv_im2col_float64(x.astype(np.float64), f.astype(np.float64),
                                         b.astype(np.float64), 1, 1, True)
    got = oracle.conv_fwd_f16(x, f, b, 1, 1, True)
    assert np.array_equal(got, ref.astype(np.float16))
