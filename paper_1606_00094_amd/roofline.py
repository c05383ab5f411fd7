"""Work accounting for the roofline report (no convolution arithmetic here).

FLOPs count two per multiply-accumulate, the convention of the paper's SGEMM
tables (Tables I-II: 128^3 -> 4.19 MF) and of its Section V formula
AI = 2MNK / (4(MN+MK+KN)).  The worked example of Section III counts one per
MAC (141 M for 10K x 96 x 147); ``flops_per_mac`` selects that reading.
"""

# MI355X published peaks used as roofline denominators.
PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_FP16_MFMA_TFLOPS = 2500.0   # dense fp16 matrix peak (half-precision entry points)
PEAK_HBM_GBPS = 8000.0


def conv_out_dims(H, W, R, S, stride, pad):
    """Output extent: the library's own answer (conv_out_dims of the C ABI, host only), so
    that the accounting can never disagree with what the kernels compute."""
    from . import binding
    return binding.conv_out_dims(H, W, R, S, stride, pad)


def conv_flops(N, C, H, W, K, R, S, stride, pad, flops_per_mac=2):
    """Algorithmic FLOPs of one forward convolution (padded taps counted)."""
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    return flops_per_mac * N * K * P * Q * C * R * S


def conv_bytes(N, C, H, W, K, R, S, stride, pad, with_bias=True):
    """Algorithmic bytes: each tensor crosses HBM once (fp32)."""
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    return 4 * (N * C * H * W + K * C * R * S + (K if with_bias else 0) + N * K * P * Q)


def im2col_gemm_bytes(N, C, H, W, K, R, S, stride, pad):
    """Bytes of the explicit-matrix form of Section III (the arithmetic-intensity
    figure): outmat + inmat + filtsmat, fp32.  Returns the three terms."""
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    rows, cols = N * P * Q, C * R * S
    return 4 * rows * K, 4 * rows * cols, 4 * cols * K


def sgemm_flops(M, N, K):
    return 2 * M * N * K


def sgemm_bytes(M, N, K):
    return 4 * (M * N + M * K + K * N)


def sgemm_ai(M, N, K):
    """Section V: AI = 2MNK / (4(MN+MK+KN))."""
    return sgemm_flops(M, N, K) / sgemm_bytes(M, N, K)


def roof_min_seconds(flops, nbytes):
    """(mfma_bound_s, hbm_bound_s) at the published peaks."""
    return flops / (PEAK_FP32_MFMA_TFLOPS * 1e12), nbytes / (PEAK_HBM_GBPS * 1e9)
