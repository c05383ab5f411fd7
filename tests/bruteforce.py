"""Independent brute-force formulations used ONLY to pin the oracle.

The convolution is restated the way the paper's Section III does it: build the
matrix of input slices ``inmat`` explicitly (one row per output point, one
column per window element), reshape the filters to ``filtsmat`` and multiply.
Nothing here is shared with oracle/ or with the HIP library.
"""
import numpy as np


def im2col(inp, R, S, stride, pad):
    """inmat[N*P*Q, R*S*C] in float64; window elements ordered (r, s, c) --
    the Y:X:C order of the paper's example, deliberately not the oracle's."""
    N, C, H, W = inp.shape
    padded = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    padded[:, :, pad:pad + H, pad:pad + W] = inp
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    rows = []
    for n in range(N):
        for p in range(P):
            for q in range(Q):
                win = padded[n, :, p * stride:p * stride + R, q * stride:q * stride + S]
                rows.append(np.transpose(win, (1, 2, 0)).reshape(-1))
    return np.stack(rows), P, Q


def filtsmat(filt):
    """filtsmat[R*S*C, K] in float64 with the same (r, s, c) row order."""
    K = filt.shape[0]
    return np.transpose(filt.astype(np.float64), (2, 3, 1, 0)).reshape(-1, K)


def matmul_loops(a, b):
    """Triple-loop matrix product in Python floats (double)."""
    M, Kd = a.shape
    Nn = b.shape[1]
    out = np.zeros((M, Nn), dtype=np.float64)
    for i in range(M):
        for j in range(Nn):
            acc = 0.0
            for t in range(Kd):
                acc += float(a[i, t]) * float(b[t, j])
            out[i, j] = acc
    return out


def conv_im2col(inp, filt, bias=None, stride=1, pad=0, relu=False, loops=True):
    """out[N,K,P,Q] as fp32 via explicit inmat x filtsmat."""
    N = inp.shape[0]
    K, _, R, S = filt.shape
    a, P, Q = im2col(inp, R, S, stride, pad)
    b = filtsmat(filt)
    om = matmul_loops(a, b) if loops else a @ b
    if bias is not None:
        om = om + bias.astype(np.float64)[None, :]
    out = om.reshape(N, P, Q, K).transpose(0, 3, 1, 2).astype(np.float32)
    if relu:
        out = np.maximum(out, np.float32(0))
    return np.ascontiguousarray(out)


def maxpool_separable(inp, ksz, stride):
    """Row-max then column-max formulation of max pooling."""
    N, C, H, W = inp.shape
    P = (H - ksz) // stride + 1
    Q = (W - ksz) // stride + 1
    rowmax = np.empty((N, C, H, Q), dtype=inp.dtype)
    for q in range(Q):
        rowmax[..., q] = inp[..., q * stride:q * stride + ksz].max(axis=-1)
    out = np.empty((N, C, P, Q), dtype=inp.dtype)
    for p in range(P):
        out[:, :, p, :] = rowmax[:, :, p * stride:p * stride + ksz, :].max(axis=2)
    return out


def conv_im2col_float64(inp, filt, bias=None, stride=1, pad=0, relu=False):
    """out[N,K,P,Q] in float64 via explicit inmat x filtsmat (library product), no
    rounding to a storage type."""
    N = inp.shape[0]
    K, _, R, S = filt.shape
    a, P, Q = im2col(inp, R, S, stride, pad)
    om = a @ filtsmat(filt)
    if bias is not None:
        om = om + np.asarray(bias, dtype=np.float64)[None, :]
    if relu:
        om = np.maximum(om, 0.0)
    return np.ascontiguousarray(om.reshape(N, P, Q, K).transpose(0, 3, 1, 2))
