/*
 * conv_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct CPU statement of what the forward
 * convolution layer computes.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the product library never does and
 * shares no code, header, table or helper with it.
 *
 * What is computed (paper Section II, the definition of the convolution
 * layer): for every output point the window of the input that starts at
 * (oy*stride, ox*stride) and spans all input channels is multiplied element by
 * element with the filter slice of that output channel and summed -- no filter
 * flip (cross-correlation).  The input is padded with zeros (Section II, on
 * padding of the input), images of a batch are independent
 * (Section II, batch dimension B), the activation max(0,x) may be fused
 * (Section II, ReLU).  The per-output-channel bias, which the paper leaves out
 * of its discussion, is added before the activation.
 *
 * Readings taken where the paper is silent:
 *   - output extent = floor((in + 2*pad - ksz)/stride) + 1 (the paper prints
 *     1 + (in - KSZ)/stride with an exactly divisible example only);
 *   - layouts are dense NCHW (activations) and KCRS (filters), fp32;
 *   - the sum is accumulated in double, the bias is added in double and the
 *     result is rounded to fp32 once, so the value is the correctly rounded
 *     exact result whatever the summation order.
 *
 * Loop order is exactly n, k, p, q, c, r, s.  No blocking, no im2col, no
 * reordering.  OpenMP only spreads the independent (n, k) pairs over cores.
 *
 * oracle_sgemm (further down) is the matrix product by its definition, pinned
 * against the float64 library product, the identity and the 1x1 convolution.
 * oracle_conv_fwd_exact leaves the result in double for storage types narrower
 * than fp32 (half precision: rounded once by the caller); pinned by a value whose
 * rounding through fp32 would differ, closed forms and the fp32 function.
 *
 * Pins (tests/test_oracle_*.py): printed worked-example sizes, brute-force
 * im2col x matmul on tiny inputs, delta filter, linearity, exact-integer data,
 * all-ones closed form, 1x1 == library matmul, batch independence,
 * translation equivariance, ReLU identity.  Every function here has a pin.
 */
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Section II output-size formula, floor reading.  Returns 0 on success,
 * -1 if the arguments do not describe a convolution with >= 1 output point. */
int oracle_conv_out_dims(int H, int W, int R, int S, int stride, int pad,
                         int *P, int *Q)
{
    if (H <= 0 || W <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return -1;
    if (H + 2 * pad < R || W + 2 * pad < S)
        return -1;
    *P = (H + 2 * pad - R) / stride + 1;
    *Q = (W + 2 * pad - S) / stride + 1;
    return 0;
}

/* Section II convolution + bias + optional ReLU.  in: N*C*H*W, filt: K*C*R*S,
 * bias: K or NULL, out: N*K*P*Q.  Returns 0 or -1 (bad arguments). */
int oracle_conv_fwd(const float *in, const float *filt, const float *bias,
                    float *out, int N, int C, int H, int W, int K, int R,
                    int S, int stride, int pad, int relu)
{
    int P, Q;
    if (!in || !filt || !out || N <= 0 || C <= 0 || K <= 0)
        return -1;
    if (oracle_conv_out_dims(H, W, R, S, stride, pad, &P, &Q) != 0)
        return -1;

#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c) {
                        for (int r = 0; r < R; ++r) {
                            for (int s = 0; s < S; ++s) {
                                int y = p * stride - pad + r;
                                int x = q * stride - pad + s;
                                if (y < 0 || y >= H || x < 0 || x >= W)
                                    continue; /* zero padding */
                                size_t ii = (((size_t)n * C + c) * H + y) * W + x;
                                size_t fi = (((size_t)k * C + c) * R + r) * S + s;
                                acc += (double)in[ii] * (double)filt[fi];
                            }
                        }
                    }
                    if (bias)
                        acc += (double)bias[k];
                    float v = (float)acc;
                    if (relu && !(v > 0.0f))
                        v = 0.0f;
                    out[(((size_t)n * K + k) * P + p) * Q + q] = v;
                }
            }
        }
    }
    return 0;
}

/* The same layer with the result left in double: the exact sum (to double
 * rounding), bias added, ReLU applied, no rounding to a storage type.  Used for
 * half-precision storage (the paper's Section VII outlook: fp16 storage for
 * bandwidth-limited cases, arithmetic in fp32): the caller passes the fp16
 * tensors widened to fp32 (exact) and rounds this result to fp16 once, so the
 * expected value is the correctly rounded exact result.  Same loop order. */
int oracle_conv_fwd_exact(const float *in, const float *filt, const float *bias,
                          double *out, int N, int C, int H, int W, int K, int R,
                          int S, int stride, int pad, int relu)
{
    int P, Q;
    if (!in || !filt || !out || N <= 0 || C <= 0 || K <= 0)
        return -1;
    if (oracle_conv_out_dims(H, W, R, S, stride, pad, &P, &Q) != 0)
        return -1;

#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c) {
                        for (int r = 0; r < R; ++r) {
                            for (int s = 0; s < S; ++s) {
                                int y = p * stride - pad + r;
                                int x = q * stride - pad + s;
                                if (y < 0 || y >= H || x < 0 || x >= W)
                                    continue; /* zero padding */
                                size_t ii = (((size_t)n * C + c) * H + y) * W + x;
                                size_t fi = (((size_t)k * C + c) * R + r) * S + s;
                                acc += (double)in[ii] * (double)filt[fi];
                            }
                        }
                    }
                    if (bias)
                        acc += (double)bias[k];
                    if (relu && !(acc > 0.0))
                        acc = 0.0;
                    out[(((size_t)n * K + k) * P + p) * Q + q] = acc;
                }
            }
        }
    }
    return 0;
}

/* Max-pooling, named in Section II among the operations of a deployed network; textbook
 * definition: window ksz x ksz, step `stride`, no padding, floor extents.
 * in: N*C*H*W, out: N*C*P*Q with P = floor((H-ksz)/stride)+1. */
int oracle_maxpool_fwd(const float *in, float *out, int N, int C, int H, int W,
                       int ksz, int stride)
{
    if (!in || !out || N <= 0 || C <= 0 || H < ksz || W < ksz || ksz <= 0 ||
        stride <= 0)
        return -1;
    int P = (H - ksz) / stride + 1;
    int Q = (W - ksz) / stride + 1;
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < N * C; ++nc) {
        const float *src = in + (size_t)nc * H * W;
        float *dst = out + (size_t)nc * P * Q;
        for (int p = 0; p < P; ++p) {
            for (int q = 0; q < Q; ++q) {
                float m = src[(size_t)(p * stride) * W + q * stride];
                for (int r = 0; r < ksz; ++r)
                    for (int s = 0; s < ksz; ++s) {
                        float v = src[(size_t)(p * stride + r) * W + q * stride + s];
                        if (v > m)
                            m = v;
                    }
                dst[(size_t)p * Q + q] = m;
            }
        }
    }
    return 0;
}

/* Matrix product by its definition (the SGEMM of Section V, row-major
 * operands): c[i][j] = sum_k a[i][k] * b[k][j], loops i, j, k in that order,
 * accumulated in double and rounded to fp32 once.  a: M*K, b: K*N, c: M*N. */
int oracle_sgemm(const float *a, const float *b, float *c, int M, int N, int K)
{
    if (!a || !b || !c || M <= 0 || N <= 0 || K <= 0)
        return -1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        for (int j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += (double)a[(size_t)i * K + k] * (double)b[(size_t)k * N + j];
            c[(size_t)i * N + j] = (float)acc;
        }
    }
    return 0;
}

/* Number of worker threads the parallel loops above will use. */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
