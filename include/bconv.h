/*
 * bconv.h -- C ABI of the MI355X (gfx950) forward convolution library.
 *
 * The operation is the convolution layer of the paper's Section II:
 *   out[n,k,p,q] = act( bias[k] + sum_{c,r,s} in[n,c,p*stride-pad+r,q*stride-pad+s]
 *                                             * filt[k,c,r,s] )
 * i.e. for every output point the window of the input starting at
 * (p*stride, q*stride) (in zero-padded coordinates) over all input channels is
 * multiplied element-wise with filter k and summed, with no filter flip; images
 * of a batch are independent; act is the identity or ReLU max(0,x), applied
 * in the same kernel (Section II notes that the activation is commonly fused).  The
 * per-output-channel bias, which the paper leaves out of its discussion, is
 * added before the activation.  Output extent (Section II size rule, floor
 * reading):  P = floor((H + 2*pad - R)/stride) + 1, same for Q with W, S.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library
 *     reads in/filt/bias and writes out, and never frees or keeps them.
 *   - Layouts are dense row-major fp32: in N*C*H*W, filt K*C*R*S, bias K (or
 *     NULL = no bias), out N*K*P*Q.  out must not overlap any input.
 *     4-byte alignment is enough.
 *   - Calls only enqueue work on a HIP stream and return; they never
 *     synchronise it.  `hip_stream` is a hipStream_t passed as void* (NULL = the
 *     null stream).
 *   - Host threads: every entry point may be called from several threads at once.
 *     Calls that share a workspace, or write the same tensor, must be ordered by
 *     the caller (one stream, or events); conv_fwd / conv_fwd_f16 / sgemm share the
 *     library's workspace and order themselves on the null stream.
 *   - Return value: BCONV_OK (0) or a negative bconv_status; on error nothing
 *     has been launched.  No C++ exception crosses the boundary.
 *   - Tensor sizes: up to 2^40 elements each.  One launch of a tiled kernel addresses
 *     at most 2 GiB of input and 2^31 output elements; a larger batch is computed
 *     as consecutive launches over runs of whole images (the images of a batch are
 *     independent, Section II), all inside the one call and on its stream.  The
 *     variant queries below then describe the launch over a full run, and a forced
 *     variant must be able to run every run.  A single image beyond those limits
 *     goes to the direct kernel (64-bit indexing).
 *   - One scalar stride and one scalar pad apply to both axes (Section II:
 *     kernel size and stride taken as scalars); R and S are independent.
 *     No groups, no dilation.
 */
#ifndef BCONV_H
#define BCONV_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BCONV_OK = 0,
  BCONV_EINVAL = -1,     /* non-positive dimension, stride <= 0, pad < 0, relu not 0/1 */
  BCONV_ENULL = -2,      /* a required pointer is NULL */
  BCONV_ESHAPE = -3,     /* no output point: H + 2*pad < R or W + 2*pad < S, or tensor too large */
  BCONV_EWORKSPACE = -4, /* workspace missing or smaller than conv_fwd_workspace_bytes() */
  BCONV_ELAUNCH = -5,    /* the HIP runtime refused an allocation or a launch */
  BCONV_EVARIANT = -6    /* variant id out of range or not applicable to this shape */
} bconv_status;

/* Section II output-size rule.  Host only.  Writes *P, *Q. */
int conv_out_dims(int H, int W, int R, int S, int stride, int pad, int* P, int* Q);

/* Forward convolution + bias + optional ReLU on the null stream, variant chosen
 * by the selection table (the role of the paper's per-operation variant and
 * blocking choice: Section V on choosing the blocking, Section VI on the variants).
 * If the chosen variant splits the reduction, partial sums go to a workspace
 * the library allocates once per device and keeps until the process ends. */
int conv_fwd(const float* in, const float* filt, const float* bias, float* out,
             int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
             int relu);

/* Same operation with explicit stream, workspace and variant.
 *   workspace / workspace_bytes: device scratch of at least
 *     conv_fwd_workspace_bytes(..., variant_id) bytes, 256-byte aligned; may be
 *     NULL/0 when that function returns 0.  Contents before and after are
 *     unspecified.  Two calls that share a workspace must be ordered on one stream.
 *   variant_id: -1 = selection table; 0 .. conv_num_variants()-1 = forced
 *     (tests, tuning sweeps); a variant that cannot run the shape gives
 *     BCONV_EVARIANT. */
int conv_fwd_ex(const float* in, const float* filt, const float* bias, float* out,
                int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                int relu, void* workspace, size_t workspace_bytes, void* hip_stream,
                int variant_id);

/* conv_fwd_ex for callers that cannot allocate device memory or let a library do so: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operation, same selection-table choice (variant_id = -1), same results bit for bit as
 * conv_fwd_ex with that variant; the partial sums of a split reduction go to a fixed array of
 * BCONV_NOALLOC_MAX_WORKSPACE_BYTES = 32 MiB of device memory that is part of the
 * library's code object (every GPU the library runs on holds one until the process ends).
 * The call allocates and frees nothing, on the device or through any library.  A shape whose
 * chosen variant needs more partial-sum space than the array holds
 * (conv_fwd_workspace_bytes(..., -1) > the maximum) gives BCONV_EWORKSPACE and launches
 * nothing.  All calls on one GPU share that GPU's array: nothing in it has to start at zero
 * (every partial sum that is read was written by the same call), but two calls that overlap
 * in time on one GPU -- different streams, or host threads without ordering -- race on it;
 * order them on one stream or with events.  Other errors as conv_fwd_ex. */
#define BCONV_NOALLOC_MAX_WORKSPACE_BYTES ((size_t)32 << 20)
int conv_fwd_noalloc(const float* in, const float* filt, const float* bias, float* out,
                     int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                     int relu, void* hip_stream);

/* The same layer with half-precision storage (Section VII names smaller storage
 * types, half floats, as the next step for bandwidth-limited cases; the arithmetic
 * stays fp32).  in, filt and out are DEVICE pointers to dense IEEE binary16 tensors
 * (same NCHW / KCRS layouts, 2-byte alignment is enough); bias stays fp32 (or NULL).
 * Elements are widened exactly, products and sums are fp32 on the matrix cores, bias
 * and ReLU are applied in fp32 and the result is rounded to binary16 once, to nearest
 * even.  Variant ids and all error codes are those of conv_fwd / conv_fwd_ex; the workspace
 * size comes from conv_fwd_f16_workspace_bytes (below); a pointer that is not
 * 2-byte aligned gives BCONV_EINVAL.  A variant with 4-element loads needs 8-byte
 * aligned in / filt here; the table's choice degrades silently to its narrow twin,
 * a forced one gives BCONV_EVARIANT. */
int conv_fwd_f16(const void* in, const void* filt, const float* bias, void* out,
                 int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                 int relu);
int conv_fwd_f16_ex(const void* in, const void* filt, const float* bias, void* out,
                    int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                    int relu, void* workspace, size_t workspace_bytes, void* hip_stream,
                    int variant_id);

/* Queries for the half-precision entry points.  Their catalogue is that of the fp32 entry
 * points (the same tiles with fp32 arithmetic, widening the elements on the way into LDS; the
 * vector-FMA first-layer kernels excepted) plus the tiles that multiply on the fp16 matrix
 * cores (names h16...: exact fp16 x fp16 products, fp32 sums, so the same numerical contract;
 * stride 1, kernels 1x1 / 3x3 / 5x5, C a multiple of eight).  Those need device scratch for the
 * filters re-laid into their reduction order, every call, and are what variant_id = -1 picks
 * for launches large enough to fill the chip; conv_fwd_ex gives BCONV_EVARIANT for them.
 *   conv_fwd_f16_selected_variant: the variant conv_fwd_f16 / conv_fwd_f16_ex(-1) would run.
 *   conv_fwd_f16_variant_applicable: 1 / 0, negative status on bad arguments.
 *   conv_fwd_f16_workspace_bytes: what conv_fwd_f16_ex needs for (shape, variant_id); for -1
 *     it covers the choice for any pointer alignment. */
int conv_fwd_f16_selected_variant(int N, int C, int H, int W, int K, int R, int S, int stride,
                                  int pad);
int conv_fwd_f16_variant_applicable(int N, int C, int H, int W, int K, int R, int S, int stride,
                                    int pad, int variant_id);
size_t conv_fwd_f16_workspace_bytes(int N, int C, int H, int W, int K, int R, int S, int stride,
                                    int pad, int variant_id);

/* Filter pre-packing for the fp16-matrix-core tiles.  The weights of a deployed network are
 * constant (the paper's Section VI folds a layout transformation into a pre-pass for the same
 * reason); those tiles need the filters re-laid from KCRS into their reduction order, which
 * conv_fwd_f16_ex does on every call.  Here the caller does it once:
 *   conv_f16_packed_filter_bytes: bytes of the packed copy for (shape, variant_id); 0 when the
 *     variant (for -1: conv_fwd_f16_selected_variant's choice) is not such a tile or the batch
 *     needs more than one launch -- then there is nothing to pack, use conv_fwd_f16_ex.
 *   conv_f16_pack_filters: filt (device, fp16 KCRS) -> packed (device, 16-byte aligned, at least
 *     that many bytes), enqueued on hip_stream.
 *   conv_fwd_f16_packed_ex: conv_fwd_f16_ex on a packed copy made for the SAME shape and
 *     variant_id (the layout depends on the tile; a copy made for another tile gives wrong
 *     results without an error); no workspace argument; bit for bit the result of
 *     conv_fwd_f16_ex with that variant.  A variant that splits the reduction (name .../sN,
 *     N > 1: what small batches get) keeps its partial sums in the library's own per-device
 *     buffer, as conv_fwd does: grown on first need, shared by the calls on that GPU, which
 *     must therefore not overlap in time.
 * Errors as conv_fwd_f16_ex; BCONV_EVARIANT where conv_f16_packed_filter_bytes returns 0. */
size_t conv_f16_packed_filter_bytes(int N, int C, int H, int W, int K, int R, int S, int stride,
                                    int pad, int variant_id);
int conv_f16_pack_filters(const void* filt, void* packed, size_t packed_bytes, int N, int C, int H,
                          int W, int K, int R, int S, int stride, int pad, void* hip_stream,
                          int variant_id);
int conv_fwd_f16_packed_ex(const void* in, const void* packed, const float* bias, void* out,
                           int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           int relu, void* hip_stream, int variant_id);

/* Activation layouts of the half-precision matrix-core path.  The paper's Section VI applies a
 * transformation to the input of its pointwise and tiled variants so that global memory is read
 * in a good pattern.  Here the input is NCHW or C8 = [N][C/8][H][W][8] -- the
 * eight consecutive channels 8j .. 8j+7 of a pixel in 16 contiguous bytes, channel count a
 * multiple of eight, the buffer 16-byte aligned.  C8 is what the fp16-matrix-core tiles stage
 * and store best (one 16-byte load per eight channels of a position, 8-byte stores), so a chain
 * of half-precision layers keeps its activations in it and converts at the ends.
 *   f16_layout_convert: fp16 activations of N x C x H x W elements from in_layout to out_layout
 *     (device pointers, distinct buffers, enqueued on hip_stream); BCONV_EINVAL unless the two
 *     layouts differ and C % 8 == 0.
 *   conv_fwd_f16_packed_layout_ex: conv_fwd_f16_packed_ex with the input in in_layout and the
 *     output (N x K x P x Q) written in out_layout.  C8 output needs C8 input and K % 8 == 0
 *     (else BCONV_EINVAL).  With both NCHW it is conv_fwd_f16_packed_ex; with C8 the result is
 *     the same set of values, element (n, k, p, q) found at its C8 position.
 *   conv_fwd_f16_c8_selected_variant: the measured (else estimated) best fp16-matrix-core tile
 *     for this shape on C8 activations, to be passed as variant_id to the packing calls and to
 *     conv_fwd_f16_packed_layout_ex (their -1 means the choice for NCHW activations, which can
 *     be a different tile, or none for a small launch); BCONV_EVARIANT when no such tile
 *     applies (stride > 1, a kernel other than 1x1 / 3x3 / 5x5, C not a multiple of eight). */
#define BCONV_LAYOUT_NCHW 0
#define BCONV_LAYOUT_C8 1
int conv_fwd_f16_c8_selected_variant(int N, int C, int H, int W, int K, int R, int S, int stride,
                                     int pad);
int f16_layout_convert(const void* in, int in_layout, void* out, int out_layout, int N, int C,
                       int H, int W, void* hip_stream);
/* conv_fwd_f16_ex with the layouts named per tensor: filters unpacked (re-laid per call into
 * the workspace, conv_fwd_f16_workspace_bytes(shape, variant_id) bytes, 16-byte aligned).  With
 * both layouts NCHW it is conv_fwd_f16_ex.  Otherwise the variant must be an fp16-matrix-core
 * tile (BCONV_EVARIANT if not): C8 input goes to the channel-octet tiles (-1 = the choice of
 * conv_fwd_f16_c8_selected_variant), NCHW input with C8 output to the first-layer tiles
 * (C <= 3, 11x11 step 4 or 7x7 step 2: how a chain enters the C8 layout without a conversion
 * pass; -1 = conv_fwd_f16_selected_variant's choice, which must be such a tile). */
int conv_fwd_f16_layout_ex(const void* in, int in_layout, const void* filt, const float* bias,
                           void* out, int out_layout, int N, int C, int H, int W, int K, int R,
                           int S, int stride, int pad, int relu, void* workspace,
                           size_t workspace_bytes, void* hip_stream, int variant_id);
int conv_fwd_f16_packed_layout_ex(const void* in, int in_layout, const void* packed,
                                  const float* bias, void* out, int out_layout, int N, int C,
                                  int H, int W, int K, int R, int S, int stride, int pad, int relu,
                                  void* hip_stream, int variant_id);

/* Bytes of workspace conv_fwd_ex needs for this shape and variant (0 if none;
 * also 0 for arguments conv_fwd_ex would reject).  For variant_id = -1 the figure
 * covers the table's choice for any pointer alignment (wide loads or their narrow
 * twins). */
size_t conv_fwd_workspace_bytes(int N, int C, int H, int W, int K, int R, int S,
                                int stride, int pad, int variant_id);

/* Single-precision matrix multiply C = A * B on row-major matrices, A M x K,
 * B K x N, C M x N (the SGEMM of the paper's Section V and Tables I-II, M = N = K
 * from 128 to 2048 there).  It runs the pointwise path: rows of A are the filters,
 * columns of B the pixels of one image, K the channels; the variant ids, the
 * workspace rule and the error codes are those of conv_fwd_ex for the shape
 * (N=1, C=K, H=1, W=N, K=M, 1x1, stride 1, pad 0).  No bias, no activation.
 * sgemm uses the null stream and the library's own workspace, like conv_fwd. */
int sgemm(const float* A, const float* B, float* C, int M, int N, int K);
int sgemm_ex(const float* A, const float* B, float* C, int M, int N, int K, void* workspace,
             size_t workspace_bytes, void* hip_stream, int variant_id);
size_t sgemm_workspace_bytes(int M, int N, int K, int variant_id);

/* Variant catalogue.  A variant is a kernel family + tile shape + reduction
 * split; the ids are stable within one build of the library. */
int conv_num_variants(void);
/* Writes a NUL-terminated name into buf (truncated to buflen). */
int conv_variant_name(int variant_id, char* buf, size_t buflen);
/* The variant conv_fwd would run for this shape, or a negative status. */
int conv_selected_variant(int N, int C, int H, int W, int K, int R, int S, int stride,
                          int pad);
/* 1 if the variant can run the shape, 0 if not, negative status on bad arguments. */
int conv_variant_applicable(int N, int C, int H, int W, int K, int R, int S, int stride,
                            int pad, int variant_id);

/* Host-only diagnostic: walks every workgroup, thread and reduction chunk of the
 * launch that (shape, variant) would produce, using the same index functions as
 * the device code, and counts LDS or global accesses that would fall outside
 * their buffers.  Returns that count (0 = clean) or a negative status.  Touches
 * no GPU. */
long long bconv_debug_audit(int N, int C, int H, int W, int K, int R, int S, int stride,
                            int pad, int variant_id);

/* Host-only diagnostic: the time estimate (arbitrary units, lower is better) that
 * the selection heuristic gives (shape, variant) when the shape is not in the
 * table; negative if the variant cannot run the shape.  Lets a tuning sweep
 * compare the heuristic's ranking with measured times. */
double bconv_debug_model_cost(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                              int variant_id);

/* Convolution + bias + optional ReLU followed by max pooling (window pool_ksz, step
 * pool_stride, no padding, floor extents) in one call: the next operation of the
 * chain in the networks the paper draws its layers from (Section II lists pooling
 * among the operations of a deployed network).  out is the POOLED tensor N*K*PP*PQ with
 * PP = floor((P-pool_ksz)/pool_stride)+1; the unpooled result is never written to
 * `out`.  When the variant splits the reduction the pooling is folded into the
 * reduction kernel (two kernels in all instead of three); otherwise the convolution
 * writes to the workspace and a pooling kernel follows.  Values are those of
 * conv_fwd_ex with the same variant followed by maxpool_fwd, bit for bit (with
 * variant_id = -1 the two entry points may pick different variants, whose sums differ
 * in rounding order).
 *   workspace: at least conv_pool_fwd_workspace_bytes(...) bytes, 256-byte aligned,
 *     always needed (with variant_id = -1 the query covers any window and alignment).
 *     variant_id as for conv_fwd_ex; -1 = conv_pool_selected_variant's choice.
 * Errors as conv_fwd_ex, plus BCONV_EINVAL for a non-positive window or step and
 * BCONV_ESHAPE when the window is larger than the convolution's output. */
int conv_pool_fwd_ex(const float* in, const float* filt, const float* bias, float* out,
                     int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                     int relu, int pool_ksz, int pool_stride, void* workspace,
                     size_t workspace_bytes, void* hip_stream, int variant_id);
size_t conv_pool_fwd_workspace_bytes(int N, int C, int H, int W, int K, int R, int S,
                                     int stride, int pad, int variant_id);
/* The variant conv_pool_fwd_ex runs with variant_id = -1 and suitably aligned pointers:
 * its own measured choice where one is listed for this shape and a 3x3 / step-2 window
 * (per-operation variant choice, Section VI), else conv_selected_variant's.  Negative
 * status on an invalid shape or window. */
int conv_pool_selected_variant(int N, int C, int H, int W, int K, int R, int S, int stride,
                               int pad, int pool_ksz, int pool_stride);

/* Measurement aid: launches `workgroups` workgroups of 256 threads that each issue
 * iters * 16 fp32 32x32x2 MFMAs per wave from registers only (iters * 16 * 4096 flops per
 * wave, four waves per workgroup) and write one float per thread to `out`
 * (workgroups * 256 floats, device memory).  Timing it gives the rate the matrix
 * pipes sustain on the machine at hand, to put beside the published peak. */
int bconv_debug_mfma_loop(float* out, int workgroups, int iters, void* hip_stream);

/* Max pooling over ksz x ksz windows stepped by `stride`, no padding, floor
 * extents (the pooling operation the paper names in Section II among the
 * operations of a deployed network; used to chain the five-layer stack).
 * in N*C*H*W -> out N*C*P*Q with P = floor((H-ksz)/stride)+1. */
int maxpool_fwd(const float* in, float* out, int N, int C, int H, int W, int ksz,
                int stride, void* hip_stream);

/* maxpool_fwd for fp16 activations in `layout` (BCONV_LAYOUT_NCHW, or BCONV_LAYOUT_C8 with
 * C % 8 == 0 and 16-byte aligned buffers), output in the same layout: what a chain of
 * half-precision layers pools with between convolutions.  A maximum is one of its inputs:
 * no rounding. */
int maxpool_fwd_f16(const void* in, void* out, int layout, int N, int C, int H, int W, int ksz,
                    int stride, void* hip_stream);

/* Static, human-readable text for a status code. */
const char* bconv_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* BCONV_H */
