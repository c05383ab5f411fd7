"""Thin ctypes binding of libbconv's C ABI (see include/bconv.h).

Argument marshalling only: tensors must already be contiguous fp32 on the GPU;
every step of the computation runs in the library's HIP kernels.  There is no
CPU fallback: if libbconv.so is missing or a call fails, an exception is raised.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbconv.so")
_lib = None

_vp = ctypes.c_void_p
_i = ctypes.c_int
_sz = ctypes.c_size_t

EXPORTS = {
    "conv_out_dims": ([_i] * 6 + [ctypes.POINTER(_i)] * 2, _i),
    "conv_fwd": ([_vp] * 4 + [_i] * 10, _i),
    "conv_fwd_ex": ([_vp] * 4 + [_i] * 10 + [_vp, _sz, _vp, _i], _i),
    "conv_fwd_noalloc": ([_vp] * 4 + [_i] * 10 + [_vp], _i),
    "conv_fwd_f16": ([_vp] * 4 + [_i] * 10, _i),
    "conv_fwd_f16_ex": ([_vp] * 4 + [_i] * 10 + [_vp, _sz, _vp, _i], _i),
    "conv_fwd_workspace_bytes": ([_i] * 10, _sz),
    "conv_fwd_f16_selected_variant": ([_i] * 9, _i),
    "conv_fwd_f16_variant_applicable": ([_i] * 10, _i),
    "conv_fwd_f16_workspace_bytes": ([_i] * 10, _sz),
    "conv_f16_packed_filter_bytes": ([_i] * 10, _sz),
    "conv_f16_pack_filters": ([_vp, _vp, _sz] + [_i] * 9 + [_vp, _i], _i),
    "conv_fwd_f16_packed_ex": ([_vp] * 4 + [_i] * 10 + [_vp, _i], _i),
    "conv_fwd_f16_packed_layout_ex": ([_vp, _i, _vp, _vp, _vp, _i] + [_i] * 10 + [_vp, _i], _i),
    "conv_fwd_f16_layout_ex": ([_vp, _i, _vp, _vp, _vp, _i] + [_i] * 10 + [_vp, _sz, _vp, _i], _i),
    "f16_layout_convert": ([_vp, _i, _vp, _i] + [_i] * 4 + [_vp], _i),
    "conv_fwd_f16_c8_selected_variant": ([_i] * 9, _i),
    "conv_pool_fwd_ex": ([_vp] * 4 + [_i] * 12 + [_vp, _sz, _vp, _i], _i),
    "conv_pool_fwd_workspace_bytes": ([_i] * 10, _sz),
    "conv_pool_selected_variant": ([_i] * 11, _i),
    "sgemm": ([_vp] * 3 + [_i] * 3, _i),
    "sgemm_ex": ([_vp] * 3 + [_i] * 3 + [_vp, _sz, _vp, _i], _i),
    "sgemm_workspace_bytes": ([_i] * 4, _sz),
    "conv_num_variants": ([], _i),
    "conv_variant_name": ([_i, ctypes.c_char_p, _sz], _i),
    "conv_selected_variant": ([_i] * 9, _i),
    "conv_variant_applicable": ([_i] * 10, _i),
    "bconv_debug_audit": ([_i] * 10, ctypes.c_longlong),
    "bconv_debug_model_cost": ([_i] * 10, ctypes.c_double),
    "bconv_debug_mfma_loop": ([_vp, _i, _i, _vp], _i),
    "maxpool_fwd": ([_vp] * 2 + [_i] * 6 + [_vp], _i),
    "maxpool_fwd_f16": ([_vp, _vp] + [_i] * 7 + [_vp], _i),
    "bconv_strerror": ([_i], ctypes.c_char_p),
}


class BconvError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, strerror(status)))


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        # torch ships its own HIP runtime; it must be in the process first so that
        # libbconv binds to that same runtime (two runtimes in one process do not
        # share devices, streams or allocations).
        import torch  # noqa: F401
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libbconv.so not built: run `python -m paper_1606_00094_amd.build` "
                               "(there is no CPU fallback)")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (argtypes, restype) in EXPORTS.items():
            fn = getattr(handle, name)
            fn.argtypes = argtypes
            fn.restype = restype
        _lib = handle
    return _lib


def strerror(status):
    return lib().bconv_strerror(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise BconvError(status, where)


def _dev_ptr(t, name, half=False):
    import torch
    if t is None:
        return None
    want = torch.float16 if half else torch.float32
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == want and t.is_contiguous()):
        raise TypeError("%s must be a contiguous %s tensor on the GPU"
                        % (name, "float16" if half else "float32"))
    return t.data_ptr()


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def conv_out_dims(H, W, R, S, stride, pad):
    P, Q = _i(0), _i(0)
    _check(lib().conv_out_dims(H, W, R, S, stride, pad, ctypes.byref(P), ctypes.byref(Q)),
           "conv_out_dims")
    return P.value, Q.value


def _dims(inp, filt):
    N, C, H, W = inp.shape
    K, C2, R, S = filt.shape
    if C != C2:
        raise ValueError("in has %d channels, filt expects %d" % (C, C2))
    return N, C, H, W, K, R, S


def conv_fwd_ex(inp, filt, bias, out, stride, pad, relu, workspace=None, stream=None, variant=-1):
    """conv_fwd_ex of the C ABI on torch tensors; enqueues on `stream` (default: torch's
    current stream) and returns `out`."""
    N, C, H, W, K, R, S = _dims(inp, filt)
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    if tuple(out.shape) != (N, K, P, Q):
        raise ValueError("out must have shape %s" % ((N, K, P, Q),))
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(lib().conv_fwd_ex(_dev_ptr(inp, "in"), _dev_ptr(filt, "filt"), _dev_ptr(bias, "bias"),
                             _dev_ptr(out, "out"), N, C, H, W, K, R, S, stride, pad,
                             1 if relu else 0, ws_ptr, ws_bytes, _stream_handle(stream),
                             int(variant)), "conv_fwd_ex")
    return out


def conv_fwd(inp, filt, bias, out, stride, pad, relu):
    """conv_fwd of the C ABI (null stream, selection table, internal workspace)."""
    N, C, H, W, K, R, S = _dims(inp, filt)
    _check(lib().conv_fwd(_dev_ptr(inp, "in"), _dev_ptr(filt, "filt"), _dev_ptr(bias, "bias"),
                          _dev_ptr(out, "out"), N, C, H, W, K, R, S, stride, pad,
                          1 if relu else 0), "conv_fwd")
    return out


def conv_fwd_noalloc(inp, filt, bias, out, stride, pad, relu, stream=None):
    """conv_fwd_noalloc of the C ABI (selection table, partial sums in the library's static
    device array, no allocation); enqueues on `stream` (default: torch's current stream)."""
    N, C, H, W, K, R, S = _dims(inp, filt)
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    if tuple(out.shape) != (N, K, P, Q):
        raise ValueError("out must have shape %s" % ((N, K, P, Q),))
    _check(lib().conv_fwd_noalloc(_dev_ptr(inp, "in"), _dev_ptr(filt, "filt"), _dev_ptr(bias, "bias"),
                                  _dev_ptr(out, "out"), N, C, H, W, K, R, S, stride, pad,
                                  1 if relu else 0, _stream_handle(stream)), "conv_fwd_noalloc")
    return out


NOALLOC_MAX_WORKSPACE_BYTES = 32 << 20   # BCONV_NOALLOC_MAX_WORKSPACE_BYTES of include/bconv.h


def conv_fwd_f16_ex(inp, filt, bias, out, stride, pad, relu, workspace=None, stream=None,
                    variant=-1):
    """conv_fwd_f16_ex of the C ABI: float16 in / filt / out, float32 bias."""
    N, C, H, W, K, R, S = _dims(inp, filt)
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    if tuple(out.shape) != (N, K, P, Q):
        raise ValueError("out must have shape %s" % ((N, K, P, Q),))
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(lib().conv_fwd_f16_ex(_dev_ptr(inp, "in", True), _dev_ptr(filt, "filt", True),
                                 _dev_ptr(bias, "bias"), _dev_ptr(out, "out", True), N, C, H, W, K,
                                 R, S, stride, pad, 1 if relu else 0, ws_ptr, ws_bytes,
                                 _stream_handle(stream), int(variant)), "conv_fwd_f16_ex")
    return out


def conv_fwd_f16(inp, filt, bias, out, stride, pad, relu):
    """conv_fwd_f16 of the C ABI (null stream, selection table, internal workspace)."""
    N, C, H, W, K, R, S = _dims(inp, filt)
    _check(lib().conv_fwd_f16(_dev_ptr(inp, "in", True), _dev_ptr(filt, "filt", True),
                              _dev_ptr(bias, "bias"), _dev_ptr(out, "out", True), N, C, H, W, K,
                              R, S, stride, pad, 1 if relu else 0), "conv_fwd_f16")
    return out


def conv_pool_fwd_ex(inp, filt, bias, out, stride, pad, relu, pool_ksz, pool_stride, workspace,
                     stream=None, variant=-1):
    """conv_pool_fwd_ex of the C ABI: convolution + bias + ReLU + max pooling; `out` is the
    pooled tensor."""
    N, C, H, W, K, R, S = _dims(inp, filt)
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    if 0 < pool_ksz <= min(P, Q) and pool_stride > 0 and tuple(out.shape) != (
            N, K, (P - pool_ksz) // pool_stride + 1, (Q - pool_ksz) // pool_stride + 1):
        raise ValueError("out must be the pooled tensor")
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(lib().conv_pool_fwd_ex(_dev_ptr(inp, "in"), _dev_ptr(filt, "filt"), _dev_ptr(bias, "bias"),
                                  _dev_ptr(out, "out"), N, C, H, W, K, R, S, stride, pad,
                                  1 if relu else 0, pool_ksz, pool_stride, ws_ptr, ws_bytes,
                                  _stream_handle(stream), int(variant)), "conv_pool_fwd_ex")
    return out


def conv_pool_fwd_workspace_bytes(N, C, H, W, K, R, S, stride, pad, variant=-1):
    return int(lib().conv_pool_fwd_workspace_bytes(N, C, H, W, K, R, S, stride, pad, int(variant)))


def conv_fwd_workspace_bytes(N, C, H, W, K, R, S, stride, pad, variant=-1):
    return int(lib().conv_fwd_workspace_bytes(N, C, H, W, K, R, S, stride, pad, int(variant)))


def _gemm_dims(a, b, c):
    M, K = a.shape
    K2, N = b.shape
    if K != K2 or tuple(c.shape) != (M, N):
        raise ValueError("sgemm shapes: A %s, B %s, C %s" % (tuple(a.shape), tuple(b.shape), tuple(c.shape)))
    return M, N, K


def sgemm(a, b, c):
    """sgemm of the C ABI: C = A * B, row-major (null stream, library workspace)."""
    M, N, K = _gemm_dims(a, b, c)
    _check(lib().sgemm(_dev_ptr(a, "A"), _dev_ptr(b, "B"), _dev_ptr(c, "C"), M, N, K), "sgemm")
    return c


def sgemm_ex(a, b, c, workspace=None, stream=None, variant=-1):
    """sgemm_ex of the C ABI; enqueues on `stream` (default: torch's current stream)."""
    M, N, K = _gemm_dims(a, b, c)
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(lib().sgemm_ex(_dev_ptr(a, "A"), _dev_ptr(b, "B"), _dev_ptr(c, "C"), M, N, K, ws_ptr,
                          ws_bytes, _stream_handle(stream), int(variant)), "sgemm_ex")
    return c


def sgemm_workspace_bytes(M, N, K, variant=-1):
    return int(lib().sgemm_workspace_bytes(M, N, K, int(variant)))


def bconv_debug_model_cost(N, C, H, W, K, R, S, stride, pad, variant):
    return float(lib().bconv_debug_model_cost(N, C, H, W, K, R, S, stride, pad, int(variant)))


def bconv_debug_mfma_loop(out, workgroups, iters, stream=None):
    """Register-only MFMA loop; returns the flops it executes."""
    if out.numel() < workgroups * 256:
        raise ValueError("out needs workgroups * 256 floats")
    _check(lib().bconv_debug_mfma_loop(_dev_ptr(out, "out"), int(workgroups), int(iters),
                                       _stream_handle(stream)), "bconv_debug_mfma_loop")
    return workgroups * 4 * iters * 16 * 4096


def conv_num_variants():
    return int(lib().conv_num_variants())


def conv_variant_name(variant):
    buf = ctypes.create_string_buffer(96)
    _check(lib().conv_variant_name(int(variant), buf, len(buf)), "conv_variant_name")
    return buf.value.decode()


def conv_selected_variant(N, C, H, W, K, R, S, stride, pad):
    v = int(lib().conv_selected_variant(N, C, H, W, K, R, S, stride, pad))
    if v < 0:
        raise BconvError(v, "conv_selected_variant")
    return v


def conv_pool_selected_variant(N, C, H, W, K, R, S, stride, pad, pool_ksz, pool_stride):
    v = int(lib().conv_pool_selected_variant(N, C, H, W, K, R, S, stride, pad, int(pool_ksz),
                                             int(pool_stride)))
    if v < 0:
        raise BconvError(v, "conv_pool_selected_variant")
    return v


def conv_fwd_f16_selected_variant(N, C, H, W, K, R, S, stride, pad):
    v = int(lib().conv_fwd_f16_selected_variant(N, C, H, W, K, R, S, stride, pad))
    if v < 0:
        raise BconvError(v, "conv_fwd_f16_selected_variant")
    return v


def conv_fwd_f16_variant_applicable(N, C, H, W, K, R, S, stride, pad, variant):
    v = int(lib().conv_fwd_f16_variant_applicable(N, C, H, W, K, R, S, stride, pad, int(variant)))
    if v < 0:
        raise BconvError(v, "conv_fwd_f16_variant_applicable")
    return bool(v)


def conv_fwd_f16_workspace_bytes(N, C, H, W, K, R, S, stride, pad, variant=-1):
    return int(lib().conv_fwd_f16_workspace_bytes(N, C, H, W, K, R, S, stride, pad, int(variant)))


def conv_f16_packed_filter_bytes(N, C, H, W, K, R, S, stride, pad, variant=-1):
    return int(lib().conv_f16_packed_filter_bytes(N, C, H, W, K, R, S, stride, pad, int(variant)))


def conv_f16_pack_filters(filt, packed, N, H, W, stride, pad, stream=None, variant=-1):
    """conv_f16_pack_filters of the C ABI: `filt` float16 K x C x R x S, `packed` any contiguous
    device tensor of at least conv_f16_packed_filter_bytes bytes."""
    K, C, R, S = filt.shape
    _check(lib().conv_f16_pack_filters(_dev_ptr(filt, "filt", True), packed.data_ptr(),
                                       packed.numel() * packed.element_size(), N, C, H, W, K, R, S, stride,
                                       pad, _stream_handle(stream), int(variant)), "conv_f16_pack_filters")
    return packed


def conv_fwd_f16_packed_ex(inp, packed, filt_shape, bias, out, stride, pad, relu, stream=None, variant=-1):
    """conv_fwd_f16_packed_ex of the C ABI; filt_shape = (K, C, R, S) of the filters `packed` was made from."""
    N, C, H, W = inp.shape
    K, C2, R, S = filt_shape
    if C != C2:
        raise ValueError("in has %d channels, the filters expect %d" % (C, C2))
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    if tuple(out.shape) != (N, K, P, Q):
        raise ValueError("out must have shape %s" % ((N, K, P, Q),))
    _check(lib().conv_fwd_f16_packed_ex(_dev_ptr(inp, "in", True), packed.data_ptr(), _dev_ptr(bias, "bias"),
                                        _dev_ptr(out, "out", True), N, C, H, W, K, R, S, stride, pad,
                                        1 if relu else 0, _stream_handle(stream), int(variant)),
           "conv_fwd_f16_packed_ex")
    return out


LAYOUT_NCHW, LAYOUT_C8 = 0, 1


def conv_fwd_f16_c8_selected_variant(N, C, H, W, K, R, S, stride, pad):
    v = int(lib().conv_fwd_f16_c8_selected_variant(N, C, H, W, K, R, S, stride, pad))
    if v < 0:
        raise BconvError(v, "conv_fwd_f16_c8_selected_variant")
    return v


def f16_layout_convert(inp, in_layout, out, out_layout, shape, stream=None):
    """f16_layout_convert of the C ABI; `shape` = (N, C, H, W) of the logical tensor.  A C8 tensor
    is passed as a tensor of shape (N, C // 8, H, W, 8)."""
    N, C, H, W = shape
    for t, lay, nm in ((inp, in_layout, "in"), (out, out_layout, "out")):
        want = (N, C // 8, H, W, 8) if lay == LAYOUT_C8 else (N, C, H, W)
        if tuple(t.shape) != want:
            raise ValueError("%s must have shape %s" % (nm, want))
    _check(lib().f16_layout_convert(_dev_ptr(inp, "in", True), int(in_layout), _dev_ptr(out, "out", True),
                                    int(out_layout), N, C, H, W, _stream_handle(stream)), "f16_layout_convert")
    return out


def conv_fwd_f16_layout_ex(inp, in_layout, filt, bias, out, out_layout, in_shape, stride, pad, relu, workspace,
                           stream=None, variant=-1):
    """conv_fwd_f16_layout_ex of the C ABI; in_shape = (N, C, H, W) of the logical input, `filt`
    float16 K x C x R x S; C8 tensors have shape (N, channels // 8, height, width, 8)."""
    N, C, H, W = in_shape
    K, C2, R, S = filt.shape
    if C != C2:
        raise ValueError("in has %d channels, the filters expect %d" % (C, C2))
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    want_in = (N, C // 8, H, W, 8) if in_layout == LAYOUT_C8 else (N, C, H, W)
    want_out = (N, K // 8, P, Q, 8) if out_layout == LAYOUT_C8 else (N, K, P, Q)
    if tuple(inp.shape) != want_in:
        raise ValueError("in must have shape %s" % (want_in,))
    if tuple(out.shape) != want_out:
        raise ValueError("out must have shape %s" % (want_out,))
    _check(lib().conv_fwd_f16_layout_ex(_dev_ptr(inp, "in", True), int(in_layout), _dev_ptr(filt, "filt", True),
                                        _dev_ptr(bias, "bias"), _dev_ptr(out, "out", True), int(out_layout),
                                        N, C, H, W, K, R, S, stride, pad, 1 if relu else 0,
                                        workspace.data_ptr() if workspace is not None else None,
                                        workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                        _stream_handle(stream), int(variant)),
           "conv_fwd_f16_layout_ex")
    return out


def conv_fwd_f16_packed_layout_ex(inp, in_layout, packed, filt_shape, bias, out, out_layout, in_shape, stride, pad,
                                  relu, stream=None, variant=-1):
    """conv_fwd_f16_packed_layout_ex of the C ABI; in_shape = (N, C, H, W) of the logical input,
    filt_shape = (K, C, R, S); C8 tensors have shape (N, channels // 8, height, width, 8)."""
    N, C, H, W = in_shape
    K, C2, R, S = filt_shape
    if C != C2:
        raise ValueError("in has %d channels, the filters expect %d" % (C, C2))
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    want_in = (N, C // 8, H, W, 8) if in_layout == LAYOUT_C8 else (N, C, H, W)
    want_out = (N, K // 8, P, Q, 8) if out_layout == LAYOUT_C8 else (N, K, P, Q)
    if tuple(inp.shape) != want_in:
        raise ValueError("in must have shape %s" % (want_in,))
    if tuple(out.shape) != want_out:
        raise ValueError("out must have shape %s" % (want_out,))
    _check(lib().conv_fwd_f16_packed_layout_ex(_dev_ptr(inp, "in", True), int(in_layout), packed.data_ptr(),
                                               _dev_ptr(bias, "bias"), _dev_ptr(out, "out", True), int(out_layout),
                                               N, C, H, W, K, R, S, stride, pad, 1 if relu else 0,
                                               _stream_handle(stream), int(variant)),
           "conv_fwd_f16_packed_layout_ex")
    return out


def conv_variant_applicable(N, C, H, W, K, R, S, stride, pad, variant):
    v = int(lib().conv_variant_applicable(N, C, H, W, K, R, S, stride, pad, int(variant)))
    if v < 0:
        raise BconvError(v, "conv_variant_applicable")
    return bool(v)


def bconv_debug_audit(N, C, H, W, K, R, S, stride, pad, variant):
    return int(lib().bconv_debug_audit(N, C, H, W, K, R, S, stride, pad, int(variant)))


def maxpool_fwd(inp, out, ksz, stride, stream=None):
    N, C, H, W = inp.shape
    _check(lib().maxpool_fwd(_dev_ptr(inp, "in"), _dev_ptr(out, "out"), N, C, H, W, ksz, stride,
                             _stream_handle(stream)), "maxpool_fwd")
    return out


def maxpool_fwd_f16(inp, out, layout, shape, ksz, stride, stream=None):
    """maxpool_fwd_f16 of the C ABI; `shape` = (N, C, H, W) of the logical input; C8 tensors have
    shape (N, C // 8, height, width, 8)."""
    N, C, H, W = shape
    P, Q = (H - ksz) // stride + 1, (W - ksz) // stride + 1
    want_in = (N, C // 8, H, W, 8) if layout == LAYOUT_C8 else (N, C, H, W)
    want_out = (N, C // 8, P, Q, 8) if layout == LAYOUT_C8 else (N, C, P, Q)
    if tuple(inp.shape) != want_in or tuple(out.shape) != want_out:
        raise ValueError("in / out must have shapes %s / %s" % (want_in, want_out))
    _check(lib().maxpool_fwd_f16(_dev_ptr(inp, "in", True), _dev_ptr(out, "out", True), int(layout), N, C, H, W,
                                 ksz, stride, _stream_handle(stream)), "maxpool_fwd_f16")
    return out


def variant_ids_by_name():
    return {conv_variant_name(v): v for v in range(conv_num_variants())}
