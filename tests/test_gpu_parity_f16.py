"""Parity of the half-precision-storage entry points against the CPU oracle.

The oracle rounds the exact result to fp16 once.  The library widens the fp16
elements exactly, multiplies exactly (an fp16 x fp16 product fits fp32) and sums in
fp32 on the matrix cores, then rounds to fp16 once.  The fp32 sum differs from the
exact one by far less than half an fp16 spacing, so the two roundings land on the same
fp16 value or on neighbours: |gpu - oracle| <= one fp16 spacing = 2^-10 * |oracle| at
most, with the fp32 path's absolute floor of 1e-5 where the terms cancel.
Integer-valued problems must match bit for bit: both sides round the same exact
integer.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import workloads
from paper_1606_00094_amd import binding
from tests.test_gpu_parity import FAMILY_SHAPES, _family_of, _tile_families

pytestmark = pytest.mark.gpu

RTOL, ATOL = 2.0 ** -10, 1e-5


def assert_close_f16(got, ref, what=""):
    assert got.dtype == np.float16 and ref.dtype == np.float16
    g, r = got.astype(np.float64), ref.astype(np.float64)
    err = np.abs(g - r)
    lim = np.maximum(ATOL, RTOL * np.abs(r))
    bad = err > lim
    if bad.any():
        i = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError("%s: %d of %d elements out of tolerance; worst at %s: got %r ref %r"
                             % (what, int(bad.sum()), bad.size, i, got[i], ref[i]))


def gpu_conv_f16(x, f, b, stride, pad, relu, variant=-1, use_simple_entry=False, guard=64,
                 shift=0):
    """Runs the fp16 entry point on host arrays; `out` sits between guard bands that must
    come back untouched.  shift > 0 places in and filt `shift` elements into their
    allocations (2-byte aligned pointers only)."""
    dev = torch.device("cuda:0")

    def put(a):
        flat = torch.zeros(a.size + shift, dtype=torch.float16, device=dev)
        flat[shift:] = torch.from_numpy(np.ascontiguousarray(a)).to(dev).reshape(-1)
        return flat[shift:].view(*a.shape)

    xd, fd = put(x), put(f)
    bd = torch.from_numpy(np.ascontiguousarray(b)).to(dev) if b is not None else None
    N, C, H, W = x.shape
    K, _, R, S = f.shape
    P, Q = binding.conv_out_dims(H, W, R, S, stride, pad)
    n_out = N * K * P * Q
    canary = 1234.5
    buf = torch.full((n_out + 2 * guard,), canary, dtype=torch.float16, device=dev)
    out = buf[guard:guard + n_out].view(N, K, P, Q)
    if use_simple_entry:
        torch.cuda.synchronize()
        binding.conv_fwd_f16(xd, fd, bd, out, stride, pad, relu)
    else:
        ws = None
        need = binding.conv_fwd_f16_workspace_bytes(N, C, H, W, K, R, S, stride, pad, variant)
        if need:
            ws = torch.zeros((need + 3) // 4, dtype=torch.float32, device=dev)
        binding.conv_fwd_f16_ex(xd, fd, bd, out, stride, pad, relu, workspace=ws, variant=variant)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert (host[:guard] == np.float16(canary)).all() and \
        (host[guard + n_out:] == np.float16(canary)).all(), "store outside the output tensor"
    return host[guard:guard + n_out].reshape(N, K, P, Q).copy()


def _layer_case(layer, N):
    """The benchmark layer's fp32 tensors rounded to fp16 (that rounding is the data's,
    not the method's); the bias stays fp32."""
    x, f, b = workloads.make_layer_inputs(layer, N)
    return x.astype(np.float16), f.astype(np.float16), b, layer.stride, layer.pad


@pytest.mark.parametrize("layer", workloads.ALL_LAYERS, ids=lambda l: l.name)
def test_f16_benchmark_layers_batch1(layer):
    x, f, b, s, p = _layer_case(layer, 1)
    for relu in (False, True):
        ref = oracle.conv_fwd_f16(x, f, b, stride=s, pad=p, relu=relu)
        got = gpu_conv_f16(x, f, b, s, p, relu)
        assert_close_f16(got, ref, "%s relu=%d" % (layer.name, relu))


@pytest.mark.parametrize("layer", workloads.ALL_LAYERS[1:], ids=lambda l: l.name)
def test_f16_benchmark_layers_batch32_every_image(layer):
    N = 32
    x, f, b, s, p = _layer_case(layer, N)
    for relu in (False, True):
        got = gpu_conv_f16(x, f, b, s, p, relu)
        ref = oracle.conv_fwd_f16(x, f, b, stride=s, pad=p, relu=relu)
        assert_close_f16(got, ref, "%s N=32 relu=%d" % (layer.name, relu))


def test_f16_simple_entry_direct_kernel_and_missing_bias():
    for layer in (workloads.TOY, workloads.PW_B):
        x, f, b, s, p = _layer_case(layer, 1)
        ref = oracle.conv_fwd_f16(x, f, b, stride=s, pad=p, relu=True)
        assert_close_f16(gpu_conv_f16(x, f, b, s, p, True, use_simple_entry=True), ref, layer.name)
        assert_close_f16(gpu_conv_f16(x, f, b, s, p, True, variant=0), ref, layer.name + " direct")
        ref = oracle.conv_fwd_f16(x, f, None, stride=s, pad=p, relu=False)
        assert_close_f16(gpu_conv_f16(x, f, None, s, p, False), ref, layer.name + " no bias")


def test_f16_matrix_core_tiles_through_the_simple_entry_and_errors():
    """A launch large enough for the fp16-matrix-core tiles through conv_fwd_f16 (library's own
    workspace for the re-laid filters), without bias and without ReLU too; the fp32 entry point
    refuses such a variant, and the half-precision one refuses it without its workspace."""
    layer, N = workloads.RED3, 8
    dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
    v = binding.conv_fwd_f16_selected_variant(*dims)
    assert binding.conv_variant_name(v).startswith("h16")
    assert not binding.conv_variant_applicable(*dims, v)
    assert binding.conv_fwd_f16_workspace_bytes(*dims, v) > 0
    x, f, b, s, p = _layer_case(layer, N)
    ref = oracle.conv_fwd_f16(x, f, b, stride=s, pad=p, relu=True)
    assert_close_f16(gpu_conv_f16(x, f, b, s, p, True, use_simple_entry=True), ref, "simple entry")
    ref = oracle.conv_fwd_f16(x, f, None, stride=s, pad=p, relu=False)
    assert_close_f16(gpu_conv_f16(x, f, None, s, p, False), ref, "no bias, no relu")
    dev = torch.device("cuda:0")
    xd, fd = torch.from_numpy(x).to(dev), torch.from_numpy(f).to(dev)
    out = torch.zeros((N, layer.K, 28, 28), dtype=torch.float16, device=dev)
    with pytest.raises(binding.BconvError) as e:
        binding.conv_fwd_f16_ex(xd, fd, None, out, s, p, True, workspace=None, variant=v)
    assert e.value.status == -4
    with pytest.raises(binding.BconvError) as e:
        binding.conv_fwd_ex(xd.float(), fd.float(), None, out.float(), s, p, True, variant=v)
    assert e.value.status == -6
    torch.cuda.synchronize()


def test_f16_prepacked_filters_equal_the_per_call_path_bit_for_bit():
    """Filters re-laid once (conv_f16_pack_filters) and used by conv_fwd_f16_packed_ex on two
    different inputs: the same bits as conv_fwd_f16_ex with that variant, and the oracle's values.
    A shape whose choice is not an fp16-matrix-core tile has nothing to pack."""
    dev = torch.device("cuda:0")
    for layer, N, variant in ((workloads.CONV3, 16, -1), (workloads.PW_A, 32, -1), (workloads.CONV2, 8, None)):
        dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
        if variant is None:     # a forced tile that is not the table's choice
            variant = binding.variant_ids_by_name()["h16k5_64x64_c16/s1"]
            assert variant != binding.conv_fwd_f16_selected_variant(*dims)
        nbytes = binding.conv_f16_packed_filter_bytes(*dims, variant)
        assert nbytes > 0 and nbytes == binding.conv_fwd_f16_workspace_bytes(
            *dims, variant if variant >= 0 else binding.conv_fwd_f16_selected_variant(*dims))
        x, f, b, s, p = _layer_case(layer, N)
        fd, bd = torch.from_numpy(f).to(dev), torch.from_numpy(b).to(dev)
        packed = torch.full(((nbytes + 3) // 4,), float("nan"), dtype=torch.float32, device=dev)
        binding.conv_f16_pack_filters(fd, packed, N, layer.H, layer.W, s, p, variant=variant)
        P, Q = binding.conv_out_dims(layer.H, layer.W, layer.R, layer.S, s, p)
        for rep in range(2):
            xr = x if rep == 0 else np.ascontiguousarray(x[::-1])
            xd = torch.from_numpy(xr).to(dev)
            got = torch.full((N, layer.K, P, Q), float("nan"), dtype=torch.float16, device=dev)
            binding.conv_fwd_f16_packed_ex(xd, packed, f.shape, bd, got, s, p, True, variant=variant)
            torch.cuda.synchronize()
            want = gpu_conv_f16(xr, f, b, s, p, True, variant=variant)
            assert np.array_equal(got.cpu().numpy(), want), (layer.name, rep)
            if rep == 0:
                assert_close_f16(want, oracle.conv_fwd_f16(xr, f, b, stride=s, pad=p, relu=True), layer.name)
        with pytest.raises(binding.BconvError) as e:       # too small a buffer for the packed copy
            binding.conv_f16_pack_filters(fd, packed[:8], N, layer.H, layer.W, s, p, variant=variant)
        assert e.value.status == -4
    layer = workloads.CONV1
    dims = (4, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
    assert binding.conv_f16_packed_filter_bytes(*dims, -1) == 0
    torch.cuda.synchronize()


# (the vector-FMA first-layer kernels are fp32-storage only)
@pytest.mark.parametrize("tile", sorted(t for t in _tile_families() if not t.startswith("fmaq")))
def test_f16_every_tile_variant_exact_on_integers(tile):
    """Each compiled tile in its fp16 instantiation, unsplit and with every applicable
    reduction split, on shapes with ragged tails: bitwise equal to the oracle."""
    fam = _family_of(tile)
    ran = 0
    for shp in FAMILY_SHAPES[fam]:
        if fam == (0, 0, 0):
            N, C, H, W, K, pad, R, S, stride = shp
        else:
            N, C, H, W, K, pad = shp
            R, S, stride = fam
        x, f, b = workloads.make_integer_problem(len(tile) + sum(shp), N, C, H, W, K, R, S)
        x, f = x.astype(np.float16), f.astype(np.float16)
        ref = oracle.conv_fwd_f16(x, f, b, stride=stride, pad=pad, relu=False)
        for v in _tile_families()[tile]:
            if not binding.conv_fwd_f16_variant_applicable(N, C, H, W, K, R, S, stride, pad, v):
                continue
            got = gpu_conv_f16(x, f, b, stride, pad, False, variant=v)
            assert np.array_equal(got, ref), "%s on %s" % (binding.conv_variant_name(v), (shp,))
            ran += 1
    assert ran > 0


def test_f16_pointers_with_two_byte_alignment_only():
    """in and filt one element into their allocations: the table's 4-element-load choice
    must degrade to its narrow twin, a forced wide variant must be refused."""
    for layer in (workloads.PW_A, workloads.CONV3, workloads.RED5):
        x, f, b, s, p = _layer_case(layer, 1)
        ref = oracle.conv_fwd_f16(x, f, b, stride=s, pad=p, relu=True)
        assert_close_f16(gpu_conv_f16(x, f, b, s, p, True, shift=1), ref, layer.name + " shifted")
    layer = workloads.PW_A
    x, f, b, s, p = _layer_case(layer, 1)
    wide = binding.variant_ids_by_name()["pw_64x64_k16_v4b4/s1"]
    with pytest.raises(binding.BconvError) as e:
        gpu_conv_f16(x, f, b, s, p, True, variant=wide, shift=1)
    assert e.value.status == -6


def test_f16_split_reduction_both_store_widths():
    # out_elems % 4 == 0 and != 0; the second through an output pointer 2 bytes off 8
    for (N, C, H, W, K, R, pad, tile) in [(1, 64, 8, 8, 40, 3, 1, "k3_64x64_k12_h/s4"),
                                          (1, 64, 7, 7, 33, 3, 1, "k3_64x64_k12_h/s4"),
                                          (1, 96, 6, 6, 40, 1, 0, "pw_64x64_k16/s3")]:
        x, f, b = workloads.make_random_problem(N * C + H, N, C, H, W, K, R, R)
        x, f = x.astype(np.float16), f.astype(np.float16)
        v = binding.variant_ids_by_name()[tile]
        ref = oracle.conv_fwd_f16(x, f, b, stride=1, pad=pad, relu=True)
        for guard in (64, 63):
            got = gpu_conv_f16(x, f, b, 1, pad, True, variant=v, guard=guard)
            assert_close_f16(got, ref, "%s guard %d" % (tile, guard))


def test_f16_rejects_odd_pointers_and_float32_tensors():
    dev = torch.device("cuda:0")
    x = torch.zeros((1, 4, 5, 5), dtype=torch.float16, device=dev)
    f = torch.zeros((3, 4, 3, 3), dtype=torch.float16, device=dev)
    out = torch.zeros((1, 3, 3, 3), dtype=torch.float16, device=dev)
    with pytest.raises(TypeError):
        binding.conv_fwd_f16(x.float(), f, None, out, 1, 0, False)
    rc = binding.lib().conv_fwd_f16(ctypes.c_void_p(x.data_ptr() + 1), f.data_ptr(), None,
                                    out.data_ptr(), 1, 4, 5, 5, 3, 3, 3, 1, 0, 0)
    assert rc == -1
    torch.cuda.synchronize()
