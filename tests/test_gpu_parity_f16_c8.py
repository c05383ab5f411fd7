"""Half-precision layers on octet-interleaved (C8 = [N][C/8][H][W][8]) activations, on the GPU.

The C8 calls compute what the NCHW calls compute; only where an element lives changes.  So
every check converts back with f16_layout_convert (itself pinned against a numpy transpose)
and compares with the oracle to the half-precision bar of test_gpu_parity_f16 -- bit for bit
on integer-valued data -- and with the NCHW path of the same tile bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from paper_1606_00094_amd import binding
from tests.test_gpu_parity import FAMILY_SHAPES, _family_of, _tile_families
from tests.test_gpu_parity_f16 import assert_close_f16

pytestmark = pytest.mark.gpu

NCHW, C8 = binding.LAYOUT_NCHW, binding.LAYOUT_C8


# shapes with K a multiple of eight (C8 output), ragged in the pixel and filter tiles, beside the
# family shapes of the every-tile tests: (N, C, H, W, K, pad)
C8_SHAPES = {
    (3, 3, 1): [(2, 16, 13, 13, 72, 1), (1, 24, 30, 31, 136, 1), (5, 8, 27, 27, 264, 1)],
    (5, 5, 1): [(2, 8, 27, 27, 72, 2), (3, 24, 14, 14, 136, 2)],
    (1, 1, 1): [(3, 40, 7, 7, 56, 0), (2, 72, 14, 14, 136, 0), (9, 32, 28, 28, 264, 0)],
}


def to_c8_numpy(a):
    n, c, h, w = a.shape
    return np.ascontiguousarray(a.reshape(n, c // 8, 8, h, w).transpose(0, 1, 3, 4, 2))


def gpu_conv_c8(x, f, b, stride, pad, relu, variant, c8_out, guard=64):
    """x, f fp16 numpy (NCHW / KCRS), b fp32 or None.  Packs the filters, converts x to C8 on the
    GPU, runs conv_fwd_f16_packed_layout_ex into a guarded buffer and returns the result as an
    NCHW numpy array (converted back on the GPU when the output was C8)."""
    dev = torch.device("cuda:0")
    N, C, H, W = x.shape
    K, _, R, S = f.shape
    P, Q = binding.conv_out_dims(H, W, R, S, stride, pad)
    dims = (N, C, H, W, K, R, S, stride, pad)
    nbytes = binding.conv_f16_packed_filter_bytes(*dims, variant)
    assert nbytes > 0, binding.conv_variant_name(variant)
    fd = torch.from_numpy(f).to(dev)
    bd = None if b is None else torch.from_numpy(b).to(dev)
    packed = torch.full(((nbytes + 3) // 4,), float("nan"), dtype=torch.float32, device=dev)
    binding.conv_f16_pack_filters(fd, packed, N, H, W, stride, pad, variant=variant)
    xd = torch.from_numpy(x).to(dev)
    x8 = torch.empty((N, C // 8, H, W, 8), dtype=torch.float16, device=dev)
    binding.f16_layout_convert(xd, NCHW, x8, C8, (N, C, H, W))
    n_out = N * K * P * Q
    # guard words on both sides of the output (multiples of eight elements keep it 16-byte aligned)
    buf = torch.full((n_out + 2 * guard,), -77.0, dtype=torch.float16, device=dev)
    body = buf[guard:guard + n_out]
    if c8_out:
        out = body.view(N, K // 8, P, Q, 8)
    else:
        out = body.view(N, K, P, Q)
    binding.conv_fwd_f16_packed_layout_ex(x8, C8, packed, f.shape, bd, out, C8 if c8_out else NCHW,
                                          (N, C, H, W), stride, pad, relu, variant=variant)
    torch.cuda.synchronize()
    assert bool((buf[:guard] == -77.0).all()) and bool((buf[guard + n_out:] == -77.0).all()), "wrote outside out"
    if c8_out:
        back = torch.empty((N, K, P, Q), dtype=torch.float16, device=dev)
        binding.f16_layout_convert(out, C8, back, NCHW, (N, K, P, Q))
        torch.cuda.synchronize()
        return back.cpu().numpy()
    return out.cpu().numpy()


def test_layout_convert_is_the_transpose_both_ways():
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(workloads.BASE_SEED + 77)
    for shape in ((1, 8, 1, 1), (3, 24, 5, 7), (2, 96, 27, 27), (5, 256, 13, 13)):
        n, c, h, w = shape
        a = rng.standard_normal(shape).astype(np.float16)
        ad = torch.from_numpy(a).to(dev)
        a8 = torch.full((n, c // 8, h, w, 8), float("nan"), dtype=torch.float16, device=dev)
        binding.f16_layout_convert(ad, NCHW, a8, C8, shape)
        assert np.array_equal(a8.cpu().numpy(), to_c8_numpy(a)), shape
        back = torch.full(shape, float("nan"), dtype=torch.float16, device=dev)
        binding.f16_layout_convert(a8, C8, back, NCHW, shape)
        assert np.array_equal(back.cpu().numpy(), a), shape
    # refusals: channels not a multiple of eight, the same layout twice, one buffer for both
    bad = torch.zeros((1, 12, 2, 2), dtype=torch.float16, device=dev)
    for call in (lambda: binding.lib().f16_layout_convert(bad.data_ptr(), NCHW, ad.data_ptr(), C8, 1, 12, 2, 2, None),
                 lambda: binding.lib().f16_layout_convert(ad.data_ptr(), NCHW, a8.data_ptr(), NCHW, n, c, h, w, None),
                 lambda: binding.lib().f16_layout_convert(ad.data_ptr(), NCHW, ad.data_ptr(), C8, n, c, h, w, None),
                 lambda: binding.lib().f16_layout_convert(ad.data_ptr(), NCHW, a8.data_ptr() + 2, C8, n, c, h, w, None)):
        assert call() == -1
    assert binding.lib().f16_layout_convert(None, NCHW, a8.data_ptr(), C8, n, c, h, w, None) == -2
    torch.cuda.synchronize()


# (the first-layer tiles h16k11s4 / h16k7s2 take three-channel NCHW input only)
@pytest.mark.parametrize("tile", sorted(t for t in _tile_families()
                                        if t.startswith("h16") and not t.startswith(("h16k11s4", "h16k7s2"))))
def test_c8_every_matrix_core_tile_exact_on_integers(tile):
    """Each fp16-matrix-core tile on C8 input, writing C8 (where K is a multiple of eight) and
    NCHW, on the ragged shapes of its family: bitwise equal to the oracle."""
    fam = _family_of(tile)
    ran = 0
    for shp in FAMILY_SHAPES[fam] + C8_SHAPES[fam]:
        N, C, H, W, K, pad = shp
        R, S, stride = fam
        if C % 8:
            continue
        x, f, b = workloads.make_integer_problem(len(tile) + sum(shp), N, C, H, W, K, R, S)
        x, f = x.astype(np.float16), f.astype(np.float16)
        ref = oracle.conv_fwd_f16(x, f, b, stride=stride, pad=pad, relu=False)
        for v in _tile_families()[tile]:          # unsplit and every reduction split that applies
            if not binding.conv_fwd_f16_variant_applicable(N, C, H, W, K, R, S, stride, pad, v):
                continue
            for c8_out in ((True, False) if K % 8 == 0 else (False,)):
                got = gpu_conv_c8(x, f, b, stride, pad, False, v, c8_out)
                assert np.array_equal(got, ref), "%s on %s, C8 out %s" % (binding.conv_variant_name(v), shp, c8_out)
                ran += 1
    assert ran > 0


@pytest.mark.parametrize("layer", [l for l in workloads.ALL_LAYERS if l.stride == 1 and l.C % 8 == 0],
                         ids=lambda l: l.name)
def test_c8_benchmark_layers_batch32_every_image(layer):
    """The benchmark layers at the benchmark batch with the tile chosen for C8 activations: every
    image against the oracle, and the same bits as the NCHW path of that tile."""
    N = 32
    dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
    v = binding.conv_fwd_f16_c8_selected_variant(*dims)
    assert binding.conv_variant_name(v).startswith("h16")
    x, f, b = workloads.make_layer_inputs(layer, N, seed=workloads.BASE_SEED + 600000 + sum(dims))
    x, f = x.astype(np.float16), f.astype(np.float16)
    ref = oracle.conv_fwd_f16(x, f, b, stride=layer.stride, pad=layer.pad, relu=True)
    got = gpu_conv_c8(x, f, b, layer.stride, layer.pad, True, v, layer.K % 8 == 0)
    assert_close_f16(got, ref, "%s via %s on C8" % (layer.name, binding.conv_variant_name(v)))
    plain = gpu_conv_c8(x, f, b, layer.stride, layer.pad, True, v, False)
    assert np.array_equal(got, plain)


def test_c8_chain_of_two_layers_stays_in_c8():
    """conv3 -> conv4 of the benchmark stack at batch 8 with the activations never leaving C8:
    equal to running the two layers through the oracle (the second on the first's rounded
    output)."""
    N = 8
    l3, l4 = workloads.CONV3, workloads.CONV4
    x, f3, b3 = workloads.make_layer_inputs(l3, N, seed=workloads.BASE_SEED + 611)
    _, f4, b4 = workloads.make_layer_inputs(l4, N, seed=workloads.BASE_SEED + 612)
    x, f3, f4 = x.astype(np.float16), f3.astype(np.float16), f4.astype(np.float16)
    dev = torch.device("cuda:0")
    mid_ref = oracle.conv_fwd_f16(x, f3, b3, stride=1, pad=l3.pad, relu=True)
    ref = oracle.conv_fwd_f16(mid_ref, f4, b4, stride=1, pad=l4.pad, relu=True)
    shapes = ((N, l3.C, l3.H, l3.W), (N, l3.K, l3.H, l3.W), (N, l4.K, l4.H, l4.W))
    bufs = [torch.empty((n, c // 8, h, w, 8), dtype=torch.float16, device=dev) for n, c, h, w in shapes]
    binding.f16_layout_convert(torch.from_numpy(x).to(dev), NCHW, bufs[0], C8, shapes[0])
    for i, (layer, f, b) in enumerate(((l3, f3, b3), (l4, f4, b4))):
        dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, 1, layer.pad)
        v = binding.conv_fwd_f16_c8_selected_variant(*dims)
        packed = torch.empty(binding.conv_f16_packed_filter_bytes(*dims, v) // 2, dtype=torch.float16, device=dev)
        binding.conv_f16_pack_filters(torch.from_numpy(f).to(dev), packed, N, layer.H, layer.W, 1, layer.pad, variant=v)
        binding.conv_fwd_f16_packed_layout_ex(bufs[i], C8, packed, f.shape, torch.from_numpy(b).to(dev), bufs[i + 1],
                                              C8, shapes[i], 1, layer.pad, True, variant=v)
    out = torch.empty(shapes[2], dtype=torch.float16, device=dev)
    binding.f16_layout_convert(bufs[2], C8, out, NCHW, shapes[2])
    torch.cuda.synchronize()
    # the middle activations agree with the oracle's to one fp16 spacing, which the second layer
    # then amplifies by at most its absolute row sums; the bar below is that bound, evaluated
    mid = torch.empty(shapes[1], dtype=torch.float16, device=dev)
    binding.f16_layout_convert(bufs[1], C8, mid, NCHW, shapes[1])
    assert_close_f16(mid.cpu().numpy(), mid_ref, "conv3 in the chain")
    ref_on_gpu_mid = oracle.conv_fwd_f16(mid.cpu().numpy(), f4, b4, stride=1, pad=l4.pad, relu=True)
    assert_close_f16(out.cpu().numpy(), ref_on_gpu_mid, "conv4 on the chain's own conv3 output")
    assert ref.shape == ref_on_gpu_mid.shape


@pytest.mark.parametrize("layout", [NCHW, C8])
def test_maxpool_f16_both_layouts(layout):
    """Pooling of fp16 activations: bit for bit the oracle's pooling (a maximum is one of its
    inputs), windows 3/2, 2/2 and 3/1, negative values, ragged extents."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(workloads.BASE_SEED + 88 + layout)
    for shape, ksz, stride in (((2, 16, 13, 13), 3, 2), ((1, 96, 55, 55), 3, 2), ((3, 8, 8, 9), 2, 2),
                               ((2, 24, 7, 5), 3, 1), ((1, 8, 3, 3), 3, 2)):
        n, c, h, w = shape
        a = rng.standard_normal(shape).astype(np.float16)
        ref = oracle.maxpool_fwd(a.astype(np.float32), ksz, stride).astype(np.float16)
        P, Q = ref.shape[2:]
        ad = torch.from_numpy(a).to(dev)
        if layout == C8:
            a8 = torch.empty((n, c // 8, h, w, 8), dtype=torch.float16, device=dev)
            binding.f16_layout_convert(ad, NCHW, a8, C8, shape)
            o8 = torch.full((n, c // 8, P, Q, 8), float("nan"), dtype=torch.float16, device=dev)
            binding.maxpool_fwd_f16(a8, o8, C8, shape, ksz, stride)
            out = torch.empty((n, c, P, Q), dtype=torch.float16, device=dev)
            binding.f16_layout_convert(o8, C8, out, NCHW, (n, c, P, Q))
        else:
            out = torch.full((n, c, P, Q), float("nan"), dtype=torch.float16, device=dev)
            binding.maxpool_fwd_f16(ad, out, NCHW, shape, ksz, stride)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), ref), (shape, ksz, stride)
    lib = binding.lib()
    assert lib.maxpool_fwd_f16(ad.data_ptr(), out.data_ptr(), C8, 1, 12, 5, 5, 3, 2, None) == -1
    assert lib.maxpool_fwd_f16(ad.data_ptr(), out.data_ptr(), NCHW, 1, 8, 2, 2, 3, 2, None) == -3
    assert lib.maxpool_fwd_f16(None, out.data_ptr(), NCHW, 1, 8, 5, 5, 3, 2, None) == -2
    assert lib.maxpool_fwd_f16(ad.data_ptr() + 2, out.data_ptr(), C8, 1, 8, 5, 5, 3, 2, None) == -1


@pytest.mark.parametrize("N", [1, 5, 32])
def test_five_layer_stack_in_half_precision_as_the_benchmark_runs_it(N):
    """The five-layer stack with fp16 storage the way bench.py times it (first layer NCHW, then
    C8 throughout): every layer against the oracle applied to that layer's actual GPU input,
    every image, to the half-precision bar."""
    import bench
    img, params = workloads.make_stack_inputs(N)
    st = bench.F16Stack(N, img, params)
    st.step()
    torch.cuda.synchronize()
    acts = st.activations_nchw()
    for li, (layer, (f, b)) in enumerate(zip(workloads.STACK, params)):
        ref16 = oracle.conv_fwd_f16(acts[li], f.astype(np.float16), b, stride=layer.stride, pad=layer.pad, relu=True)
        if li in workloads.STACK_POOL_AFTER:
            ref16 = oracle.maxpool_fwd(ref16.astype(np.float32), 3, 2).astype(np.float16)
        assert_close_f16(acts[li + 1], ref16, "f16 stack N=%d %s" % (N, layer.name))
    assert acts[-1].shape == (N, 256, 13, 13)


def test_c8_refusals():
    """C8 output from NCHW input, C8 output with K not a multiple of eight, a misaligned C8
    pointer, an unknown layout: BCONV_EINVAL; a tile that is not an fp16-matrix-core one:
    BCONV_EVARIANT; shapes no such tile serves have no C8 choice."""
    dev = torch.device("cuda:0")
    N, C, H, W, K = 2, 16, 9, 9, 12
    dims = (N, C, H, W, K, 3, 3, 1, 1)
    v = binding.conv_fwd_f16_c8_selected_variant(*dims)
    x8 = torch.zeros((N, C // 8, H, W, 8), dtype=torch.float16, device=dev)
    xn = torch.zeros((N, C, H, W), dtype=torch.float16, device=dev)
    out = torch.zeros((N * K * H * W + 16,), dtype=torch.float16, device=dev)
    packed = torch.zeros(binding.conv_f16_packed_filter_bytes(*dims, v) // 2, dtype=torch.float16, device=dev)
    lib = binding.lib()

    def call(inp, il, o, ol, k=K, variant=v):
        return lib.conv_fwd_f16_packed_layout_ex(inp, il, packed.data_ptr(), None, o, ol, N, C, H, W, k, 3, 3, 1, 1,
                                                 0, None, variant)
    assert call(x8.data_ptr(), C8, out.data_ptr(), NCHW) == 0
    assert call(xn.data_ptr(), NCHW, out.data_ptr(), NCHW) == 0
    assert call(xn.data_ptr(), NCHW, out.data_ptr(), C8, k=8) == -1
    assert call(x8.data_ptr(), C8, out.data_ptr(), C8) == -1            # K = 12
    assert call(x8.data_ptr() + 2, C8, out.data_ptr(), NCHW) == -1
    assert call(x8.data_ptr(), C8, out.data_ptr() + 2, C8, k=8) == -1
    assert call(x8.data_ptr(), 2, out.data_ptr(), NCHW) == -1
    assert call(x8.data_ptr(), C8, out.data_ptr(), NCHW, variant=binding.conv_selected_variant(*dims)) == -6
    l1 = workloads.CONV1
    assert lib.conv_fwd_f16_c8_selected_variant(4, l1.C, l1.H, l1.W, l1.K, l1.R, l1.S, l1.stride, l1.pad) == -6
    assert lib.conv_fwd_f16_c8_selected_variant(4, 16, 9, 9, 8, 3, 3, 2, 1) == -6
    torch.cuda.synchronize()


@pytest.mark.parametrize("N", [1, 5, 32])
def test_first_layer_tiles_write_c8_directly(N):
    """conv_fwd_f16_layout_ex, NCHW in -> C8 out, on the first benchmark layer (the first-layer
    fp16-matrix-core tiles are the half-precision path's choice there at every batch): every
    image against the oracle, and the same bits as the NCHW output of the same call."""
    layer = workloads.CONV1
    dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
    v = binding.conv_fwd_f16_selected_variant(*dims)
    assert binding.conv_variant_name(v).startswith("h16k11s4"), binding.conv_variant_name(v)
    x, f, b = workloads.make_layer_inputs(layer, N, seed=workloads.BASE_SEED + 620 + N)
    x, f = x.astype(np.float16), f.astype(np.float16)
    dev = torch.device("cuda:0")
    P, Q = binding.conv_out_dims(layer.H, layer.W, layer.R, layer.S, layer.stride, layer.pad)
    xd, fd, bd = torch.from_numpy(x).to(dev), torch.from_numpy(f).to(dev), torch.from_numpy(b).to(dev)
    ws = torch.zeros(binding.conv_fwd_f16_workspace_bytes(*dims, v) // 4 + 1, dtype=torch.float32, device=dev)
    o8 = torch.full((N, layer.K // 8, P, Q, 8), float("nan"), dtype=torch.float16, device=dev)
    binding.conv_fwd_f16_layout_ex(xd, NCHW, fd, bd, o8, C8, x.shape, layer.stride, layer.pad, True, ws)
    got = torch.empty((N, layer.K, P, Q), dtype=torch.float16, device=dev)
    binding.f16_layout_convert(o8, C8, got, NCHW, (N, layer.K, P, Q))
    plain = torch.full((N, layer.K, P, Q), float("nan"), dtype=torch.float16, device=dev)
    binding.conv_fwd_f16_layout_ex(xd, NCHW, fd, bd, plain, NCHW, x.shape, layer.stride, layer.pad, True, ws)
    torch.cuda.synchronize()
    ref = oracle.conv_fwd_f16(x, f, b, stride=layer.stride, pad=layer.pad, relu=True)
    assert_close_f16(got.cpu().numpy(), ref, "conv1 N=%d to C8" % N)
    assert torch.equal(got, plain)
    lib = binding.lib()
    # a first-layer tile cannot read C8; too small a workspace; C8 out with K not a multiple of eight
    args = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad, 1)
    assert lib.conv_fwd_f16_layout_ex(xd.data_ptr(), NCHW, fd.data_ptr(), bd.data_ptr(), o8.data_ptr(), C8, *args,
                                      ws.data_ptr(), 16, None, v) == -4
    assert lib.conv_fwd_f16_layout_ex(xd.data_ptr(), NCHW, fd.data_ptr(), bd.data_ptr(), o8.data_ptr(), C8,
                                      N, layer.C, layer.H, layer.W, 92, layer.R, layer.S, layer.stride, layer.pad, 1,
                                      ws.data_ptr(), ws.numel() * 4, None, v) == -1


@pytest.mark.parametrize("tile,shape", [("h16k11s4_p64", (1, 3, 51, 55, 40, 11, 4, 0)),
                                        ("h16k7s2_p32", (1, 3, 29, 31, 40, 7, 2, 3))])
def test_first_layer_tiles_keep_an_infinity_inside_its_windows(tile, shape):
    """One +Inf input element: the outputs whose window contains it are non-finite, every other
    output is the oracle's finite value (the kernel's reduction slots past the kernel width read
    neighbouring columns; they must not leak)."""
    N, C, H, W, K, R, stride, pad = shape
    v = binding.variant_ids_by_name()[tile + "/s1"]
    x, f, b = workloads.make_integer_problem(99, N, C, H, W, K, R, R)
    x, f = x.astype(np.float16), np.abs(f).astype(np.float16) + np.float16(1)
    x[0, 1, H // 2, W // 2] = np.float16(np.inf)
    with np.errstate(invalid="ignore"):
        ref = oracle.conv_fwd_f16(x, f, b, stride=stride, pad=pad, relu=False)
    dev = torch.device("cuda:0")
    P, Q = ref.shape[2:]
    dims = (N, C, H, W, K, R, R, stride, pad)
    ws = torch.zeros(binding.conv_fwd_f16_workspace_bytes(*dims, v) // 4 + 1, dtype=torch.float32, device=dev)
    out = torch.empty((N, K, P, Q), dtype=torch.float16, device=dev)
    binding.conv_fwd_f16_ex(torch.from_numpy(x).to(dev), torch.from_numpy(f).to(dev), torch.from_numpy(b).to(dev), out,
                            stride, pad, False, workspace=ws, variant=v)
    got = out.cpu().numpy()
    finite = np.isfinite(ref)
    assert 0 < (~finite).sum() < ref.size
    assert np.array_equal(np.isfinite(got), finite)
    assert np.array_equal(got[finite], ref[finite])


@pytest.mark.parametrize("fam", [(3, 3, 1), (5, 5, 1), (1, 1, 1)], ids=lambda f: "%dx%d" % f[:2])
def test_c8_tiles_keep_an_infinity_inside_its_windows(fam):
    """The channel-octet tiles pad the last chunk's channels with zero filters; the input side of
    those channels must be zero too (it is: octets past the last channel are not loaded).  One
    +Inf input element, every applicable tile, C8 in and out."""
    R, S, stride = fam
    N, C, H, W, K, pad = C8_SHAPES[fam][0]
    x, f, b = workloads.make_integer_problem(5 + R, N, C, H, W, K, R, S)
    x, f = x.astype(np.float16), (np.abs(f) + 1).astype(np.float16)
    x[N - 1, C - 1, H // 2, W // 2] = np.float16(np.inf)
    ref = oracle.conv_fwd_f16(x, f, b, stride=stride, pad=pad, relu=False)
    finite = np.isfinite(ref)
    assert 0 < (~finite).sum() < ref.size
    ran = 0
    for tile, ids in sorted((t, ids) for t, ids in _tile_families().items()
                            if t.startswith("h16") and _family_of(t) == fam):
        v = ids[0]
        if not binding.conv_fwd_f16_variant_applicable(N, C, H, W, K, R, S, stride, pad, v):
            continue
        got = gpu_conv_c8(x, f, b, stride, pad, False, v, True)
        assert np.array_equal(np.isfinite(got), finite), tile
        assert np.array_equal(got[finite], ref[finite]), tile
        ran += 1
    assert ran > 0


UNLISTED_C8 = [(3, 256, 28, 28, 256, 3, 3, 1, 1), (3, 512, 14, 14, 512, 1, 1, 1, 0), (2, 48, 14, 14, 128, 5, 5, 1, 2),
               (8, 160, 7, 7, 320, 3, 3, 1, 1), (1, 64, 56, 56, 256, 1, 1, 1, 0), (2, 512, 14, 14, 512, 3, 3, 1, 1),
               (1, 24, 9, 11, 40, 3, 3, 1, 0), (4, 8, 5, 5, 16, 5, 5, 1, 2)]


@pytest.mark.parametrize("dims", UNLISTED_C8, ids=lambda d: "N%d_C%d_%dx%d_K%d_%dx%d" % d[:7])
def test_c8_unlisted_shapes_through_the_cost_model(dims):
    """Shapes neither half-precision table lists: the variant the fitted cost model picks (tile
    and reduction split) applies and gives the oracle's values on C8 activations."""
    N, C, H, W, K, R, S, stride, pad = dims
    v = binding.conv_fwd_f16_c8_selected_variant(*dims)
    name = binding.conv_variant_name(v)
    assert name.startswith("h16") and binding.conv_fwd_f16_variant_applicable(*dims, v), name
    x, f, b = workloads.make_random_problem(workloads.BASE_SEED + 640 + sum(dims), N, C, H, W, K, R, S, dist="u01")
    x, f = x.astype(np.float16), (f * np.float32(0.05)).astype(np.float16)
    ref = oracle.conv_fwd_f16(x, f, b, stride=stride, pad=pad, relu=True)
    got = gpu_conv_c8(x, f, b, stride, pad, True, v, K % 8 == 0)
    assert_close_f16(got, ref, "%s via %s" % (dims, name))
