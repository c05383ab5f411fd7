"""Host-side tests of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, rejects bad arguments before touching the device,
and its launch plans pass the bounds audit for the benchmark shapes."""
import ctypes
import os
import re

import pytest

import workloads
from paper_1606_00094_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "bconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", text)
    return sorted(set(n for n in names if n.startswith(("conv_", "bconv_", "maxpool_", "sgemm", "f16_"))))


def test_library_loads_and_exports_every_declared_symbol():
    lib = ctypes.CDLL(binding.LIB_PATH)
    declared = _declared_functions()
    assert "conv_fwd" in declared and "conv_fwd_ex" in declared and "maxpool_fwd" in declared
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == declared


def test_out_dims_and_errors():
    assert binding.conv_out_dims(227, 227, 11, 11, 4, 0) == (55, 55)
    assert binding.conv_out_dims(10, 12, 3, 5, 2, 1) == (5, 5)
    lib = binding.lib()
    P, Q = ctypes.c_int(), ctypes.c_int()
    assert lib.conv_out_dims(3, 3, 5, 5, 1, 0, ctypes.byref(P), ctypes.byref(Q)) == -3
    assert lib.conv_out_dims(3, 3, 1, 1, 0, 0, ctypes.byref(P), ctypes.byref(Q)) == -1
    assert lib.conv_out_dims(3, 3, 1, 1, 1, -1, ctypes.byref(P), ctypes.byref(Q)) == -1
    assert lib.conv_out_dims(3, 3, 1, 1, 1, 0, None, None) == -2


def test_conv_fwd_rejects_bad_arguments_without_a_gpu():
    lib = binding.lib()
    fake = ctypes.c_void_p(4096)   # never dereferenced: every call below fails validation
    ok_dims = (1, 3, 8, 8, 4, 3, 3, 1, 1)
    assert lib.conv_fwd(None, fake, fake, fake, *ok_dims, 1) == -2
    assert lib.conv_fwd(fake, None, fake, fake, *ok_dims, 0) == -2
    assert lib.conv_fwd(fake, fake, fake, None, *ok_dims, 0) == -2
    assert lib.conv_fwd(fake, fake, fake, fake, 0, 3, 8, 8, 4, 3, 3, 1, 1, 0) == -1
    assert lib.conv_fwd(fake, fake, fake, fake, 1, 3, 8, 8, 4, 3, 3, 0, 1, 0) == -1
    assert lib.conv_fwd(fake, fake, fake, fake, 1, 3, 8, 8, 4, 3, 3, 1, -1, 0) == -1
    assert lib.conv_fwd(fake, fake, fake, fake, *ok_dims, 2) == -1
    assert lib.conv_fwd(fake, fake, fake, fake, 1, 3, 2, 2, 4, 5, 5, 1, 0, 0) == -3
    nv = binding.conv_num_variants()
    assert lib.conv_fwd_ex(fake, fake, fake, fake, *ok_dims, 0, None, 0, None, nv) == -6
    assert lib.conv_fwd_ex(fake, fake, fake, fake, *ok_dims, 0, None, 0, None, -2) == -6
    assert lib.maxpool_fwd(None, fake, 1, 1, 5, 5, 3, 2, None) == -2
    assert lib.maxpool_fwd(fake, fake, 1, 1, 2, 2, 3, 2, None) == -3
    assert lib.maxpool_fwd(fake, fake, 1, 1, 5, 5, 0, 2, None) == -1
    for st in range(-6, 1):
        assert binding.strerror(st) != "unknown status"
    assert binding.strerror(-99) == "unknown status"


def test_conv_fwd_f16_rejects_bad_arguments_without_a_gpu():
    lib = binding.lib()
    fake = ctypes.c_void_p(4096)   # never dereferenced: every call below fails validation
    odd = ctypes.c_void_p(4097)
    ok_dims = (1, 3, 8, 8, 4, 3, 3, 1, 1)
    assert lib.conv_fwd_f16(None, fake, fake, fake, *ok_dims, 1) == -2
    assert lib.conv_fwd_f16(fake, fake, fake, None, *ok_dims, 0) == -2
    assert lib.conv_fwd_f16(fake, fake, fake, fake, 1, 0, 8, 8, 4, 3, 3, 1, 1, 0) == -1
    assert lib.conv_fwd_f16(fake, fake, fake, fake, *ok_dims, 3) == -1
    assert lib.conv_fwd_f16(fake, fake, fake, fake, 1, 3, 2, 2, 4, 5, 5, 1, 0, 0) == -3
    # half elements need 2-byte aligned tensors
    assert lib.conv_fwd_f16(odd, fake, fake, fake, *ok_dims, 0) == -1
    assert lib.conv_fwd_f16(fake, odd, fake, fake, *ok_dims, 0) == -1
    assert lib.conv_fwd_f16_ex(fake, fake, fake, odd, *ok_dims, 0, None, 0, None, -1) == -1
    nv = binding.conv_num_variants()
    assert lib.conv_fwd_f16_ex(fake, fake, fake, fake, *ok_dims, 0, None, 0, None, nv) == -6


def test_default_workspace_size_covers_every_pointer_alignment():
    """With variant -1 the choice depends on whether the pointers allow the wide loads;
    the size query cannot know and must cover the narrow-load choices too."""
    names = binding.variant_ids_by_name()
    for layer in workloads.ALL_LAYERS:
        dims = (1, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
        chosen = binding.conv_selected_variant(*dims)
        assert binding.conv_fwd_workspace_bytes(*dims, -1) >= binding.conv_fwd_workspace_bytes(*dims, chosen)
    assert names["direct"] == 0


def test_conv_pool_rejects_bad_arguments_and_sizes_its_workspace_without_a_gpu():
    lib = binding.lib()
    fake = ctypes.c_void_p(4096)
    ok = (1, 3, 8, 8, 4, 3, 3, 1, 1)
    assert lib.conv_pool_fwd_ex(None, fake, fake, fake, *ok, 1, 3, 2, fake, 1 << 20, None, -1) == -2
    assert lib.conv_pool_fwd_ex(fake, fake, fake, fake, *ok, 1, 0, 2, fake, 1 << 20, None, -1) == -1
    assert lib.conv_pool_fwd_ex(fake, fake, fake, fake, *ok, 1, 3, -1, fake, 1 << 20, None, -1) == -1
    assert lib.conv_pool_fwd_ex(fake, fake, fake, fake, *ok, 1, 9, 1, fake, 1 << 20, None, -1) == -3
    assert lib.conv_pool_fwd_ex(fake, fake, fake, fake, *ok, 1, 3, 2, fake, 1 << 20, None,
                                binding.conv_num_variants()) == -6
    assert lib.conv_pool_fwd_ex(fake, fake, fake, fake, *ok, 1, 3, 2, None, 0, None, 0) == -4
    names = binding.variant_ids_by_name()
    dims = (1, 256, 13, 13, 384, 3, 3, 1, 1)
    conv_bytes = 384 * 169 * 4
    assert binding.conv_pool_fwd_workspace_bytes(*dims, names["direct"]) == conv_bytes
    assert binding.conv_pool_fwd_workspace_bytes(*dims, names["k3_64x64_k12/s1"]) == conv_bytes
    assert binding.conv_pool_fwd_workspace_bytes(*dims, names["k3_64x64_k12/s4"]) == 4 * conv_bytes
    assert binding.conv_pool_fwd_workspace_bytes(*dims, -1) >= conv_bytes
    assert binding.conv_pool_fwd_workspace_bytes(1, 256, 13, 13, 384, 3, 3, 1, 1, binding.conv_num_variants()) == 0


def test_variant_catalogue():
    nv = binding.conv_num_variants()
    assert nv > 10
    names = [binding.conv_variant_name(v) for v in range(nv)]
    assert names[0] == "direct"
    assert len(set(names)) == nv
    buf = ctypes.create_string_buffer(4)
    assert binding.lib().conv_variant_name(1, buf, 4) == 0 and len(buf.value) == 3
    assert binding.lib().conv_variant_name(nv, buf, 4) == -6


@pytest.mark.parametrize("layer", workloads.ALL_LAYERS, ids=lambda l: l.name)
def test_selection_and_audit_for_benchmark_shapes(layer):
    for N in (1, 5, 32):
        dims = (N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
        v = binding.conv_selected_variant(*dims)
        assert v > 0, "benchmark shapes must get a tiled MFMA variant"
        assert binding.conv_variant_applicable(*dims, v)
        assert binding.bconv_debug_audit(*dims, v) == 0


def test_audit_every_applicable_variant_on_small_batch():
    checked = 0
    for layer in workloads.ALL_LAYERS:
        dims = (2, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad)
        for v in range(1, binding.conv_num_variants()):
            if binding.conv_variant_applicable(*dims, v):
                assert binding.bconv_debug_audit(*dims, v) == 0, binding.conv_variant_name(v)
                checked += 1
    assert checked > 100


def test_workspace_query_matches_split():
    names = binding.variant_ids_by_name()
    dims = (1, 256, 13, 13, 384, 3, 3, 1, 1)
    assert binding.conv_fwd_workspace_bytes(*dims, names["k3_64x64_k12/s1"]) == 0
    assert binding.conv_fwd_workspace_bytes(*dims, names["k3_64x64_k12/s4"]) == 4 * 384 * 169 * 4
    assert binding.conv_fwd_workspace_bytes(*dims, names["direct"]) == 0


def test_sgemm_rejects_bad_arguments_without_a_gpu():
    lib = binding.lib()
    fake = ctypes.c_void_p(4096)   # never dereferenced: every call below fails validation
    assert lib.sgemm(None, fake, fake, 4, 4, 4) == -2
    assert lib.sgemm(fake, fake, None, 4, 4, 4) == -2
    assert lib.sgemm(fake, fake, fake, 0, 4, 4) == -1
    assert lib.sgemm_ex(fake, fake, fake, 4, 4, 4, None, 0, None, binding.conv_num_variants()) == -6
    assert binding.sgemm_workspace_bytes(64, 64, 64, 0) == 0


def test_every_selection_table_row_resolves_to_its_variant():
    """A row whose tile name is missing from the catalogue, or which cannot run its shape,
    would silently fall back to the heuristic: each row must come back as written."""
    path = os.path.join(ROOT, "paper_1606_00094_amd", "csrc", "selection_table.inc")
    rows = re.findall(r'\{(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), "(\w+)", (\d+)\}',
                      open(path).read())
    assert len(rows) >= 44
    for row in rows:
        dims = tuple(int(v) for v in row[:9])
        want = "%s/s%s" % (row[9], row[10])
        assert binding.conv_variant_name(binding.conv_selected_variant(*dims)) == want, (dims, want)


def test_pooled_selection_table_rows_and_fallback():
    """Each row of the convolution + pooling table comes back as written for a 3x3 / step-2
    window and is applicable; any other window, and any shape the table does not list, takes
    the convolution's own choice; the variant -1 workspace query covers both choices."""
    path = os.path.join(ROOT, "paper_1606_00094_amd", "csrc", "pool_selection_table.inc")
    rows = re.findall(r'\{(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), "(\w+)", (\d+)\}',
                      open(path).read())
    assert rows
    for row in rows:
        dims = tuple(int(v) for v in row[:9])
        want = "%s/s%s" % (row[9], row[10])
        v = binding.conv_pool_selected_variant(*dims, 3, 2)
        assert binding.conv_variant_name(v) == want, (dims, want)
        assert binding.conv_variant_applicable(*dims, v)
        own = binding.conv_selected_variant(*dims)
        assert own != v                                   # listed only where it differs
        assert binding.conv_pool_selected_variant(*dims, 2, 2) == own
        need = binding.conv_pool_fwd_workspace_bytes(*dims, -1)
        assert need >= binding.conv_pool_fwd_workspace_bytes(*dims, v)
        assert need >= binding.conv_pool_fwd_workspace_bytes(*dims, own)
    dims = (3, 24, 13, 11, 40, 3, 3, 1, 1)                # not a table shape
    assert binding.conv_pool_selected_variant(*dims, 3, 2) == binding.conv_selected_variant(*dims)
    lib = binding.lib()
    assert lib.conv_pool_selected_variant(*dims, 0, 2) == -1
    assert lib.conv_pool_selected_variant(*dims, 3, 0) == -1
    assert lib.conv_pool_selected_variant(*dims, 14, 1) == -3
    assert lib.conv_pool_selected_variant(1, 0, 13, 11, 40, 3, 3, 1, 1, 3, 2) < 0


def test_batches_beyond_one_launch_are_planned_as_runs_of_images():
    """An input above 2 GiB with more than one image is not a case for the direct kernel:
    the queries describe near-equal runs of whole images, each within one launch's reach."""
    layer = (3, 227, 227, 96, 11, 11, 4, 0)                 # 618 KB per image: 3472 images fit one launch
    one = binding.conv_selected_variant(2000, *layer)
    assert binding.conv_variant_name(one) != "direct"
    assert binding.conv_selected_variant(4000, *layer) == one   # two runs of 2000
    assert binding.conv_variant_applicable(4000, *layer, one) == 1
    assert binding.conv_fwd_workspace_bytes(4000, *layer, -1) == binding.conv_fwd_workspace_bytes(2000, *layer, -1)
    split = binding.variant_ids_by_name()["k11s4_32x128_k2_np/s2"]
    assert binding.conv_fwd_workspace_bytes(4000, *layer, split) == \
        binding.conv_fwd_workspace_bytes(2000, *layer, split) > 0
    # 3473 images: one run of 1737 and one of 1736; the workspace covers the larger
    assert binding.conv_fwd_workspace_bytes(3473, *layer, split) == \
        binding.conv_fwd_workspace_bytes(1737, *layer, split)
    assert binding.conv_pool_fwd_workspace_bytes(3473, *layer, split) == \
        binding.conv_pool_fwd_workspace_bytes(1737, *layer, split)
    # the unpooled output of one run, not of the whole batch
    unsplit = binding.variant_ids_by_name()["k11s4_32x128_k2_np/s1"]
    assert binding.conv_pool_fwd_workspace_bytes(4000, *layer, unsplit) == 2000 * 96 * 55 * 55 * 4
    # one image that is too large by itself: still the direct kernel
    assert binding.conv_variant_name(binding.conv_selected_variant(2, 16, 6000, 6000, 2, 3, 3, 1, 0)) == "direct"
    # small shapes are untouched: an audit over a toy batch counts one launch
    assert binding.bconv_debug_audit(3, 5, 9, 9, 7, 3, 3, 1, 1, binding.conv_selected_variant(3, 5, 9, 9, 7, 3, 3, 1, 1)) == 0


def test_half_precision_selection_on_random_shapes_without_a_gpu():
    """The half-precision queries on seeded random stride-1 shapes: the choice for C8 activations
    is an applicable fp16-matrix-core variant whose estimate is the smallest among the applicable
    ones, its workspace covers the packed filters, and shapes those tiles cannot serve have no
    C8 choice."""
    import numpy as np
    rng = np.random.default_rng(20160601)
    names = {v: binding.conv_variant_name(v) for v in range(binding.conv_num_variants())}
    h16 = [v for v, n in names.items() if n.startswith("h16") and not n.startswith(("h16k11s4", "h16k7s2"))]
    lib = binding.lib()
    checked = 0
    for _ in range(40):
        R = int(rng.choice([1, 3, 5]))
        N, C, K = int(rng.integers(1, 40)), 8 * int(rng.integers(1, 40)), int(rng.integers(1, 300))
        H, W = int(rng.integers(R, 40)), int(rng.integers(R, 40))
        pad = 0 if R == 1 else int(rng.integers(0, R // 2 + 1))
        dims = (N, C, H, W, K, R, R, 1, pad)
        v = binding.conv_fwd_f16_c8_selected_variant(*dims)
        assert v in h16 and binding.conv_fwd_f16_variant_applicable(*dims, v), (dims, names[v])
        costs = {u: binding.bconv_debug_model_cost(*dims, u) for u in h16
                 if binding.conv_fwd_f16_variant_applicable(*dims, u)}
        assert all(c > 0 for c in costs.values())
        assert costs[v] <= min(costs.values()) * (1 + 1e-12) or _listed_c8(dims), (dims, names[v])
        assert binding.conv_fwd_f16_workspace_bytes(*dims, v) >= binding.conv_f16_packed_filter_bytes(*dims, v) > 0
        checked += 1
    assert checked == 40
    assert lib.conv_fwd_f16_c8_selected_variant(2, 12, 9, 9, 8, 3, 3, 1, 1) == -6      # C % 8 != 0
    assert lib.conv_fwd_f16_c8_selected_variant(2, 16, 9, 9, 8, 3, 3, 2, 1) == -6      # stride 2
    assert lib.conv_fwd_f16_c8_selected_variant(2, 16, 9, 9, 8, 7, 7, 1, 3) == -6      # 7x7


def _listed_c8(dims):
    text = open(os.path.join(ROOT, "paper_1606_00094_amd", "csrc", "f16_c8_selection_table.inc")).read()
    return ("{%d, %d, %d, %d, %d, %d, %d, %d, %d," % dims) in text
