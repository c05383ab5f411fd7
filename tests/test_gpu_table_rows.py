"""Every row of the selection tables on the GPU, through variant -1.

A row names the tile and reduction split measured best for one exact (layer, batch) shape.
For each row the library must (a) pick exactly that variant when asked to choose and
(b) give the oracle's result, every image element by element, within
|gpu - oracle| <= max(1e-5, 1e-4 * |oracle|).  Rows of the pooled table go through the
convolution + pooling call and are compared with the oracle's convolution followed by its
pooling.  The square matrix-product rows (one "image" whose pixels are the columns) are the
shapes of test_sgemm_table_sizes and are compared here as layers as well.
"""
import os
import re

import numpy as np
import pytest
import torch

import oracle
import workloads
from paper_1606_00094_amd import binding
from tests.test_gpu_parity import assert_close, gpu_conv, gpu_conv_pool
from tests.test_gpu_parity_f16 import assert_close_f16, gpu_conv_f16

pytestmark = pytest.mark.gpu

CSRC = os.path.join(os.path.dirname(os.path.abspath(binding.__file__)), "csrc")
ROW = re.compile(r'^\{(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), "([^"]+)", (\d+)\}')


def table_rows(fname):
    rows = []
    with open(os.path.join(CSRC, fname)) as fh:
        for line in fh:
            m = ROW.match(line)
            if m:
                rows.append(tuple(int(g) for g in m.groups()[:9]) + (m.group(10), int(m.group(11))))
    assert rows, fname
    return rows


def _row_id(row):
    return "N%d_C%d_%dx%d_K%d_%dx%d_s%d_p%d" % row[:9]


def _layer_of(dims):
    """The benchmark layer (or matrix-product shape) a row was swept on, for its value
    distributions; a row of any other shape is drawn like a middle layer."""
    for l in workloads.ALL_LAYERS + workloads.SGEMM_LAYERS:
        if (l.C, l.H, l.W, l.K, l.R, l.S, l.stride, l.pad) == dims[1:]:
            return l
    return workloads.Layer("row", *dims[1:], "u01", "n001", "u01b")


@pytest.mark.parametrize("row", table_rows("selection_table.inc"), ids=_row_id)
def test_selection_table_row(row):
    dims, tile, nsplit = row[:9], row[9], row[10]
    N, C, H, W, K, R, S, stride, pad = dims
    chosen = binding.conv_variant_name(binding.conv_selected_variant(*dims))
    assert chosen == "%s/s%d" % (tile, nsplit), "variant -1 resolves to %s" % chosen
    layer = _layer_of(dims)
    x, f, b = workloads.make_layer_inputs(layer, N, seed=workloads.BASE_SEED + 300000 + sum(dims))
    ref = oracle.conv_fwd(x, f, b, stride=stride, pad=pad, relu=True)
    got = gpu_conv(x, f, b, stride, pad, True)
    assert_close(got, ref, "%s via %s" % (_row_id(row), chosen))


@pytest.mark.parametrize("row", table_rows("pool_selection_table.inc"), ids=_row_id)
def test_pool_selection_table_row(row):
    dims, tile, nsplit = row[:9], row[9], row[10]
    N, C, H, W, K, R, S, stride, pad = dims
    chosen = binding.conv_variant_name(binding.conv_pool_selected_variant(*dims, 3, 2))
    assert chosen == "%s/s%d" % (tile, nsplit), "variant -1 resolves to %s" % chosen
    layer = _layer_of(dims)
    x, f, b = workloads.make_layer_inputs(layer, N, seed=workloads.BASE_SEED + 400000 + sum(dims))
    ref = oracle.maxpool_fwd(oracle.conv_fwd(x, f, b, stride=stride, pad=pad, relu=True), 3, 2)
    got = gpu_conv_pool(x, f, b, stride, pad, True, 3, 2)
    assert_close(got, ref, "%s + pool via %s" % (_row_id(row), chosen))


@pytest.mark.parametrize("row", table_rows("f16_selection_table.inc"), ids=_row_id)
def test_f16_selection_table_row(row):
    """Rows of the half-precision table (tiles on the fp16 matrix cores): the half-precision
    entry point picks the row's tile and gives the correctly rounded exact result to within one
    fp16 spacing, every image."""
    dims, tile, nsplit = row[:9], row[9], row[10]
    N, C, H, W, K, R, S, stride, pad = dims
    chosen = binding.conv_variant_name(binding.conv_fwd_f16_selected_variant(*dims))
    assert chosen == "%s/s%d" % (tile, nsplit), "variant -1 resolves to %s" % chosen
    layer = _layer_of(dims)
    x, f, b = workloads.make_layer_inputs(layer, N, seed=workloads.BASE_SEED + 500000 + sum(dims))
    x, f = x.astype(np.float16), f.astype(np.float16)
    ref = oracle.conv_fwd_f16(x, f, b, stride=stride, pad=pad, relu=True)
    got = gpu_conv_f16(x, f, b, stride, pad, True)
    assert_close_f16(got, ref, "%s via %s" % (_row_id(row), chosen))


@pytest.mark.parametrize("row", table_rows("f16_c8_selection_table.inc"), ids=_row_id)
def test_f16_c8_selection_table_row(row):
    """Rows of the table for octet-interleaved activations: the query returns the row's tile, and
    that tile on C8 input (C8 output where K allows) gives the oracle's values, every image."""
    from tests.test_gpu_parity_f16_c8 import gpu_conv_c8
    dims, tile, nsplit = row[:9], row[9], row[10]
    N, C, H, W, K, R, S, stride, pad = dims
    v = binding.conv_fwd_f16_c8_selected_variant(*dims)
    assert binding.conv_variant_name(v) == "%s/s%d" % (tile, nsplit)
    layer = _layer_of(dims)
    x, f, b = workloads.make_layer_inputs(layer, N, seed=workloads.BASE_SEED + 700000 + sum(dims))
    x, f = x.astype(np.float16), f.astype(np.float16)
    ref = oracle.conv_fwd_f16(x, f, b, stride=stride, pad=pad, relu=True)
    got = gpu_conv_c8(x, f, b, stride, pad, True, v, K % 8 == 0)
    assert_close_f16(got, ref, "%s via %s on C8" % (_row_id(row), tile))


def test_rows_cover_the_batch_points():
    """The tables list the ten benchmark layers and the toy layer at every batch size the
    benchmark, the stack sweep and the paper's batch points (1, 5, 20) use."""
    have = {r[:9] for r in table_rows("selection_table.inc")}
    for l in workloads.ALL_LAYERS:
        for N in (1, 2, 4, 5, 8, 16, 20, 32, 64, 128, 256):
            assert (N, l.C, l.H, l.W, l.K, l.R, l.S, l.stride, l.pad) in have, (l.name, N)
    torch.cuda.synchronize()
