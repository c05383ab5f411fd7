"""The FLOP / byte accounting used for the roofline report reproduces the
figures the paper prints (SGEMM tables, Section V formula, Section III worked
example)."""
import os

import pytest

from paper_1606_00094_amd import roofline

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows():
    rows = []
    with open(os.path.join(GOLDEN, "sgemm_tables.txt")) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([float(t) for t in line.split()])
    return rows


@pytest.mark.parametrize("row", _rows())
def test_sgemm_table_columns(row):
    size, nbytes, flops, ai = row
    n = int(size)
    # printed with three significant digits
    assert roofline.sgemm_bytes(n, n, n) == pytest.approx(nbytes, rel=6e-3)
    assert roofline.sgemm_flops(n, n, n) == pytest.approx(flops, rel=6e-3)
    assert roofline.sgemm_ai(n, n, n) == pytest.approx(ai, rel=6e-3)


def _kv():
    out = {}
    with open(os.path.join(GOLDEN, "worked_example.txt")) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def test_worked_example_bytes_and_macs():
    g = _kv()
    args = (1, 3, 205, 205, 96, 7, 7, 2, 0)
    o, i, f = roofline.im2col_gemm_bytes(*args)
    assert o / 1e6 == pytest.approx(g["outmat_MB"], abs=0.005)
    assert i / 1e6 == pytest.approx(g["inmat_MB"], abs=0.005)
    assert f / 1e6 == pytest.approx(g["filtsmat_MB"], abs=0.005)
    assert (o + i + f) / 1e6 == pytest.approx(g["total_MB"], abs=0.01)
    macs = roofline.conv_flops(*args, flops_per_mac=1)
    assert macs == 10000 * 96 * 147
    assert macs / 1e6 == pytest.approx(g["macs_M"], abs=0.5)
    assert macs / (o + i + f) == pytest.approx(g["ai_one_flop_per_mac"], abs=0.05)
    # two flops per MAC, the convention of the SGEMM tables
    assert roofline.conv_flops(*args) == 2 * macs


def test_layer_table_figures():
    # first layer: 96 x 3025 x 363 GEMM -> 210.8 MFLOP, bytes 4*(in+filt+bias+out)
    assert roofline.conv_flops(1, 3, 227, 227, 96, 11, 11, 4, 0) == 2 * 96 * 3025 * 363
    assert roofline.conv_bytes(1, 3, 227, 227, 96, 11, 11, 4, 0) == \
        4 * (3 * 227 * 227 + 96 * 363 + 96 + 96 * 3025)
    mf, hb = roofline.roof_min_seconds(157.3e12, 8e12)
    assert mf == pytest.approx(1.0) and hb == pytest.approx(1.0)
