import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a gfx950 GPU and the built HIP library")


@pytest.fixture(params=["big", "wide"])
def gemm_tile(request, monkeypatch):
    """Runs a GEMM test once per workgroup tile of the MFMA kernel (256 x 256 and 256 x 128): the library reads
    SNIP_GEMM_TILE at every GEMM call, so both tiles see every shape, whatever the launcher would pick itself."""
    monkeypatch.setenv("SNIP_GEMM_TILE", request.param)
    return request.param


@pytest.fixture(params=["wave", "workgroup"])
def quant_both_unit(request, monkeypatch):
    """Runs a test of the one-pass two-orientation quantize once per work distribution (a wave or a workgroup per
    128-column unit): the library reads SNIP_QUANT_BOTH_UNIT at every call."""
    monkeypatch.setenv("SNIP_QUANT_BOTH_UNIT", request.param)
    return request.param


@pytest.fixture(params=["wave", "workgroup"])
def quant_col_unit(request, monkeypatch):
    """Runs a test of the column-block quantize once per work distribution (a wave or a workgroup per 128-column
    unit): the library reads SNIP_QUANT_COL_UNIT at every call."""
    monkeypatch.setenv("SNIP_QUANT_COL_UNIT", request.param)
    return request.param
