"""GPU parity of the LINEAR schedule (the unfactored nest run as it stands) against the oracle,
which computes the same nest in fp64: shrunken workloads and the degenerate structures."""
import numpy as np
import pytest

from paper_2311_09549_amd import synth

from helpers import assert_parity, run_library
from test_gpu_parity_edges import KINDS, _case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid,scale", [(1, 1.0), (2, 0.004), (3, 0.003), (4, 0.003), (5, 0.004)])
def test_parity_linear_small(oracle, cid, scale):
    cfg = synth.config(cid, scale)
    data = synth.generate(cfg)
    print(f"config {cid} scale {scale} linear nnz={cfg['nnz']}", flush=True)
    con, got = run_library(cfg, data, "linear")
    assert got.shape == tuple(synth.output_shape(cfg))
    assert_parity(oracle, cfg, data, got)


@pytest.mark.parametrize("name", ["empty", "single", "one_slice", "one_fiber", "unit_fibers", "count_1025", "corners"])
@pytest.mark.parametrize("kind", list(KINDS))
def test_parity_linear_degenerate_structure(oracle, kind, name):
    cfg, data = _case(kind, name)
    print(f"{kind} {name} linear dims={cfg['dims']} nnz={cfg['nnz']}", flush=True)
    con, got = run_library(cfg, data, "linear")
    if cfg["nnz"] == 0:
        assert np.all(got == 0) and not np.signbit(got).any()
        return
    assert_parity(oracle, cfg, data, got)


@pytest.mark.parametrize("dtype,ranks", [("f64", (8, 8)), ("f32", (12, 20)), ("f32", (4, 12))])
def test_parity_linear_any_rank(oracle, dtype, ranks):
    """The unfactored nest has no kernel per rank: ranks no fused kernel is instantiated for run too."""
    cfg = dict(synth.config(3, 0.002), dtype=dtype, ranks=ranks)
    data = synth.generate(cfg)
    print(f"order-3 chain {dtype} ranks {ranks} linear nnz={cfg['nnz']}", flush=True)
    con, got = run_library(cfg, data, "linear")
    assert_parity(oracle, cfg, data, got)
