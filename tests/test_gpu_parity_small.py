"""GPU parity of the HIP path against the fp64 oracle on shrunken versions of the five
workloads (sizes the oracle finishes in seconds, several tiles, ragged tails)."""
import numpy as np
import pytest

from paper_2311_09549_amd import synth

from helpers import assert_parity, run_library

pytestmark = pytest.mark.gpu

SMALL = [(1, 1.0), (2, 0.004), (3, 0.003), (4, 0.003), (5, 0.004)]


@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("cid,scale", SMALL)
def test_parity_small(oracle, cid, scale, which):
    cfg = synth.config(cid, scale)
    data = synth.generate(cfg)
    print(f"config {cid} scale {scale} {which} nnz={cfg['nnz']}", flush=True)
    con, got = run_library(cfg, data, which)
    worst = assert_parity(oracle, cfg, data, got)
    print(f"  max scaled error {worst:.3e}", flush=True)
