"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Every element of the output of every workload is compared with the oracle (its linear nest
over all nonzeros takes seconds to a minute on the host cores); the oracle's result and its
sum of absolute partial products are computed once per workload and shared by the schedules.
"""
import os
import time

import numpy as np
import pytest

from paper_2311_09549_amd import synth

from helpers import TOL, run_library

pytestmark = pytest.mark.gpu

CACHE = os.path.join(os.environ.get("TMPDIR", "/tmp"), "sc_synth_cache")
_data = {}
_ref = {}


def _get(cid):
    if cid not in _data:
        _data.clear()  # keep one large problem in memory at a time
        _ref.clear()
        cfg = synth.config(cid)
        _data[cid] = (cfg, synth.generate(cfg, cache_dir=CACHE))
    return _data[cid]


def _oracle_whole(oracle, cid):
    """The oracle's result and tolerance scale for the whole workload, computed once."""
    if cid not in _ref:
        cfg, data = _get(cid)
        t0 = time.time()
        ref = oracle.contract(cfg["kind"], data["coords"], data["vals"], cfg["dims"], data["factors"])
        bound = oracle.abs_bound(cfg["kind"], data["coords"], data["vals"], cfg["dims"], data["factors"])
        print(f"  oracle over all {cfg['nnz']} nonzeros of config {cid}: {time.time() - t0:.1f} s", flush=True)
        _ref[cid] = (ref, bound)
    return _ref[cid]


def _check_all(oracle, cid, cfg, got):
    """Compare every output element with the oracle; returns (rows checked, worst scaled error)."""
    ref, bound = _oracle_whole(oracle, cid)
    assert got.shape == ref.shape
    err = np.abs(got.astype(np.float64) - ref)
    tol = TOL[cfg["dtype"]]
    worst = float((err / np.maximum(bound, 1e-300)).max())
    assert np.all(err <= tol * bound), f"max scaled error {worst:.3e} > {tol}"
    return ref.shape[0], worst


VARIANTS = [("fused", False), ("fissioned", False), ("linear", False), ("fused", True), ("fissioned", True)]


@pytest.mark.parametrize("which,det", VARIANTS, ids=[w + ("-deterministic" if d else "") for w, d in VARIANTS])
@pytest.mark.parametrize("cid", [2, 3, 4, 5])
def test_parity_full(oracle, cid, which, det):
    """All schedules of one workload run one after the other, so that its inputs are generated and
    its oracle result is computed once.  Deterministic schedules also have to reproduce their first
    execution bit for bit (the heaviest slices span thousands of tiles)."""
    from paper_2311_09549_amd import binding as sc
    from paper_2311_09549_amd.driver import Contraction

    cfg, data = _get(cid)
    print(f"config {cid} full size {which}{' deterministic' if det else ''} nnz={cfg['nnz']}", flush=True)
    if det:
        con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                          sc.schedule(which, deterministic=True), synth.output_shape(cfg))
        con.run()
        got = con.result().copy()
        con.out.fill_(float("nan"))
        con.run()
        assert con.result().tobytes() == got.tobytes()
    else:
        con, got = run_library(cfg, data, which)
    assert not np.isnan(got).any()
    nrows, worst = _check_all(oracle, cid, cfg, got)
    assert nrows == cfg["dims"][0]
    print(f"  rows checked {nrows}, max scaled error {worst:.3e}, workspace {con.ws_bytes} bytes", flush=True)
    # empty slices give exactly +0 rows
    empty = np.ones(cfg["dims"][0], dtype=bool)
    empty[np.unique(data["coords"][0])] = False
    z = got[empty]
    assert np.all(z == 0) and not np.signbit(z).any()
    del con
