"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle is evaluated on the whole problem where that takes seconds (MTTKRP, SDDMM->SpMM)
and on a sample of top-level slices otherwise (every output row depends on its own slice
only, so a row subset is an exact sub-problem): the heaviest slices, which are the ones
split across many work tiles, plus a random sample of ordinary ones.
"""
import os

import numpy as np
import pytest

from paper_2311_09549_amd import synth

from helpers import TOL, run_library

pytestmark = pytest.mark.gpu

CACHE = os.path.join(os.environ.get("TMPDIR", "/tmp"), "sc_synth_cache")
_data = {}


def _get(cid):
    if cid not in _data:
        _data.clear()  # keep one large problem in memory at a time
        cfg = synth.config(cid)
        _data[cid] = (cfg, synth.generate(cfg, cache_dir=CACHE))
    return _data[cid]


def _check_rows(oracle, cfg, data, got, rows):
    """Compare output rows `rows` with the oracle run on the nonzeros of those slices."""
    coords, vals = data["coords"], data["vals"]
    keep = np.isin(coords[0], rows)
    sub = [c[keep] for c in coords]
    ref = oracle.contract(cfg["kind"], sub, vals[keep], cfg["dims"], data["factors"])[rows]
    bound = oracle.abs_bound(cfg["kind"], sub, vals[keep], cfg["dims"], data["factors"])[rows]
    err = np.abs(got[rows].astype(np.float64) - ref)
    tol = TOL[cfg["dtype"]]
    worst = float((err / np.maximum(bound, 1e-300)).max())
    assert np.all(err <= tol * bound), f"max scaled error {worst:.3e} > {tol}"
    return worst


def _sample_rows(data, dims0, n_heavy, n_random, seed):
    counts = np.bincount(data["coords"][0], minlength=dims0)
    heavy = np.argsort(counts)[::-1][:n_heavy]
    rng = np.random.default_rng(seed)
    rest = rng.choice(dims0, size=n_random, replace=False)
    return np.unique(np.concatenate([heavy, rest]))


@pytest.mark.parametrize("which", ["fused", "fissioned", "linear"])
@pytest.mark.parametrize("cid,n_heavy,n_random", [(2, None, None), (3, 40, 3000), (4, None, None), (5, 10, 500)])
def test_parity_full(oracle, cid, n_heavy, n_random, which):
    cfg, data = _get(cid)
    print(f"config {cid} full size {which} nnz={cfg['nnz']}", flush=True)
    con, got = run_library(cfg, data, which)
    assert not np.isnan(got).any()
    dims0 = cfg["dims"][0]
    rows = np.arange(dims0) if n_heavy is None else _sample_rows(data, dims0, n_heavy, n_random, 77)
    worst = _check_rows(oracle, cfg, data, got, rows)
    print(f"  rows checked {rows.size}, max scaled error {worst:.3e}", flush=True)
    # empty slices give exactly +0 rows
    empty = np.ones(dims0, dtype=bool)
    empty[np.unique(data["coords"][0])] = False
    z = got[empty]
    assert np.all(z == 0) and not np.signbit(z).any()
    del con


@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("cid,n_heavy,n_random", [(2, None, None), (3, 40, 3000), (4, None, None), (5, 10, 500)])
def test_parity_full_deterministic(oracle, cid, n_heavy, n_random, which):
    """The deterministic schedules at full size: same bar, and a second execution of the plan
    reproduces the first bit for bit (the heaviest slices span thousands of tiles)."""
    from paper_2311_09549_amd import binding as sc
    from paper_2311_09549_amd.driver import Contraction

    cfg, data = _get(cid)
    print(f"config {cid} full size {which} deterministic nnz={cfg['nnz']}", flush=True)
    con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                      sc.schedule(which, deterministic=True), synth.output_shape(cfg))
    con.run()
    got = con.result().copy()
    con.out.fill_(float("nan"))
    con.run()
    again = con.result()
    assert not np.isnan(got).any()
    assert again.tobytes() == got.tobytes()
    dims0 = cfg["dims"][0]
    rows = np.arange(dims0) if n_heavy is None else _sample_rows(data, dims0, n_heavy, n_random, 77)
    worst = _check_rows(oracle, cfg, data, got, rows)
    print(f"  rows checked {rows.size}, max scaled error {worst:.3e}, workspace {con.ws_bytes} bytes", flush=True)
    del con
