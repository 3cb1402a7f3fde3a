"""The temporaries a FISSIONED plan leaves in the workspace, checked on their own against the
oracle's named intermediates (Section 4.2): one row per CSF node in node order, the values of
T(i,j,m) / T(i,j,r) / T1(i,j,k,n), T2(i,j,m,n) and of the sampled matrix T(i,j).  Rows of fibers
that span several tiles are the ones combined by atomics or, under a deterministic schedule, by the
fix-up kernels."""
import numpy as np
import pytest

from paper_2311_09549_amd import binding as sc
from paper_2311_09549_amd import synth
from paper_2311_09549_amd.driver import Contraction

from helpers import TOL
from test_gpu_parity_edges import _case

pytestmark = pytest.mark.gpu


def _check(got, ref, bound, dtype, what):
    assert got.shape == ref.shape, what
    assert not np.isnan(got).any(), what
    err = np.abs(got.astype(np.float64) - ref)
    worst = float((err / np.maximum(bound, 1e-300)).max()) if ref.size else 0.0
    assert np.all(err <= TOL[dtype] * bound), f"{what}: max scaled error {worst:.3e}"


def _check_all(oracle, cfg, data, con):
    coords, vals, dims, fac = data["coords"], data["vals"], cfg["dims"], data["factors"]
    absf = [np.abs(f) for f in fac]
    kind, dtype = cfg["kind"], cfg["dtype"]
    if kind in ("ttmc3", "mttkrp3"):
        _, ref = oracle.intermediate_leaf(coords, vals, dims, fac[1])
        _, bnd = oracle.intermediate_leaf(coords, np.abs(vals), dims, absf[1])
        _check(con.intermediate(0), ref, bnd, dtype, "T")
    elif kind == "ttmc4":
        _, ref = oracle.intermediate_leaf(coords, vals, dims, fac[2])
        _, bnd = oracle.intermediate_leaf(coords, np.abs(vals), dims, absf[2])
        _check(con.intermediate(0), ref, bnd, dtype, "T1")
        _, ref = oracle.intermediate_t2_order4(coords, vals, dims, fac[1], fac[2])
        _, bnd = oracle.intermediate_t2_order4(coords, np.abs(vals), dims, absf[1], absf[2])
        _check(con.intermediate(1), ref.reshape(ref.shape[0], -1), bnd.reshape(ref.shape[0], -1), dtype, "T2")
    else:
        ref = oracle.intermediate_sampled(coords, vals, fac[0], fac[1])
        bnd = oracle.intermediate_sampled(coords, np.abs(vals), absf[0], absf[1])
        _check(con.intermediate(0).reshape(-1), ref, bnd, dtype, "sampled values")


@pytest.mark.parametrize("det", [False, True])
@pytest.mark.parametrize("cid,scale", [(1, 1.0), (2, 0.004), (3, 0.003), (4, 0.003), (5, 0.004)])
def test_fissioned_temporaries_small(oracle, cid, scale, det):
    cfg = synth.config(cid, scale)
    data = synth.generate(cfg)
    print(f"config {cid} scale {scale} fissioned det={det}: temporaries", flush=True)
    con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                      sc.schedule("fissioned", deterministic=det), synth.output_shape(cfg))
    con.workspace.view(np_dtype_view(cfg)).fill_(float("nan"))
    con.run()
    _check_all(oracle, cfg, data, con)


def np_dtype_view(cfg):
    import torch
    return torch.float64 if cfg["dtype"] == "f64" else torch.float32


@pytest.mark.parametrize("det", [False, True])
@pytest.mark.parametrize("name", ["one_slice", "one_fiber", "unit_fibers", "count_1025"])
@pytest.mark.parametrize("kind", ["mttkrp3", "ttmc3", "sddmm_spmm", "ttmc4"])
def test_fissioned_temporaries_degenerate(oracle, kind, name, det):
    cfg, data = _case(kind, name)
    print(f"{kind} {name} fissioned det={det}: temporaries", flush=True)
    con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                      sc.schedule("fissioned", deterministic=det), synth.output_shape(cfg))
    con.run()
    _check_all(oracle, cfg, data, con)
