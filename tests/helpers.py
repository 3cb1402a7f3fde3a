"""Shared pieces of the GPU parity tests."""
import numpy as np

from paper_2311_09549_amd import binding as sc
from paper_2311_09549_amd import synth
from paper_2311_09549_amd.driver import Contraction

TOL = {"f32": 1e-5, "f64": 1e-12}   # |gpu - oracle| <= TOL * sum|partial products|


def default_schedule(kind, which):
    names = {"ttmc3": ["T(i,j,m)"], "mttkrp3": ["T(i,j,r)"], "sddmm_spmm": ["T(i,j)"],
             "ttmc4": ["T1(i,j,k,n)", "T2(i,j,m,n)"], "ttmc_all": ["T1(i,j,n)", "T2(i,m,n)"],
             "mttkrp_gemm": ["T1(i,j,r)", "T2(i,r)"], "sddmm_spmm_gemm": ["T1(i,j)", "T2(i,l)"]}[kind]
    if which == "linear":
        return sc.schedule("linear")
    if which == "fused":
        return sc.schedule("fused", names, [0] * len(names))
    return sc.schedule("fissioned", names, [0] * len(names))


def run_library(cfg, data, which):
    con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                      default_schedule(cfg["kind"], which), synth.output_shape(cfg))
    con.run()
    return con, con.result()


def assert_parity(oracle, cfg, data, got, rows=None):
    """Element-wise check against the oracle, scaled by the sum of |partial products|."""
    kind, dims = cfg["kind"], cfg["dims"]
    ref = oracle.contract(kind, data["coords"], data["vals"], dims, data["factors"])
    bound = oracle.abs_bound(kind, data["coords"], data["vals"], dims, data["factors"])
    assert got.shape == ref.shape
    assert not np.isnan(got).any(), "output has elements the library never wrote"
    tol = TOL[cfg["dtype"]]
    err = np.abs(got.astype(np.float64) - ref)
    worst = float((err / np.maximum(bound, 1e-300)).max()) if bound.size else 0.0
    assert np.all(err <= tol * bound), f"max scaled error {worst:.3e} > {tol}"
    if kind == "ttmc_all":   # the output has no sparse index: no rows of empty slices
        return worst
    # rows of empty slices: exactly +0
    empty = np.ones(dims[0], dtype=bool)
    empty[np.unique(data["coords"][0])] = False
    z = got[empty]
    assert np.all(z == 0) and not np.signbit(z).any()
    return worst
