"""GPU parity of the trailing-GEMM kernels of Table 2 -- kernel 8 <MTTKRP,GEMM> and kernel 2
<SDDMM,SpMM,GEMM> -- against the oracle's perfectly nested loops: every schedule class of the sparse
part (fused, fissioned, unfactored, picked by the cost evaluator), atomic and deterministic, both
precisions, ranks on and off the matrix-core tile, the row temporary left in the workspace, and the
two full-size workloads bench.py times."""
import os

import numpy as np
import pytest

from paper_2311_09549_amd import binding as sc
from paper_2311_09549_amd import synth
from paper_2311_09549_amd.driver import Contraction

from helpers import TOL, assert_parity

pytestmark = pytest.mark.gpu

CACHE = os.path.join(os.environ.get("TMPDIR", "/tmp"), "sc_synth_cache")


def _run(cfg, data, which, det=False):
    con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                      sc.schedule(which, deterministic=det), synth.output_shape(cfg))
    con.run()
    return con, con.result()


@pytest.mark.parametrize("which", ["fused", "fissioned", "linear", "auto"])
@pytest.mark.parametrize("cid,scale,dtype,ranks", [
    (7, 0.003, "f32", (32, 64)), (7, 0.003, "f32", (16, 16)), (7, 0.003, "f32", (64, 20)), (7, 0.003, "f64", (32, 16)),
    (7, 0.003, "f32", (128, 128)), (7, 0.0005, "f32", (8, 4)),
    (8, 0.002, "f32", (64, 64, 64)), (8, 0.002, "f32", (16, 16, 32)), (8, 0.002, "f32", (32, 32, 12)), (8, 0.002, "f64", (16, 16, 16)),
])
def test_parity_trailing_gemm(oracle, cid, scale, dtype, ranks, which):
    cfg = dict(synth.config(cid, scale), dtype=dtype, ranks=ranks)
    data = synth.generate(cfg)
    print(f"{cfg['kind']} {which} {dtype} ranks={ranks} dims={cfg['dims']} nnz={cfg['nnz']}", flush=True)
    con, got = _run(cfg, data, which)
    print("  " + sc.plan_describe(con.plan).splitlines()[1], flush=True)
    assert_parity(oracle, cfg, data, got)


@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("cid,scale", [(7, 0.01), (8, 0.005)])
def test_deterministic_is_bit_reproducible(oracle, cid, scale, which):
    cfg = synth.config(cid, scale)
    data = synth.generate(cfg)
    con, first = _run(cfg, data, which, det=True)
    first = first.copy()
    con.out.fill_(float("nan"))
    con.run()
    assert con.result().tobytes() == first.tobytes()
    assert_parity(oracle, cfg, data, first)


def test_row_temporary_in_the_workspace(oracle):
    """T2(i,r): the MTTKRP rows, alone against the oracle's MTTKRP (the producer of kernel 8)."""
    cfg = synth.config(7, 0.005)
    data = synth.generate(cfg)
    con, _ = _run(cfg, data, "fused")
    rows = con.intermediate(1).astype(np.float64)
    C, D, E = data["factors"]
    ref = oracle.contract("mttkrp3", data["coords"], data["vals"], cfg["dims"], [C, D])
    bound = oracle.abs_bound("mttkrp3", data["coords"], data["vals"], cfg["dims"], [C, D])
    assert rows.shape == ref.shape
    assert np.all(np.abs(rows - ref) <= TOL["f32"] * bound)


@pytest.mark.parametrize("which", ["fused", "fissioned", "linear"])
def test_parity_full_size_kernel8(oracle, which):
    """The tensor of workload 2 (20 M nonzeros), R = 32, M = 64: every element against the perfectly nested loop."""
    cfg = synth.config(7)
    data = synth.generate(cfg, cache_dir=CACHE)
    me = test_parity_full_size_kernel8
    if not hasattr(me, "ref"):
        me.ref = (oracle.contract(cfg["kind"], data["coords"], data["vals"], cfg["dims"], data["factors"]),
                  oracle.abs_bound(cfg["kind"], data["coords"], data["vals"], cfg["dims"], data["factors"]))
    ref, bound = me.ref
    con, got = _run(cfg, data, which)
    assert not np.isnan(got).any()
    err = np.abs(got.astype(np.float64) - ref)
    print(f"kernel 8 full size {which}: rows checked {ref.shape[0]}, max scaled error {float((err / np.maximum(bound, 1e-300)).max()):.3e}", flush=True)
    assert np.all(err <= TOL["f32"] * bound)
    empty = np.ones(cfg["dims"][0], dtype=bool)
    empty[np.unique(data["coords"][0])] = False
    assert np.all(got[empty] == 0) and not np.signbit(got[empty]).any()


@pytest.mark.parametrize("which", ["fused", "fissioned"])
def test_parity_full_size_kernel2(oracle, which):
    """The matrix of workload 4 (16 M entries), K = L = M = 64.  The perfectly nested loop of kernel 2 has K L M =
    262,144 iterations per stored entry (4 * 10^12 in all), so the whole output is compared with the oracle's kernel 1
    times the last factor (numpy matmul in fp64; the pins show the two agree), and the rows of a random sample of
    slices with the perfectly nested loop itself."""
    cfg = synth.config(8)
    data = synth.generate(cfg, cache_dir=CACHE)
    X, Y, Z, F = data["factors"]
    me = test_parity_full_size_kernel2
    if not hasattr(me, "ref"):
        p = oracle.contract("sddmm_spmm", data["coords"], data["vals"], cfg["dims"], [X, Y, Z])
        pb = oracle.abs_bound("sddmm_spmm", data["coords"], data["vals"], cfg["dims"], [X, Y, Z])
        me.ref = (p @ F.astype(np.float64), pb @ np.abs(F.astype(np.float64)))
    ref, bound = me.ref
    con, got = _run(cfg, data, which)
    assert not np.isnan(got).any()
    err = np.abs(got.astype(np.float64) - ref)
    print(f"kernel 2 full size {which}: rows checked {ref.shape[0]}, max scaled error {float((err / np.maximum(bound, 1e-300)).max()):.3e}", flush=True)
    assert np.all(err <= TOL["f32"] * bound)
    # a sample of ordinary slices against the perfectly nested loop (an output row depends on its slice only)
    counts = np.bincount(data["coords"][0], minlength=cfg["dims"][0])
    rng = np.random.default_rng(5)
    rows = rng.choice(np.flatnonzero((counts > 0) & (counts <= 64)), size=300, replace=False)
    keep = np.isin(data["coords"][0], rows)
    sub = [c[keep] for c in data["coords"]]
    r2 = oracle.contract(cfg["kind"], sub, data["vals"][keep], cfg["dims"], data["factors"])[rows]
    b2 = oracle.abs_bound(cfg["kind"], sub, data["vals"][keep], cfg["dims"], data["factors"])[rows]
    assert np.all(np.abs(got[rows].astype(np.float64) - r2) <= TOL["f32"] * b2)
