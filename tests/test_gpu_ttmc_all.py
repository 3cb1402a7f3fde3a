"""GPU parity of the all-mode TTMC (Table 2, kernel 5) under the three schedules Table 2 lists for
it, against the oracle's perfectly nested loop: every schedule class the library offers for each,
atomic and deterministic, both precisions, several dense sizes; the temporaries a FISSIONED
execution leaves in the workspace against the oracle's named intermediates; and one workload of the
first dense sizes of the paper's auxiliary-memory table (L = M = N = 16) at full size."""
import os

import numpy as np
import pytest

from paper_2311_09549_amd import binding as sc
from paper_2311_09549_amd import synth
from paper_2311_09549_amd.driver import Contraction

from helpers import TOL, assert_parity

pytestmark = pytest.mark.gpu

# (schedule class, named temporaries): schedule 2 (default), 2, 1, 3 of Table 2
VARIANTS = [("fused", ()), ("fissioned", ("T1(i,j,n)", "T2(i,m,n)")), ("fissioned", ("T(i,j,n)",)), ("fused", ("T(i,m,n)",)), ("linear", ())]
IDS = ["schedule2-fused", "schedule2-fissioned", "schedule1", "schedule3", "linear"]


def _contraction(cfg, data, which, names, det=False):
    return Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                       sc.schedule(which, list(names), [0] * len(names), deterministic=det), synth.output_shape(cfg))


def _cfg(scale, dtype="f32", ranks=(16, 16, 16), seed_offset=0):
    cfg = dict(synth.config(6, scale), dtype=dtype, ranks=ranks, seed_offset=seed_offset)
    return cfg, synth.generate(cfg)


@pytest.mark.parametrize("which,names", VARIANTS, ids=IDS)
@pytest.mark.parametrize("scale", [0.002, 0.02])
@pytest.mark.parametrize("dtype,ranks", [("f32", (16, 16, 16)), ("f64", (16, 16, 16)), ("f32", (8, 16, 8)), ("f32", (32, 4, 32)),
                                         ("f64", (4, 8, 8)), ("f32", (64, 16, 16)), ("f32", (128, 32, 32)), ("f32", (16, 128, 128)),
                                         ("f32", (64, 64, 64))])
def test_parity_three_schedules(oracle, dtype, ranks, scale, which, names):
    cfg, data = _cfg(scale, dtype, ranks)
    print(f"ttmc_all {which} {names} {dtype} ranks={ranks} dims={cfg['dims']} nnz={cfg['nnz']}", flush=True)
    con = _contraction(cfg, data, which, names)
    print(sc.plan_describe(con.plan).splitlines()[1], flush=True)
    con.run()
    assert_parity(oracle, cfg, data, con.result())


@pytest.mark.parametrize("which,names", VARIANTS[:3], ids=IDS[:3])
def test_deterministic_is_bit_reproducible(oracle, which, names):
    cfg, data = _cfg(0.02)
    con = _contraction(cfg, data, which, names, det=True)
    con.run()
    first = con.result().copy()
    con.out.fill_(float("nan"))
    con.run()
    assert con.result().tobytes() == first.tobytes()
    assert_parity(oracle, cfg, data, first)


def test_schedule3_cannot_be_deterministic():
    cfg, data = _cfg(0.002)
    with pytest.raises(sc.ScError, match="SC_ERR_SCHED_UNSUPPORTED"):
        _contraction(cfg, data, "fused", ("T(i,m,n)",), det=True)


def test_temporaries_left_in_the_workspace(oracle):
    """t(i,j,n) per fiber and the per-slice tiles T2(i,m,n), alone against the oracle's intermediates."""
    cfg, data = _cfg(0.01)
    C, D, E = data["factors"]
    bound_t = oracle.intermediate_leaf(data["coords"], np.abs(data["vals"]), cfg["dims"], np.abs(E))[1]
    pre, t_ref = oracle.intermediate_leaf(data["coords"], data["vals"], cfg["dims"], E)
    spre, s_ref = oracle.intermediate_slice_ttmc_all(data["coords"], data["vals"], cfg["dims"], D, E)
    s_bound = oracle.intermediate_slice_ttmc_all(data["coords"], np.abs(data["vals"]), cfg["dims"], np.abs(D), np.abs(E))[1]
    for which, names in VARIANTS[:3]:
        con = _contraction(cfg, data, which, names)
        con.run()
        con.result()
        if which == "fissioned":
            t = con.intermediate(0).astype(np.float64)
            assert t.shape == t_ref.shape
            assert np.all(np.abs(t - t_ref) <= TOL["f32"] * bound_t), names
        if len(names) != 1:   # schedule 2: the tiles of every coordinate of the first mode, empty slices as +0 rows
            s = con.intermediate(1).astype(np.float64).reshape(cfg["dims"][0], 16, 16)
            assert np.all(np.abs(s[spre[0]] - s_ref) <= TOL["f32"] * s_bound)
            empty = np.ones(cfg["dims"][0], dtype=bool)
            empty[spre[0]] = False
            assert np.all(s[empty] == 0)


@pytest.mark.parametrize("which,names", VARIANTS, ids=IDS)
def test_parity_full_size(oracle, which, names):
    """40,000 x 20,000 x 8,000, 4 M Zipf(1.1) nonzeros, L = M = N = 16: every element against the oracle."""
    cfg = synth.config(6)
    data = synth.generate(cfg, cache_dir=os.path.join(os.environ.get("TMPDIR", "/tmp"), "sc_synth_cache"))
    if not hasattr(test_parity_full_size, "ref"):
        test_parity_full_size.ref = (oracle.contract(cfg["kind"], data["coords"], data["vals"], cfg["dims"], data["factors"]),
                                     oracle.abs_bound(cfg["kind"], data["coords"], data["vals"], cfg["dims"], data["factors"]))
    ref, bound = test_parity_full_size.ref
    con = _contraction(cfg, data, which, names)
    con.run()
    got = con.result().astype(np.float64)
    assert not np.isnan(got).any()
    err = np.abs(got - ref)
    worst = float((err / bound).max())
    print(f"ttmc_all full size {which} {names}: max scaled error {worst:.3e}, workspace {con.ws_bytes} bytes", flush=True)
    assert np.all(err <= TOL["f32"] * bound)


@pytest.mark.parametrize("cid", [9, 10])
def test_uniform_motivating_cases_on_sampled_outputs(oracle, cid):
    """Cases 1 and 2 of Section 3 (uniform 1800 x 800 x 1000 at sparsity 0.008 and 1800 x 1600 x 2000 at 0.002,
    L, M, N = 64, 16, 32; 11.5 M nonzeros each).  The perfectly nested loop over the whole output would take
    3.8 * 10^11 iterations, so the oracle is run on sampled outputs: an element A(l,m,n) depends on column l of C,
    m of D and n of E only, hence 4 x 4 x 4 sampled columns form an exact sub-problem.  All three schedules."""
    cfg = synth.config(cid)
    data = synth.generate(cfg, cache_dir=os.path.join(os.environ.get("TMPDIR", "/tmp"), "sc_synth_cache"))
    C, D, E = data["factors"]
    rng = np.random.default_rng(cid)
    ls, ms, ns = (np.sort(rng.choice(f.shape[1], 4, replace=False)) for f in (C, D, E))
    sub = [np.ascontiguousarray(C[:, ls]), np.ascontiguousarray(D[:, ms]), np.ascontiguousarray(E[:, ns])]
    ref = oracle.contract("ttmc_all", data["coords"], data["vals"], cfg["dims"], sub)
    bound = oracle.abs_bound("ttmc_all", data["coords"], data["vals"], cfg["dims"], sub)
    first = None
    for (which, names), label in zip(VARIANTS, IDS):
        con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                          sc.schedule(which, list(names), [0] * len(names)), synth.output_shape(cfg), share=first)
        first = first or con
        con.run()
        got = con.result().astype(np.float64)
        assert not np.isnan(got).any()
        pick = got[np.ix_(ls, ms, ns)]
        worst = float((np.abs(pick - ref) / bound).max())
        print(f"uniform case {cid - 8} {label}: 64 sampled outputs, max scaled error {worst:.3e}", flush=True)
        assert np.all(np.abs(pick - ref) <= TOL["f32"] * bound)
        # schedules agree with one another over the whole output (each within its own bound of the exact result)
        if con is not first:
            full_bound_proxy = np.abs(got).max()
            assert np.all(np.abs(got - first.result().astype(np.float64)) <= 1e-4 * full_bound_proxy)
