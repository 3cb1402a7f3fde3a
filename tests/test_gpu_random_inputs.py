"""GPU parity on seeded random valid inputs: random shapes, entry counts (empty to tens of
thousands), uniform or heavily skewed coordinates, supported ranks and precisions, all three
schedule classes, atomic and deterministic combination, and random tile caps (so that tiles cut
the tree in ever different places).  Every case is checked element-wise against the oracle; a
combination the library documents as unavailable must be refused at plan creation, never run."""
import numpy as np
import pytest

from paper_2311_09549_amd import binding as sc
from paper_2311_09549_amd import synth
from paper_2311_09549_amd.driver import Contraction

from helpers import assert_parity

pytestmark = pytest.mark.gpu

KIND_CFG = {"mttkrp3": 2, "ttmc3": 3, "sddmm_spmm": 4, "ttmc4": 5}
RANKS = {"mttkrp3": [(8,), (16,), (32,), (64,)], "ttmc3": [(16, 16), (8, 16), (4, 32), (16, 8), (32, 64), (16, 32), (64, 16), (128, 32)],
         "sddmm_spmm": [(16, 16), (32, 32), (64, 64), (128, 128)], "ttmc4": [(8, 8, 8), (4, 8, 8), (16, 8, 8), (12, 8, 8)]}
KNOBS = ("tile_leaves", "tile_nodes_a", "tile_nodes_b")


def _random_case(seed):
    rng = np.random.default_rng([4242, seed])
    kind = list(KIND_CFG)[rng.integers(0, 4)]
    base = synth.config(KIND_CFG[kind], 0.001)
    order = len(base["dims"])
    dims = tuple(int(x) for x in rng.integers(3, 300, order))
    if kind == "sddmm_spmm":
        dims = (max(dims), max(dims))
    total = int(np.prod([float(d) for d in dims]))
    nnz = int(min(rng.integers(0, 30000), total // 2))
    style = int(rng.integers(0, 3))
    if nnz:
        if style == 0:   # uniform
            flat = rng.choice(total, nnz, replace=False) if total < 5_000_000 else np.unique(rng.integers(0, total, nnz))
            cols = list(np.unravel_index(np.sort(flat), dims))
        else:            # a few heavy slices and fibers
            cols = [np.minimum(rng.pareto(1.0 if style == 1 else 0.5, nnz).astype(np.int64), d - 1) for d in dims]
            cols[-1] = rng.integers(0, dims[-1], nnz)
            key = np.zeros(nnz, np.int64)
            for c, d in zip(cols, dims):
                key = key * d + c
            _, first = np.unique(key, return_index=True)
            cols = [c[first] for c in cols]
        coords = [np.ascontiguousarray(c.astype(np.int32)) for c in cols]
    else:
        coords = [np.zeros(0, np.int32) for _ in range(order)]
    nnz = len(coords[0])
    dtype = "f64" if rng.integers(0, 4) == 0 else "f32"
    which = ["fused", "fissioned", "linear"][rng.integers(0, 3)]
    ranks = RANKS[kind][rng.integers(0, len(RANKS[kind]))]
    if which == "linear" and kind != "sddmm_spmm":
        ranks = tuple(int(4 * rng.integers(1, 9)) for _ in ranks)   # the unfactored nest takes any rank (rows of 16 bytes)
    det = bool(rng.integers(0, 2)) and which != "linear"
    cfg = dict(base, dims=dims, nnz=nnz, dtype=dtype, ranks=ranks)
    dt = np.float64 if dtype == "f64" else np.float32
    vals = rng.uniform(-1, 1, nnz).astype(dt)
    factors = [rng.standard_normal(s).astype(dt) for s in synth.factor_shapes(cfg)]
    caps = (int(rng.integers(32, 1025)), int(rng.integers(8, 300)), int(rng.integers(2, 80))) if rng.integers(0, 3) else (0, 0, 0)
    return cfg, dict(cfg=cfg, coords=coords, vals=vals, factors=factors), which, det, caps


@pytest.mark.parametrize("first", [0, 40, 80, 120, 160, 200])
def test_parity_random_valid_inputs(oracle, first):
    ran = 0
    for seed in range(first, first + 40):
        cfg, data, which, det, caps = _random_case(seed)
        print(f"case {seed}: {cfg['kind']} {which} det={det} {cfg['dtype']} ranks={cfg['ranks']} dims={cfg['dims']} nnz={cfg['nnz']} caps={caps}",
              flush=True)
        for k, v in zip(KNOBS, caps):
            sc.tuning_set(k, v)
        try:
            try:
                con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                                  sc.schedule(which, deterministic=det), synth.output_shape(cfg))
            except sc.ScError as ex:
                assert "SC_ERR_SCHED_UNSUPPORTED" in str(ex), ex   # caps no kernel takes, or fp64 order 4 deterministic
                continue
            con.out.fill_(float("nan"))
            con.run()
            got = con.result().copy()
            # the first failing case ends the loop: nothing more runs on the GPU after a mismatch
            if cfg["nnz"] == 0:
                assert np.all(got == 0), f"case {seed}"
            else:
                assert_parity(oracle, cfg, data, got)
            if det:
                con.out.fill_(float("nan"))
                con.run()
                assert con.result().tobytes() == got.tobytes(), f"case {seed}: second execution differs"
            ran += 1
            del con
        finally:
            for k in KNOBS:
                sc.tuning_set(k, 0)
    assert ran >= 30


# ---- kernels 5, 8 and 2 of Table 2: the all-mode TTMC under its schedules, the trailing dense products ----
NEXT_KIND_CFG = {"ttmc_all": 6, "mttkrp_gemm": 7, "sddmm_spmm_gemm": 8}
K5_SCHEDULES = [("fused", ()), ("fissioned", ("T1(i,j,n)", "T2(i,m,n)")), ("fissioned", ("T(i,j,n)",)), ("fused", ("T(i,m,n)",)), ("linear", ())]


def _random_next_case(seed):
    rng = np.random.default_rng([777, seed])
    kind = list(NEXT_KIND_CFG)[rng.integers(0, 3)]
    base = synth.config(NEXT_KIND_CFG[kind], 0.001)
    order = len(base["dims"])
    dims = tuple(int(x) for x in rng.integers(3, 200, order))
    if order == 2:
        dims = (max(dims), max(dims))
    total = int(np.prod([float(d) for d in dims]))
    nnz = int(min(rng.integers(1, 20000), total // 2))
    if rng.integers(0, 2):
        flat = np.unique(rng.integers(0, total, nnz))
    else:   # most entries in the leading slices
        flat = np.unique((rng.pareto(0.7, nnz) * 50).astype(np.int64) % total)
    coords = [np.ascontiguousarray(c.astype(np.int32)) for c in np.unravel_index(np.sort(flat), dims)]
    nnz = len(coords[0])
    dtype = "f64" if rng.integers(0, 5) == 0 else "f32"
    if kind == "ttmc_all":
        ranks = (int(rng.choice([8, 16, 32, 64, 128])), int(rng.choice([8, 16, 32, 64])), int(rng.choice([8, 16, 32, 64])))
        which, names = K5_SCHEDULES[rng.integers(0, 5)]
    elif kind == "mttkrp_gemm":
        ranks = (int(rng.choice([8, 16, 32, 64])), int(rng.choice([8, 16, 24, 64, 128])))
        which, names = ["fused", "fissioned", "linear"][rng.integers(0, 3)], ()
    else:
        r = int(rng.choice([16, 32, 64]))
        ranks = (r, r, int(rng.choice([8, 16, 48, 64])))
        which, names = ["fused", "fissioned", "linear"][rng.integers(0, 3)], ()
    det = bool(rng.integers(0, 2)) and which != "linear" and names != ("T(i,m,n)",)
    cfg = dict(base, dims=dims, nnz=nnz, dtype=dtype, ranks=ranks)
    dt = np.float64 if dtype == "f64" else np.float32
    data = dict(cfg=cfg, coords=coords, vals=rng.uniform(-1, 1, nnz).astype(dt),
                factors=[rng.standard_normal(s).astype(dt) for s in synth.factor_shapes(cfg)])
    return cfg, data, which, names, det


@pytest.mark.parametrize("first", [0, 50, 100])
def test_parity_random_valid_inputs_of_the_composed_kernels(oracle, first):
    ran = 0
    for seed in range(first, first + 50):
        cfg, data, which, names, det = _random_next_case(seed)
        print(f"case {seed}: {cfg['kind']} {which} {names} det={det} {cfg['dtype']} ranks={cfg['ranks']} dims={cfg['dims']} nnz={cfg['nnz']}", flush=True)
        try:
            con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                              sc.schedule(which, list(names), [0] * len(names), deterministic=det), synth.output_shape(cfg))
        except sc.ScError as ex:
            assert "SC_ERR_SCHED_UNSUPPORTED" in str(ex), ex
            continue
        con.out.fill_(float("nan"))
        con.run()
        got = con.result().copy()
        assert_parity(oracle, cfg, data, got)   # the first failing case ends the loop
        if det:
            con.out.fill_(float("nan"))
            con.run()
            assert con.result().tobytes() == got.tobytes(), f"case {seed}: second execution differs"
        ran += 1
        del con
    assert ran >= 40
