"""GPU parity on the degenerate structures of the method: nothing stored, a single entry, all
entries in one slice / one fiber (a node cut by many tiles at every level), fibers of one entry
only, entry counts that land exactly on, just below and just above tile multiples, stored zeros,
coordinates at both ends of every mode.  Both schedules, all seven nests, element-wise against the
oracle (same bar as the other parity tests)."""
import numpy as np
import pytest

from paper_2311_09549_amd import synth

from helpers import assert_parity, run_library

pytestmark = pytest.mark.gpu

KINDS = {"mttkrp3": 2, "ttmc3": 3, "sddmm_spmm": 4, "ttmc4": 5, "ttmc_all": 6, "mttkrp_gemm": 7, "sddmm_spmm_gemm": 8}   # kind -> workload whose expression and ranks it borrows


def _sorted_unique(cols, dims):
    key = np.zeros(len(cols[0]), dtype=np.int64)
    for c, d in zip(cols, dims):
        key = key * d + c
    _, first = np.unique(key, return_index=True)   # sorted by the lexicographic key
    return [np.ascontiguousarray(c[first].astype(np.int32)) for c in cols]


def _structure(name, order, rng):
    """dims and sorted distinct coordinates of one degenerate structure."""
    if name == "empty":
        dims = (7, 9, 11, 5)[:order]
        return dims, [np.zeros(0, np.int32) for _ in range(order)]
    if name == "single":
        dims = (7, 9, 11, 5)[:order]
        return dims, [np.array([d - 1], np.int32) for d in dims]
    if name == "one_slice":            # every entry in slice i = 3: the slice is cut by many tiles
        dims = (6, 90, 80, 12)[:order] if order > 2 else (6, 40000)
        n = 6000
        cols = [np.full(n, 3)] + [rng.integers(0, d, n) for d in dims[1:]]
        return dims, _sorted_unique(cols, dims)
    if name == "one_fiber":            # every entry in one leaf fiber: cut by many tiles at every level
        dims = (5, 6, 7, 6000)[4 - order:] if order > 2 else (5, 6000)
        n = 5000
        lead = [np.full(n, d // 2) for d in dims[:-1]]
        cols = lead + [rng.permutation(dims[-1])[:n]]
        return dims, _sorted_unique(cols, dims)
    if name == "unit_fibers":          # every leaf fiber holds one entry
        dims = (40, 50, 60, 30)[:order] if order > 2 else (2500, 60)
        n = 1800
        lead = rng.permutation(int(np.prod(dims[:-1])))[:n]
        cols = list(np.unravel_index(lead, dims[:-1])) + [rng.integers(0, dims[-1], n)]
        return dims, _sorted_unique(cols, dims)
    if name.startswith("count_"):      # entry counts around multiples of the tile sizes
        n = int(name.split("_")[1])
        dims = (30, 40, 50, 20)[:order] if order > 2 else (300, 400)
        flat = rng.permutation(int(np.prod(dims)))[:n]
        return dims, _sorted_unique(list(np.unravel_index(flat, dims)), dims)
    if name == "corners":              # first and last coordinate of every mode, nothing in between
        dims = (9, 8, 7, 6)[:order]
        grids = np.meshgrid(*[np.array([0, d - 1]) for d in dims], indexing="ij")
        return dims, _sorted_unique([g.ravel() for g in grids], dims)
    raise ValueError(name)


def _case(kind, name, zeros=False):
    base = synth.config(KINDS[kind], 0.001)
    order = len(base["dims"])
    rng = np.random.default_rng([77, KINDS[kind], sum(map(ord, name))])
    dims, coords = _structure(name, order, rng)
    if kind in ("sddmm_spmm", "sddmm_spmm_gemm"):
        dims = (max(dims), max(dims))      # X is indexed by i, Y and Z by j: one square shape keeps it simple
    cfg = dict(base, dims=tuple(int(d) for d in dims), nnz=len(coords[0]))
    dt = np.float32 if cfg["dtype"] == "f32" else np.float64
    vals = rng.uniform(-1, 1, len(coords[0])).astype(dt)
    if zeros and len(vals):
        vals[:: 3] = 0                      # stored zeros are ordinary entries
    factors = [rng.standard_normal(shape).astype(dt) for shape in synth.factor_shapes(cfg)]
    return cfg, dict(cfg=cfg, coords=coords, vals=vals, factors=factors)


STRUCTURES = ["empty", "single", "one_slice", "one_fiber", "unit_fibers", "count_1023", "count_1024", "count_1025",
              "count_3072", "corners"]


@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("name", STRUCTURES)
@pytest.mark.parametrize("kind", list(KINDS))
def test_parity_degenerate_structure(oracle, kind, name, which):
    cfg, data = _case(kind, name)
    print(f"{kind} {name} {which} dims={cfg['dims']} nnz={cfg['nnz']}", flush=True)
    con, got = run_library(cfg, data, which)
    assert got.shape == tuple(synth.output_shape(cfg))
    if cfg["nnz"] == 0:
        assert np.all(got == 0) and not np.signbit(got).any()
        return
    assert_parity(oracle, cfg, data, got)


@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("kind", list(KINDS))
def test_parity_stored_zeros(oracle, kind, which):
    cfg, data = _case(kind, "count_3072", zeros=True)
    print(f"{kind} stored zeros {which} nnz={cfg['nnz']}", flush=True)
    con, got = run_library(cfg, data, which)
    assert_parity(oracle, cfg, data, got)


@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("kind", list(KINDS))
def test_parity_padded_leading_dimension(oracle, kind, which):
    """Factor rows longer than the rank (ld > cols): the padding holds NaN, so any read outside the
    first `cols` elements of a row shows up in the result."""
    import torch
    from paper_2311_09549_amd import binding as sc
    from paper_2311_09549_amd.driver import Contraction
    from helpers import default_schedule

    cfg, data = _case(kind, "count_3072")
    print(f"{kind} ld > cols {which} nnz={cfg['nnz']}", flush=True)
    con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                      default_schedule(cfg["kind"], which), synth.output_shape(cfg))
    padded = []
    for n, f in enumerate(con.factors):
        big = torch.full((f.shape[0], f.shape[1] + 4 * (n + 1)), float("nan"), dtype=f.dtype, device=f.device)
        big[:, : f.shape[1]] = f
        padded.append(big[:, : f.shape[1]])
        assert sc.dense_view(padded[-1]).ld == f.shape[1] + 4 * (n + 1)
    con.factors = padded
    con.run()
    assert_parity(oracle, cfg, data, con.result())


@pytest.mark.parametrize("kind", list(KINDS))
def test_parity_on_a_side_stream(oracle, kind):
    """All launches of an execution go to the caller's stream: queued behind a long fill on a side
    stream, the result is complete once that stream (and only that stream) has been waited for."""
    import torch
    from paper_2311_09549_amd.driver import Contraction
    from helpers import default_schedule

    cfg, data = _case(kind, "count_3072")
    con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                      default_schedule(cfg["kind"], "fissioned"), synth.output_shape(cfg))
    torch.cuda.synchronize()
    side = torch.cuda.Stream()   # default priority
    with torch.cuda.stream(side):
        ballast = torch.empty(64 << 20, dtype=torch.float32, device="cuda:0")
        for _ in range(4):
            ballast.fill_(1.0)   # keeps the side stream busy ahead of the library's kernels
        con.run(stream=side.cuda_stream)
    side.synchronize()
    got = con.out.cpu().numpy()
    assert_parity(oracle, cfg, data, got)
