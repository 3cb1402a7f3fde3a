"""GPU parity of the HIP path against the fp64 oracle on shrunken versions of the five
workloads (sizes the oracle finishes in seconds, several tiles, ragged tails)."""
import numpy as np
import pytest

from paper_2311_09549_amd import binding as sc
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


@pytest.mark.gpu
def test_stream_copy_copies():
    """The calibration copy kernel moves exactly the bytes it is given (ragged grid tail included)."""
    import torch
    n = 16 * (256 * 8192 + 37)
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros_like(src)
    sc.stream_copy(dst, src, n, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


@pytest.mark.parametrize("per_cu", [1, 3, 64])
@pytest.mark.parametrize("cid,scale", [(3, 0.003), (5, 0.004)])
def test_parity_any_run_length(oracle, cid, scale, per_cu):
    """The persistent fused kernels carry slice sums across the tiles of a run; the result must
    not depend on how the tiles are cut into runs (long runs, and one tile per run)."""
    sc.tuning_set("persistent_per_cu", per_cu)
    sc.tuning_set("tile_leaves", 128)   # many tiles per slice
    try:
        cfg = synth.config(cid, scale)
        data = synth.generate(cfg)
        print(f"config {cid} scale {scale} fused, {per_cu} workgroups per CU", flush=True)
        con, got = run_library(cfg, data, "fused")
        assert_parity(oracle, cfg, data, got)
    finally:
        sc.tuning_set("persistent_per_cu", 0)
        sc.tuning_set("tile_leaves", 0)


@pytest.mark.gpu
@pytest.mark.parametrize("det", [False, True])
@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("cid,scale", [(1, 1.0), (2, 0.002), (3, 0.002), (4, 0.002), (5, 0.002)])
def test_parity_with_small_ragged_tiles(oracle, cid, scale, which, det):
    """Tile caps far below the built-in ones and not multiples of anything the kernels use: nearly
    every tile then cuts a node at every level of the tree, under both schedules, with atomic and
    with deterministic combination of the pieces."""
    knobs = {"tile_leaves": 96, "tile_nodes_a": 24, "tile_nodes_b": 6}
    for k, v in knobs.items():
        sc.tuning_set(k, v)
    try:
        cfg = synth.config(cid, scale)
        data = synth.generate(cfg)
        print(f"config {cid} scale {scale} {which} det={det} small tiles nnz={cfg['nnz']}", flush=True)
        from paper_2311_09549_amd.driver import Contraction
        con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                          sc.schedule(which, deterministic=det), synth.output_shape(cfg))
        assert sc.plan_tile_count(con.plan) >= cfg["nnz"] // 96
        con.run()
        got = con.result().copy()
        assert_parity(oracle, cfg, data, got)
        if det:
            con.out.fill_(float("nan"))
            con.run()
            assert con.result().tobytes() == got.tobytes()
    finally:
        for k in knobs:
            sc.tuning_set(k, 0)


@pytest.mark.gpu
def test_library_loaded_before_torch_touches_the_gpu():
    """A fresh process that calls the library before torch has initialised the GPU must still find
    the device afterwards (both bind to the one HIP runtime that torch ships)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("from paper_2311_09549_amd import binding as sc\n"
            "sc.tuning_set('tile_leaves', 0)\n"
            "import torch\n"
            "assert torch.cuda.is_available()\n"
            "x = torch.ones(4, device='cuda:0')\n"
            "assert float(x.sum()) == 4.0\n"
            "print('ok')\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "ok" in r.stdout, r.stdout + r.stderr
