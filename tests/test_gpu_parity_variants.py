"""GPU parity on rank / dtype variants of the small workloads, so that every kernel family is
exercised: the generic order-3 and order-4 kernels (fp64, ranks the matrix-core kernels do not
cover), MTTKRP at every supported rank, SDDMM->SpMM at other widths."""
import pytest

from paper_2311_09549_amd import synth

from helpers import assert_parity, run_library

pytestmark = pytest.mark.gpu

VARIANTS = [
    # (config id, scale, dtype, ranks)
    (2, 0.003, "f32", (8,)), (2, 0.003, "f32", (16,)), (2, 0.003, "f32", (64,)), (2, 0.003, "f64", (32,)), (2, 0.003, "f64", (8,)),
    (3, 0.002, "f32", (8, 16)), (3, 0.002, "f32", (16, 32)), (3, 0.002, "f32", (4, 8)), (3, 0.002, "f64", (16, 16)),
    (4, 0.002, "f32", (32, 32)), (4, 0.002, "f32", (16, 16)), (4, 0.002, "f64", (64, 64)),
    (5, 0.003, "f32", (16, 8, 8)), (5, 0.003, "f32", (4, 8, 8)), (5, 0.003, "f64", (8, 8, 8)),
    # the widest ranks: 128-wide rows of the temporaries (order 3), 16 x 16 tiles of the second temporary (order 4)
    (2, 0.003, "f32", (128,)), (2, 0.003, "f64", (128,)), (3, 0.002, "f32", (128, 128)), (3, 0.002, "f32", (16, 128)),
    (3, 0.002, "f32", (128, 16)), (3, 0.002, "f64", (64, 128)), (5, 0.003, "f32", (16, 16, 16)), (5, 0.003, "f32", (8, 16, 16)),
]


@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("cid,scale,dtype,ranks", VARIANTS)
def test_parity_variant(oracle, cid, scale, dtype, ranks, which):
    cfg = synth.config(cid, scale)
    cfg["dtype"] = dtype
    cfg["ranks"] = ranks
    data = synth.generate(cfg)
    print(f"config {cid} scale {scale} {dtype} ranks {ranks} {which}", flush=True)
    con, got = run_library(cfg, data, which)
    assert_parity(oracle, cfg, data, got)


@pytest.mark.parametrize("cid,scale", [(1, 1.0), (2, 0.003), (3, 0.002), (4, 0.002), (5, 0.003), (6, 0.01)])
def test_parity_schedule_picked_by_the_cost_evaluator(oracle, cid, scale):
    """SC_SCHED_AUTO plans execute like the class they settle on."""
    from paper_2311_09549_amd import binding as sc
    from paper_2311_09549_amd.driver import Contraction

    cfg = synth.config(cid, scale)
    data = synth.generate(cfg)
    con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"], sc.schedule("auto"),
                      synth.output_shape(cfg))
    print(f"config {cid}: evaluator chose {sc.plan_chosen(con.plan)}", flush=True)
    con.run()
    assert_parity(oracle, cfg, data, con.result())
    if cid == 3:   # ranks only the unfactored nest takes: the evaluator falls back to it
        import numpy as np
        cfg = dict(cfg, ranks=(12, 20))
        data = synth.generate(cfg)
        con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"], sc.schedule("auto"),
                          synth.output_shape(cfg))
        assert sc.plan_chosen(con.plan) == ("linear", 0)
        con.run()
        assert_parity(oracle, cfg, data, con.result())


@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("ranks", [(16, 32), (64, 64), (128, 16)])
def test_parity_wide_ranks_with_padded_leading_dimension(oracle, ranks, which):
    """The matrix-core kernel for rank pairs beyond 16 x 16 with factor rows longer than the rank (ld > cols): the padding
    holds NaN, so a read outside the first `cols` elements of a row, or a row offset taken from cols instead of ld, shows."""
    import torch
    from paper_2311_09549_amd import binding as sc
    from paper_2311_09549_amd.driver import Contraction

    cfg = dict(synth.config(3, 0.002), ranks=ranks)
    data = synth.generate(cfg)
    con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"], sc.schedule(which),
                      synth.output_shape(cfg))
    padded = []
    for n, f in enumerate(con.factors):
        big = torch.full((f.shape[0], f.shape[1] + 4 * (n + 1)), float("nan"), dtype=f.dtype, device=f.device)
        big[:, : f.shape[1]] = f
        padded.append(big[:, : f.shape[1]])
        assert sc.dense_view(padded[-1]).ld == f.shape[1] + 4 * (n + 1)
    con.factors = padded
    con.run()
    assert_parity(oracle, cfg, data, con.result())
