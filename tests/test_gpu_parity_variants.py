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
