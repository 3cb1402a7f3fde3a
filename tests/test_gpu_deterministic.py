"""GPU checks of the deterministic schedules: the result meets the same parity bar as the
atomic schedules, two executions of one plan and two plans of one problem give bit-identical
outputs, and rows that span many tiles (one heavy slice) are summed correctly."""
import numpy as np
import pytest

from paper_2311_09549_amd import binding as sc
from paper_2311_09549_amd import synth
from paper_2311_09549_amd.driver import Contraction

from helpers import assert_parity
from test_gpu_parity_edges import _case

pytestmark = pytest.mark.gpu


def _run_twice(cfg, data, which="fused"):
    outs = []
    for _ in range(2):   # two plans, two executions each
        con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"],
                          sc.schedule(which, deterministic=True), synth.output_shape(cfg))
        con.run()
        outs.append(con.result().copy())
        con.out.fill_(float("nan"))
        con.run()
        outs.append(con.result().copy())
    return outs


@pytest.mark.parametrize("cid,scale,which", [(1, 1.0, "fused"), (1, 1.0, "fissioned"), (2, 0.004, "fissioned"), (2, 0.02, "fissioned"),
                                             (3, 0.003, "fissioned"), (3, 0.01, "fissioned"), (2, 0.004, "fused"), (2, 0.02, "fused"), (3, 0.003, "fused"), (3, 0.01, "fused"),
                                             (4, 0.003, "fused"), (4, 0.01, "fissioned"), (5, 0.004, "fused"), (5, 0.004, "fissioned"), (5, 0.02, "fissioned")])
def test_deterministic_parity_and_repeatability(oracle, cid, scale, which):
    cfg = synth.config(cid, scale)
    data = synth.generate(cfg)
    print(f"config {cid} scale {scale} {which} deterministic nnz={cfg['nnz']}", flush=True)
    outs = _run_twice(cfg, data, which)
    assert_parity(oracle, cfg, data, outs[0])
    for o in outs[1:]:
        assert o.tobytes() == outs[0].tobytes()


@pytest.mark.parametrize("name", ["one_slice", "one_fiber", "count_3072", "single"])
@pytest.mark.parametrize("kind,which", [("mttkrp3", "fused"), ("mttkrp3", "fissioned"), ("ttmc3", "fused"), ("ttmc3", "fissioned"),
                                        ("sddmm_spmm", "fused"), ("sddmm_spmm", "fissioned"), ("ttmc4", "fused"), ("ttmc4", "fissioned")])
def test_deterministic_degenerate_structures(oracle, kind, which, name):
    cfg, data = _case(kind, name)
    print(f"{kind} {name} {which} deterministic dims={cfg['dims']} nnz={cfg['nnz']}", flush=True)
    outs = _run_twice(cfg, data, which)
    assert_parity(oracle, cfg, data, outs[0])
    for o in outs[1:]:
        assert o.tobytes() == outs[0].tobytes()


@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("dtype,ranks", [("f32", (8, 32)), ("f32", (32, 8)), ("f64", (16, 16)), ("f64", (4, 64))])
def test_deterministic_general_outer_product_kernel(oracle, dtype, ranks, which):
    """The order-3 chain at ranks / precisions the matrix-core kernel does not cover."""
    cfg = dict(synth.config(3, 0.003), dtype=dtype, ranks=ranks)
    data = synth.generate(cfg)
    print(f"order-3 chain {dtype} ranks {ranks} {which} deterministic nnz={cfg['nnz']}", flush=True)
    outs = _run_twice(cfg, data, which)
    assert_parity(oracle, cfg, data, outs[0])
    for o in outs[1:]:
        assert o.tobytes() == outs[0].tobytes()
