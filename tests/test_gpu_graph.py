"""An execution is only kernel launches on the caller's stream (no allocation, no
synchronisation, no memset nodes), so it can be captured into a HIP graph.  Every replay is
checked: against the oracle for the atomic schedules, bit for bit against the eager result for
the deterministic ones, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2311_09549_amd import binding as sc
from paper_2311_09549_amd import synth
from paper_2311_09549_amd.driver import Contraction

from helpers import assert_parity, default_schedule

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid,scale,which,det", [(2, 0.01, "fused", False), (2, 0.01, "fused", True), (2, 0.01, "fissioned", False),
                                                 (3, 0.005, "fused", True), (4, 0.005, "fissioned", True), (5, 0.004, "fused", False)])
def test_captured_execution_replays_correctly(oracle, cid, scale, which, det):
    import torch

    cfg = synth.config(cid, scale)
    data = synth.generate(cfg)
    sched = sc.schedule(which, deterministic=True) if det else default_schedule(cfg["kind"], which)
    con = Contraction(cfg["expr"], data["coords"], data["vals"], cfg["dims"], data["factors"], sched, synth.output_shape(cfg))
    con.run()
    eager = con.result().copy()
    assert_parity(oracle, cfg, data, eager)

    side = torch.cuda.Stream()   # default priority
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        con.run(stream=torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        con.out.fill_(float("nan"))          # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = con.out.cpu().numpy()
        print(f"config {cid} {which} det={det} replay {rep}", flush=True)
        if det:
            assert got.tobytes() == eager.tobytes()
        else:
            assert_parity(oracle, cfg, data, got)
