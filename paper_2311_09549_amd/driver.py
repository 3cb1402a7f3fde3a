"""Convenience wrapper used by the tests, the smoke check and the benchmark: uploads a
problem with PyTorch (device memory and streams only), plans it and queues executions.
No arithmetic happens here."""
from __future__ import annotations

import numpy as np

from . import binding as sc


class Contraction:
    """One planned contraction resident on the GPU."""

    def __init__(self, expr, coords, vals, dims, factors, sched, out_shape, device="cuda:0", share=None):
        """`share`: another Contraction of the same problem whose converted CSF arrays and device
        copies of the operands are reused (a second schedule of one problem)."""
        import torch
        self.torch = torch
        self.device = torch.device(device)
        if share is not None:
            self.host_csf, self.csf, self.factors = share.host_csf, share.csf, share.factors
            self.plan = sc.plan_create(expr, self.host_csf, [np.ascontiguousarray(f) for f in factors], sched)
        else:
            self.host_csf = sc.coo_to_csf(list(coords), vals, dims)
            self.plan = sc.plan_create(expr, self.host_csf, [np.ascontiguousarray(f) for f in factors], sched)
            self.csf = self.host_csf.to_device(self.device)
            self.factors = [torch.from_numpy(np.ascontiguousarray(f)).to(self.device) for f in factors]
        tdt = torch.float64 if np.asarray(vals).dtype == np.float64 else torch.float32
        # NaN-filled so that any element the library fails to write is caught
        self.out = torch.full(tuple(int(s) for s in out_shape), float("nan"), dtype=tdt, device=self.device)
        self.ws_bytes = sc.plan_workspace_bytes(self.plan)
        self.workspace = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=self.device)
        assert self.workspace.data_ptr() % 256 == 0

    def run(self, stream=None):
        s = stream if stream is not None else self.torch.cuda.current_stream(self.device).cuda_stream
        sc.execute(self.plan, self.csf, self.factors, self.out, self.workspace, self.ws_bytes, s)

    def result(self) -> np.ndarray:
        self.torch.cuda.synchronize(self.device)
        return self.out.cpu().numpy()

    def intermediate(self, index: int) -> np.ndarray:
        """FISSIONED only: the temporary as left in the workspace by the last run."""
        off, rows, cols = sc.plan_intermediate(self.plan, index)
        self.torch.cuda.synchronize(self.device)
        esz = self.out.element_size()
        raw = self.workspace[off: off + rows * cols * esz].cpu().numpy()
        return raw.view(np.float64 if esz == 8 else np.float32).reshape(rows, cols)
