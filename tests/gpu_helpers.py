"""Helpers for the GPU parity tests: run a layer table through the C ABI and through the oracle."""
import numpy as np
import torch

import paper_2504_08795_amd as D
import workloads as wl
from oracle import forward as F

TOL = {"fp32": 1e-3, "bf16": 2e-2}     # spec tolerances on whole-network logits


def rel_err(got, want):
    """(max-norm relative error, L2 relative error); element-wise ratios are not used because logits cross zero."""
    got = np.asarray(got, np.float64).reshape(-1)
    want = np.asarray(want, np.float64).reshape(-1)
    assert got.shape == want.shape
    assert np.isfinite(got).all(), "non-finite values in the GPU result"
    d = got - want
    return float(np.abs(d).max() / max(np.abs(want).max(), 1e-30)), float(np.linalg.norm(d) / max(np.linalg.norm(want), 1e-30))


def out_elems(layers, shp):
    c, h, w = wl.layer_shapes(layers, shp)[-1]
    return c * h * w


class GpuNet:
    """One task registered on one partition of `n_cu` CUs, for direct forward passes."""

    def __init__(self, layers, weights, shp, dtype, k=1, n_cu=128, flags=0, extra_partitions=(), plan_cus=0):
        self.layers, self.shp, self.dtype = layers, shp, dtype
        D.daris_init(0, 0, flags)
        if plan_cus:
            D.daris_set_plan_cus(plan_cus)
        self.parts = [D.daris_create_partition(n_cu)] + [D.daris_create_partition(n) for n in extra_partitions]
        dnn, self._keep = D.make_dnn(layers, weights, shp, dtype)
        self.task = D.daris_register_task(dnn, 10_000_000, 10_000_000, D.LP)
        if k > 1:
            D.daris_split_stages(self.task, k)
        self.n_out = out_elems(layers, shp)

    def forward(self, x, part=0):
        xd = torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda()
        yd = torch.full((self.n_out,), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()          # the library runs on queues of its own: the buffers must be complete first
        D.daris_forward(self.task, xd, yd, self.parts[part])
        return yd.cpu().numpy()

    def close(self):
        D.daris_shutdown()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
        return False


def oracle_logits(layers, weights, x, dtype):
    return F.forward(layers, weights, x, dtype)
