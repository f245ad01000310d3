"""The entry point that allocates nothing (daris_forward_static) against the existing one (daris_forward), through the
C ABI: bit-identical logits, both within the parity tolerance of the CPU oracle, on calls in a row that share the static
device scratch -- a larger network first, then a smaller input, then the larger one again."""
import numpy as np
import pytest
import torch

import paper_2504_08795_amd as D
import workloads as wl
from gpu_helpers import TOL, oracle_logits, rel_err

pytestmark = pytest.mark.gpu


def _register(net, dtype, seed):
    layers, shp = wl.build_net(net)
    weights = wl.make_weights(layers, seed)
    dnn, keep = D.make_dnn(layers, weights, shp, dtype)
    t = D.daris_register_task(dnn, 10_000_000, 10_000_000, D.LP)
    x = wl.make_inputs(shp, seed, 1, "uniform" if net == "tiny" else "normal")[0]
    return dict(task=t, layers=layers, weights=weights, shp=shp, dtype=dtype, x=x, xd=torch.from_numpy(x).cuda(), n_out=layers[-1].c_out, keep=keep)


def _run(fn, c, part):
    y = torch.full((c["n_out"],), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    fn(c["task"], c["xd"], y, part)
    return y.cpu().numpy()


def test_forward_static_matches_forward_on_calls_in_a_row():
    D.daris_init(0, 0, 0)
    try:
        parts = [D.daris_create_partition(128), D.daris_create_partition(96)]
        big16 = _register("resnet18", "bf16", 31)      # bf16 bit patterns are left in the scratch for the fp32 call after it
        small = _register("tiny", "fp32", 32)          # the smaller input: 3x32x32 instead of 3x224x224
        big32 = _register("resnet18", "fp32", 33)
        N = wl.nets
        huge_layers = [N.Layer(op=N.OP_CONV, c_in=3, c_out=64, k=3, stride=1, pad=1, act=1, in_from=-1)]
        rng = np.random.default_rng(1)
        dnn, keep = D.make_dnn(huge_layers, [(rng.normal(0, 0.1, (64, 3, 3, 3)).astype(np.float32), np.zeros(64, np.float32))], (3, 320, 320), "fp32")
        huge = D.daris_register_task(dnn, 10_000_000, 10_000_000, D.LP)
        with pytest.raises(D.DarisError) as e:         # no stream exists yet: creating them would allocate
            D.daris_forward_static(small["task"], small["xd"], torch.zeros(10, device="cuda"), parts[0])
        assert e.value.code == D.ESTATE
        ref = {k: _run(D.daris_forward, c, parts[0]) for k, c in (("big16", big16), ("small", small), ("big32", big32))}
        want = {k: oracle_logits(c["layers"], c["weights"], c["x"], c["dtype"]) for k, c in (("big16", big16), ("small", small), ("big32", big32))}
        order = [("big16", big16, 0), ("small", small, 0), ("big32", big32, 1), ("small", small, 1), ("big16", big16, 1)]
        for name, c, p in order:
            y = torch.full((c["n_out"],), float("nan"), dtype=torch.float32, device="cuda")
            torch.cuda.synchronize()
            free_before = torch.cuda.mem_get_info()[0]
            D.daris_forward_static(c["task"], c["xd"], y, parts[p])
            assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated or freed during the call"
            got = y.cpu().numpy()
            np.testing.assert_array_equal(got, ref[name], err_msg=f"{name} on partition {p}")
            e_max, e_l2 = rel_err(got, want[name])
            assert e_max <= TOL[c["dtype"]] and e_l2 <= TOL[c["dtype"]], (name, e_max, e_l2)
        # a network whose tensors do not fit the 16 MiB array is refused with a clear error, and nothing breaks afterwards
        with pytest.raises(D.DarisError) as e:
            D.daris_forward_static(huge, torch.zeros(3 * 320 * 320, device="cuda"), torch.zeros(64 * 320 * 320, device="cuda"), parts[0])
        assert e.value.code == D.ERANGE and "static scratch holds" in str(e.value)
        np.testing.assert_array_equal(_run(D.daris_forward_static, small, parts[0]), ref["small"])
        np.testing.assert_array_equal(_run(D.daris_forward, big32, parts[1]), ref["big32"])
    finally:
        D.daris_shutdown()
