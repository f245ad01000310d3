"""Whole-network GPU parity: logits of every architecture against the oracle at the benchmark spec's tolerances
(1e-3 fp32, 2e-2 bf16), bit-identical logits across stage splits and partitions, per-layer drill-down."""
import numpy as np
import pytest

import paper_2504_08795_amd as D
import workloads as wl
from gpu_helpers import TOL, GpuNet, oracle_logits, rel_err
from oracle import forward as F

pytestmark = pytest.mark.gpu

CASES = [("tiny", "fp32", "uniform"), ("resnet18", "fp32", "normal"), ("resnet50", "bf16", "normal"), ("resnet50", "fp32", "normal"),
         ("mobilenet_v2", "fp32", "normal"), ("vgg16", "fp32", "normal"), ("resnet18", "bf16", "normal"), ("mobilenet_v2", "bf16", "normal")]


@pytest.mark.parametrize("net,dtype,dist", CASES)
def test_network_logits(net, dtype, dist):
    layers, shp = wl.build_net(net)
    weights = wl.make_weights(layers, 4242)
    xs = wl.make_inputs(shp, 4242, 2, dist)
    k = {"tiny": 2, "resnet18": 3, "resnet50": 4, "vgg16": 3, "mobilenet_v2": 3}[net]
    with GpuNet(layers, weights, shp, dtype, k=k) as g:
        for x in xs:
            got = g.forward(x)
            want = oracle_logits(layers, weights, x, dtype)
            e_max, e_l2 = rel_err(got, want)
            print(f"{net} {dtype}: max-norm rel err {e_max:.3e}, l2 rel err {e_l2:.3e}, argmax {got.argmax()} vs {want.argmax()}")
            assert e_max <= TOL[dtype] and e_l2 <= TOL[dtype], (e_max, e_l2)


@pytest.mark.parametrize("net,dtype", [("resnet18", "fp32"), ("resnet50", "bf16"), ("mobilenet_v2", "fp32")])
def test_logits_bit_identical_across_splits_and_partitions(net, dtype):
    layers, shp = wl.build_net(net)
    weights = wl.make_weights(layers, 7)
    x = wl.make_inputs(shp, 7, 1, "normal")[0]
    outs = []
    for k, n_cu in ((1, 128), (4, 128), (3, 64)):
        with GpuNet(layers, weights, shp, dtype, k=k, n_cu=n_cu, extra_partitions=(192,)) as g:
            outs.append(g.forward(x, part=0))
            outs.append(g.forward(x, part=1))
    for o in outs[1:]:
        np.testing.assert_array_equal(o, outs[0])


@pytest.mark.parametrize("net,dtype,plan_cus", [("resnet18", "fp32", 64), ("resnet18", "fp32", 96), ("resnet50", "bf16", 64), ("mobilenet_v2", "fp32", 32),
                                                 ("vgg16", "fp32", 96)])
def test_plans_balanced_for_another_partition_size(net, dtype, plan_cus):
    """daris_set_plan_cus changes how the convolutions are cut into workgroups (other tiles, other K slices): the logits must
    meet the same tolerance, and still be the same bit for bit on every partition the task runs in."""
    layers, shp = wl.build_net(net)
    weights = wl.make_weights(layers, 13)
    x = wl.make_inputs(shp, 13, 1, "normal")[0]
    want = oracle_logits(layers, weights, x, dtype)
    with GpuNet(layers, weights, shp, dtype, k=3, n_cu=plan_cus, extra_partitions=(192,), plan_cus=plan_cus) as g:
        a, b = g.forward(x, part=0), g.forward(x, part=1)
        plans = [D.daris_get_launch_plan(g.task, l) for l in range(len(layers))]
    with GpuNet(layers, weights, shp, dtype, k=3, n_cu=plan_cus) as g:
        default_plans = [D.daris_get_launch_plan(g.task, l) for l in range(len(layers))]
    assert any(p["grid_x"] != q["grid_x"] for p, q in zip(plans, default_plans))     # the case is what it claims to be
    np.testing.assert_array_equal(a, b)
    e_max, e_l2 = rel_err(a, want)
    assert e_max <= TOL[dtype] and e_l2 <= TOL[dtype], (e_max, e_l2)


def test_every_legal_cut_in_use():
    """MobileNetV2 with as many stages as the cut rule allows: stages of a single layer, among them depthwise layers that are
    otherwise computed inside the following convolution's launch.  Same logits, bit for bit, as with one stage."""
    from oracle import staging
    layers, shp = wl.build_net("mobilenet_v2")
    weights = wl.make_weights(layers, 17)
    x = wl.make_inputs(shp, 17, 1, "normal")[0]
    k = len(staging.legal_cuts(layers)) + 1
    with GpuNet(layers, weights, shp, "fp32", k=1) as g:
        one = g.forward(x)
    with GpuNet(layers, weights, shp, "fp32", k=k) as g:
        many = g.forward(x)
        assert len(D.daris_get_stage_cuts(g.task)) == k
        D.daris_calibrate_afet(g.task, g.parts[0], 1)            # runs stage by stage: every stage must have something to launch
        D.daris_split_stages(g.task, 2)
        two = g.forward(x)
    np.testing.assert_array_equal(one, many)
    np.testing.assert_array_equal(one, two)
    e_max, e_l2 = rel_err(one, oracle_logits(layers, weights, x, "fp32"))
    assert e_max <= TOL["fp32"] and e_l2 <= TOL["fp32"]


@pytest.mark.parametrize("net,dtype", [("resnet18", "fp32"), ("resnet50", "bf16"), ("mobilenet_v2", "fp32"), ("mobilenet_v2", "bf16")])
def test_plain_launch_shapes_agree_with_the_fused_ones(net, dtype):
    """The launch-count optimisations -- a residual block's shortcut and first convolution in one launch, the input layout
    conversion folded into the first convolution -- can be switched off when a task is registered: the plain launches
    must meet the same tolerance against the oracle, and agree with the fused ones to rounding."""
    layers, shp = wl.build_net(net)
    weights = wl.make_weights(layers, 11)
    x = wl.make_inputs(shp, 11, 1, "normal")[0]
    want = oracle_logits(layers, weights, x, dtype)
    with GpuNet(layers, weights, shp, dtype, k=3) as g:
        fused = g.forward(x)
        n_pairs = sum(1 for l in range(len(layers)) if D.daris_get_launch_plan(g.task, l)["pair_lead"])
    assert n_pairs >= (2 if net == "mobilenet_v2" else 3)      # MobileNetV2: depthwise layers computed inside the projections
    with GpuNet(layers, weights, shp, dtype, k=3, flags=D.NO_PAIR | D.NO_FUSED_INGEST | D.NO_FUSED_DW) as g:
        plain = g.forward(x)
        assert not any(D.daris_get_launch_plan(g.task, l)["pair_lead"] for l in range(len(layers)))
    for got in (fused, plain):
        e_max, e_l2 = rel_err(got, want)
        assert e_max <= TOL[dtype] and e_l2 <= TOL[dtype], (e_max, e_l2)
    assert rel_err(plain, fused)[0] <= TOL[dtype]


@pytest.mark.parametrize("net", ["mobilenet_v2", "resnet50"])
def test_bf16_layers_on_the_oracles_own_inputs(net):
    """The max-norm check that the chained drill-down cannot apply to bf16 intermediates (one rounding that falls the other
    way upstream moves single elements downstream by whole bf16 steps): every layer alone, fed with the ORACLE's bf16 input
    tensor of that layer.  With upstream decisions out of the picture, each output element must be the oracle's value or its
    bf16 neighbour (fp32 versus double accumulation can still tip one rounding), and only a small share may differ at all."""
    import dataclasses
    layers, shp = wl.build_net(net)
    weights = wl.make_weights(layers, 5)
    x = wl.make_inputs(shp, 5, 1, "normal")[0]
    _, acts = F.forward(layers, weights, x, "bf16", return_all=True)
    shapes = wl.layer_shapes(layers, shp)
    worst_share, checked = 0.0, 0
    for l, L in enumerate(layers[:-1]):                       # the last layer's logits stay fp32: covered by the logits tests
        if L.res_from >= 0:
            continue                                          # needs two input tensors; its sum is covered by the chained runs
        xin = x if L.in_from < 0 else np.asarray(acts[L.in_from], np.float32).reshape(shapes[L.in_from])
        one = [dataclasses.replace(L, in_from=-1, res_from=-1)]
        with GpuNet(one, [weights[l]], xin.shape, "bf16") as g:
            got = g.forward(xin).astype(np.float64)
        want = np.asarray(acts[l], np.float64).reshape(-1)
        step = np.abs(want) * 2.0 ** -7 + 1e-6 * np.abs(want).max()        # one bf16 step of the element (8 significant bits)
        assert (np.abs(got - want) <= step).all(), (l, L.name, float(np.abs(got - want).max()), float(np.abs(want).max()))
        share = float((got != want).mean())
        assert share <= 0.001, (l, L.name, share)
        worst_share = max(worst_share, share)
        checked += 1
    assert checked >= 35
    print(f"{net} bf16, each layer on the oracle's input: at most {100 * worst_share:.3f} % of a layer's elements differ, none by more than one step")


@pytest.mark.parametrize("net,dtype", [("resnet18", "fp32"), ("resnet50", "bf16"), ("mobilenet_v2", "fp32")])
def test_every_layer_output(net, dtype):
    """Drill-down with one buffer per layer: each intermediate tensor against the oracle's."""
    layers, shp = wl.build_net(net)
    weights = wl.make_weights(layers, 5)
    x = wl.make_inputs(shp, 5, 1, "normal")[0]
    want, acts = F.forward(layers, weights, x, dtype, return_all=True)
    shapes = wl.layer_shapes(layers, shp)
    with GpuNet(layers, weights, shp, dtype, flags=D.KEEP_ACTIVATIONS) as g:
        g.forward(x)
        worst = 0.0
        for l in range(len(layers) - 1):          # the last layer writes straight into the logits
            c, h, w = shapes[l]
            got = D.daris_read_layer(g.task, l, c * h * w)
            e_max, e_l2 = rel_err(got, acts[l])
            worst = max(worst, e_max)
            # bf16: an upstream rounding decision that falls the other way moves single elements of a clipped
            # (ReLU6) intermediate tensor by several bf16 steps, so for bf16 intermediates only the L2 error is gated
            assert e_l2 <= TOL[dtype], (l, layers[l].name, e_max, e_l2)
            if dtype == "fp32":
                assert e_max <= TOL[dtype], (l, layers[l].name, e_max, e_l2)
    print(f"{net} {dtype}: worst per-layer max-norm rel err {worst:.3e}")
