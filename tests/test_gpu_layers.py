"""GPU parity of every kernel against the CPU oracle, one or two layers at a time, through the C ABI.
Shapes span several tiles, ragged M / N / K tails, split-K, both strides and both arithmetic types."""
import numpy as np
import pytest

import workloads as wl
import paper_2504_08795_amd as D
from gpu_helpers import GpuNet, oracle_logits, rel_err

pytestmark = pytest.mark.gpu
N = wl.nets
RNG = np.random.default_rng(99)

# per-layer bars, far inside the whole-network tolerances: fp32 accumulation over K <= 4608 terms versus a double sum
# (~sqrt(K) * 2^-24 relative to the row norm), bf16 one final rounding (2^-9) on top
LAYER_TOL = {"fp32": 2e-5, "bf16": 6e-3}


def rand_w(L, scale=None):
    cg = L.c_in // L.groups
    if L.op == N.OP_CONV:
        w = RNG.normal(0, np.sqrt(2.0 / (cg * L.k * L.k)), (L.c_out, cg, L.k, L.k))
    else:
        w = RNG.normal(0, np.sqrt(2.0 / L.c_in), (L.c_out, L.c_in))
    return w.astype(np.float32), RNG.normal(0, 0.3, L.c_out).astype(np.float32)


def run_case(layers, shp, dtype, tol=None):
    weights = [rand_w(L) if L.op in (N.OP_CONV, N.OP_FC) else (None, None) for L in layers]
    x = RNG.normal(0, 1, shp).astype(np.float32)
    want = oracle_logits(layers, weights, x, dtype)
    with GpuNet(layers, weights, shp, dtype) as net:
        got = net.forward(x)
    e_max, e_l2 = rel_err(got, want)
    tol = tol or LAYER_TOL[dtype]
    assert e_max <= tol and e_l2 <= tol, (e_max, e_l2)
    return got, want


CONV_CASES = [
    # (cin, h, w, cout, k, s, p, act)  -- comment: what it stresses
    (3, 32, 32, 16, 3, 1, 1, 1),      # Tiny c1: padded 3-channel input, N = 16 < tile
    (16, 32, 32, 32, 3, 1, 1, 1),     # Tiny c2
    (32, 16, 16, 64, 3, 1, 1, 1),     # Tiny c4
    (3, 64, 64, 64, 7, 2, 3, 1),      # stem 7x7 s2 (quarter-size image)
    (64, 28, 28, 64, 3, 1, 1, 1),     # layer1-like, M = 784
    (64, 29, 27, 128, 3, 2, 1, 1),    # stride 2, odd sizes, ragged M
    (64, 28, 28, 128, 1, 2, 0, 0),    # 1x1 s2 downsample, no activation
    (128, 14, 14, 256, 3, 1, 1, 1),   # M = 196 -> split-K
    (512, 7, 7, 512, 3, 1, 1, 1),     # M = 49, K = 4608 -> deep split-K
    (256, 7, 7, 1024, 1, 1, 0, 1),    # 1x1 wide N
    (24, 13, 13, 40, 1, 1, 0, 2),     # ragged everything, ReLU6
    (40, 9, 11, 24, 3, 1, 1, 0),      # K = 360: K tail inside a tile
    (8, 5, 5, 8, 3, 1, 1, 1),         # smaller than any tile
    (32, 56, 56, 64, 3, 1, 1, 1),     # M = 3136: many M tiles
    (16, 112, 112, 96, 1, 1, 0, 2),   # MobileNet expand: M = 12544, largest tile variant
    (1, 7, 7, 4, 3, 1, 1, 0),         # degenerate: one input channel, four outputs
    (4, 3, 3, 8, 3, 1, 0, 1),         # output is a single pixel (M = 1)
    (8, 1, 1, 12, 1, 1, 0, 0),        # 1x1 image, 1x1 kernel: a plain mat-vec
    (4, 9, 9, 4, 3, 3, 0, 0),         # stride equal to the kernel size: no window overlap
    (8, 6, 6, 8, 3, 1, 2, 1),         # padding larger than half the kernel: whole windows of zeros at the border
    (256, 14, 14, 200, 3, 1, 1, 1),   # 16-pixel tiles (M = 196: ragged last tile), N = 200: 13 blocks of 16, the last one ragged
    (512, 7, 7, 520, 3, 1, 1, 2),     # 16-pixel tiles, M = 49, 33 channel blocks, K = 4608, ReLU6
    (64, 224, 224, 64, 3, 1, 1, 1),   # the largest layer of any configuration (VGG-16 conv1_2): M = 50176
    (3, 224, 224, 64, 3, 1, 1, 1),    # VGG-16 conv1_1: K = 27, M = 50176
]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "x".join(map(str, c)))
def test_conv(case, dtype):
    cin, h, w, cout, k, s, p, act = case
    layers = [N.Layer(op=N.OP_CONV, c_in=cin, c_out=cout, k=k, stride=s, pad=p, act=act, in_from=-1)]
    run_case(layers, (cin, h, w), dtype)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("cin,hw,cout,s", [(64, 28, 128, 2), (64, 14, 64, 1), (256, 7, 512, 2)])
def test_conv_residual_block(cin, hw, cout, s, dtype):
    """downsample 1x1 (or identity) + 3x3 + 3x3 with residual add before ReLU: the basic-block epilogue."""
    layers = []
    if s != 1 or cin != cout:
        layers.append(N.Layer(op=N.OP_CONV, c_in=cin, c_out=cout, k=1, stride=s, pad=0, act=0, in_from=-1))
        skip, base = 0, 1
    else:
        layers.append(N.Layer(op=N.OP_MAXPOOL, c_in=cin, c_out=cin, k=1, stride=1, pad=0, in_from=-1))   # identity copy as tensor 0
        skip, base = 0, 1
    layers.append(N.Layer(op=N.OP_CONV, c_in=cin, c_out=cout, k=3, stride=s, pad=1, act=1, in_from=-1))
    layers.append(N.Layer(op=N.OP_CONV, c_in=cout, c_out=cout, k=3, stride=1, pad=1, act=1, in_from=base, res_from=skip))
    run_case(layers, (cin, hw, hw), dtype, tol={"fp32": 5e-5, "bf16": 1.2e-2}[dtype])


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("cin,h,w,mid,cout,s,ds_first", [
    (64, 28, 28, 32, 128, 2, True),     # ResNet-50 shape of block: shortcut 1x1 s2 and 1x1 s1 read the same tensor, different output sizes
    (64, 28, 28, 32, 128, 2, False),    # the same with the shortcut listed after the first convolution
    (40, 13, 11, 24, 72, 1, True),      # ragged sizes: padding workgroups between the two problems of the launch
    (256, 14, 14, 64, 512, 2, True),    # heavier problem split over K (its reduction follows the joint launch)
    (32, 9, 9, 96, 96, 1, False),       # channel block counts 3 and 3: the wide-tile variant does not apply to either
])
def test_conv_pair_in_bottleneck_block(cin, h, w, mid, cout, s, ds_first, dtype):
    """Two convolutions reading one tensor (issued as one launch) inside a bottleneck block with a strided middle layer."""
    ds = N.Layer(op=N.OP_CONV, c_in=cin, c_out=cout, k=1, stride=s, pad=0, act=0, in_from=-1)
    c1 = N.Layer(op=N.OP_CONV, c_in=cin, c_out=mid, k=1, stride=1, pad=0, act=1, in_from=-1)
    layers = [ds, c1] if ds_first else [c1, ds]
    i_ds, i_c1 = (0, 1) if ds_first else (1, 0)
    layers.append(N.Layer(op=N.OP_CONV, c_in=mid, c_out=mid, k=3, stride=s, pad=1, act=1, in_from=i_c1))
    layers.append(N.Layer(op=N.OP_CONV, c_in=mid, c_out=cout, k=1, stride=1, pad=0, act=1, in_from=2, res_from=i_ds))
    run_case(layers, (cin, h, w), dtype, tol={"fp32": 5e-5, "bf16": 1.5e-2}[dtype])


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("c,h,w,s", [(32, 112, 112, 1), (96, 57, 55, 2), (144, 28, 28, 1), (960, 7, 7, 1), (24, 9, 9, 2)])
def test_depthwise(c, h, w, s, dtype):
    layers = [N.Layer(op=N.OP_CONV, c_in=c, c_out=c, k=3, stride=s, pad=1, groups=c, act=2, in_from=-1)]
    run_case(layers, (c, h, w), dtype)


# (block input channels, hidden channels, h, w, depthwise stride, output channels, residual)
DW_PROJECT_CASES = [
    (16, 32, 112, 112, 1, 16, True),    # MobileNetV2's first block: K = 32, one chunk per wave, 392 pixel tiles
    (16, 96, 113, 111, 2, 24, False),   # stride 2 on odd sizes: 57 x 56 outputs, ragged last tile
    (24, 144, 56, 56, 1, 24, True),     # 144 channels: whole 64-byte rows in fp32 only (bf16 keeps the separate launch)
    (16, 64, 56, 56, 1, 64, False),     # 64 output channels: one tile of two channel blocks in bf16 (fused), two tiles in fp32 (not)
    (32, 192, 28, 28, 2, 64, False),    # the rest: too few pixel tiles or several channel blocks, the depthwise launch stays
    (64, 384, 14, 14, 1, 64, True),
    (160, 960, 7, 7, 1, 320, False),
    (40, 64, 9, 9, 1, 40, True),
]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("case", DW_PROJECT_CASES, ids=lambda c: "x".join(map(str, c)))
def test_depthwise_computed_inside_the_projection(case, dtype):
    """An inverted residual block's depthwise 3x3 convolution computed inside the launch of the 1x1 convolution that reads it:
    against the oracle, and against the same block with the depthwise layer in a launch of its own (bit for bit when the
    1x1 convolution keeps its plan, since the fused producer accumulates in the same order)."""
    cin, hid, h, w, s, cout, res = case
    if res:
        assert s == 1 and cin == cout
    layers = [N.Layer(op=N.OP_CONV, c_in=3, c_out=cin, k=3, stride=1, pad=1, act=0, in_from=-1),
              N.Layer(op=N.OP_CONV, c_in=cin, c_out=hid, k=1, stride=1, pad=0, act=2, in_from=0),
              N.Layer(op=N.OP_CONV, c_in=hid, c_out=hid, k=3, stride=s, pad=1, groups=hid, act=2, in_from=1),
              N.Layer(op=N.OP_CONV, c_in=hid, c_out=cout, k=1, stride=1, pad=0, act=0, in_from=2, res_from=0 if res else -1)]
    weights = [rand_w(L) for L in layers]
    x = RNG.normal(0, 1, (3, h, w)).astype(np.float32)
    want = oracle_logits(layers, weights, x, dtype)
    outs, plans = [], []
    for flags in (0, D.NO_FUSED_DW):
        with GpuNet(layers, weights, (3, h, w), dtype, flags=flags) as net:
            outs.append(net.forward(x))
            plans.append([D.daris_get_launch_plan(net.task, l) for l in range(4)])
    # fused where the hidden tensor's pixels are whole 64-byte rows and the 1x1 convolution has at least 96 pixel tiles and one
    # channel tile of a staged kernel variant
    o = plans[1][3]
    want_fused = (hid * (4 if dtype == "fp32" else 2)) % 64 == 0 and o["MT"] >= 96 and o["NTn"] == 1 and (dtype == "bf16" or o["tn"] == 1)
    assert (plans[0][2]["pair_with"] == 3) == want_fused and plans[1][2]["pair_with"] == -1    # the case runs the path it names
    assert want_fused == {"fp32": case in DW_PROJECT_CASES[:3], "bf16": case in DW_PROJECT_CASES[:2] + DW_PROJECT_CASES[3:4]}[dtype]
    tol = {"fp32": 5e-5, "bf16": 1.5e-2}[dtype]
    for got in outs:
        e_max, e_l2 = rel_err(got, want)
        assert e_max <= tol and e_l2 <= tol, (e_max, e_l2)
    if all(plans[0][3][k] == plans[1][3][k] for k in ("kernel_id", "splitk", "sz", "sw", "rows")):
        np.testing.assert_array_equal(outs[0], outs[1])


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("c,h,w,k,s,p", [(64, 112, 112, 3, 2, 1), (32, 32, 32, 2, 2, 0), (3, 9, 7, 3, 2, 1), (16, 15, 15, 2, 2, 0)])
def test_maxpool(c, h, w, k, s, p, dtype):
    layers = [N.Layer(op=N.OP_MAXPOOL, c_in=c, c_out=c, k=k, stride=s, pad=p, in_from=-1)]
    weights = [(None, None)]
    x = (-np.abs(RNG.normal(0, 1, (c, h, w))) - 0.5).astype(np.float32)       # all negative: padding must not win
    want = oracle_logits(layers, weights, x, dtype)
    with GpuNet(layers, weights, (c, h, w), dtype) as net:
        got = net.forward(x)
    np.testing.assert_array_equal(got, want)                                  # selection only: bit exact


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("c,h,w", [(512, 7, 7), (1280, 7, 7), (20, 3, 5)])
def test_gavgpool(c, h, w, dtype):
    layers = [N.Layer(op=N.OP_GAVGPOOL, c_in=c, c_out=c, in_from=-1)]
    run_case(layers, (c, h, w), dtype, tol={"fp32": 1e-6, "bf16": 4e-3}[dtype])


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("c,h,w,n,act", [(64, 8, 8, 10, 0), (512, 1, 1, 1000, 0), (32, 7, 7, 4096, 1), (3, 5, 5, 7, 0)])
def test_fc(c, h, w, n, act, dtype):
    layers = [N.Layer(op=N.OP_FC, c_in=c * h * w, c_out=n, act=act, in_from=-1)]
    run_case(layers, (c, h, w), dtype)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_fc_chain_with_padded_vector(dtype):
    """FC -> FC where the intermediate vector length (10) is not a multiple of the 16-byte vector."""
    layers = [N.Layer(op=N.OP_FC, c_in=16 * 4 * 4, c_out=10, act=1, in_from=-1), N.Layer(op=N.OP_FC, c_in=10, c_out=6, in_from=0)]
    run_case(layers, (16, 4, 4), dtype, tol={"fp32": 2e-5, "bf16": 1e-2}[dtype])


def test_identity_passthrough_is_exact():
    """ingest + 1x1 max-pool + egress moves every value unchanged (layout conversions only)."""
    layers = [N.Layer(op=N.OP_MAXPOOL, c_in=5, c_out=5, k=1, stride=1, pad=0, in_from=-1)]
    x = RNG.normal(0, 1, (5, 6, 7)).astype(np.float32)
    with GpuNet(layers, [(None, None)], (5, 6, 7), "fp32") as net:
        np.testing.assert_array_equal(net.forward(x), x.reshape(-1))


def test_joint_launch_whose_earlier_member_has_a_residual_operand():
    """L2 (3x3, + L0's output as residual) and L3 (1x1) both read L1 and share a launch that is issued at L3.  L0's output
    is read last by L2, so its buffer falls free exactly when L3's output is placed: it must not be reused before the
    joint launch (and L2's split-K reduction) have read it."""
    def c(i, r=-1, k=3, cin=32):
        return N.Layer(op=N.OP_CONV, c_in=cin, c_out=32, k=k, stride=1, pad=k // 2, act=1, in_from=i, res_from=r)
    layers = [c(-1, cin=3), c(0), c(1, 0), c(1, -1, 1), c(3, 2), N.Layer(op=N.OP_GAVGPOOL, c_in=32, c_out=32, in_from=4),
              N.Layer(op=N.OP_FC, c_in=32, c_out=10, in_from=5)]
    for dtype in ("fp32", "bf16"):
        run_case(layers, (3, 12, 12), dtype, tol={"fp32": 2e-5, "bf16": 2e-2}[dtype])
