"""Pins of the forward-pass oracle against things other than itself: brute force, closed forms,
structural identities and PyTorch CPU float64 library routines."""
import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import workloads as wl
from oracle import forward as F

RNG = np.random.default_rng(1234)


def brute_conv(x, w, b, stride, pad, groups):
    """Second formulation: explicit zero-padded copy, window gather, float64 dot product."""
    x = np.asarray(x, np.float64)
    w = np.asarray(w, np.float64)
    c, h, wd = x.shape
    co, cg, k, _ = w.shape
    xp = np.zeros((c, h + 2 * pad, wd + 2 * pad))
    xp[:, pad:pad + h, pad:pad + wd] = x
    ho, wo = (h + 2 * pad - k) // stride + 1, (wd + 2 * pad - k) // stride + 1
    y = np.zeros((co, ho, wo))
    og = co // groups
    for o in range(co):
        g = o // og
        for i in range(ho):
            for j in range(wo):
                win = xp[g * cg:(g + 1) * cg, i * stride:i * stride + k, j * stride:j * stride + k]
                y[o, i, j] = float(np.dot(win.reshape(-1), w[o].reshape(-1))) + (0.0 if b is None else b[o])
    return y


@pytest.mark.parametrize("c,h,w,co,k,s,p,g", [
    (1, 4, 4, 1, 3, 1, 1, 1), (3, 6, 5, 2, 3, 1, 1, 1), (2, 6, 6, 4, 3, 2, 1, 1), (3, 7, 7, 2, 7, 2, 3, 1),
    (4, 5, 6, 4, 3, 1, 1, 4), (4, 6, 6, 6, 3, 2, 1, 2), (3, 5, 5, 5, 1, 1, 0, 1), (2, 6, 6, 3, 1, 2, 0, 1),
    (2, 5, 4, 2, 2, 2, 0, 1), (1, 3, 3, 1, 3, 1, 0, 1),
])
def test_conv_matches_brute_force(c, h, w, co, k, s, p, g):
    x = RNG.normal(size=(c, h, w)).astype(np.float32)
    wt = RNG.normal(size=(co, c // g, k, k)).astype(np.float32)
    b = RNG.normal(size=co).astype(np.float32)
    got = F.conv2d(x, wt, b, s, p, g)
    want = brute_conv(x, wt, b, s, p, g)
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-6 * max(1.0, np.abs(want).max()))


@pytest.mark.parametrize("c,h,w,co,k,s,p,g", [
    (16, 20, 17, 24, 3, 1, 1, 1), (8, 23, 23, 16, 3, 2, 1, 1), (3, 32, 32, 8, 7, 2, 3, 1),
    (24, 14, 14, 24, 3, 1, 1, 24), (24, 15, 15, 24, 3, 2, 1, 24), (32, 9, 9, 48, 1, 1, 0, 1), (32, 9, 9, 48, 1, 2, 0, 1),
])
def test_conv_matches_torch_float64(c, h, w, co, k, s, p, g):
    x = RNG.normal(size=(c, h, w)).astype(np.float32)
    wt = RNG.normal(size=(co, c // g, k, k)).astype(np.float32)
    b = RNG.normal(size=co).astype(np.float32)
    r = None
    want = TF.conv2d(torch.from_numpy(x).double()[None], torch.from_numpy(wt).double(), torch.from_numpy(b).double(),
                     stride=s, padding=p, groups=g)[0].numpy()
    r = RNG.normal(size=want.shape).astype(np.float32)
    for act in (0, 1, 2):
        ref = want + r
        if act == 1:
            ref = np.maximum(ref, 0)
        elif act == 2:
            ref = np.clip(ref, 0, 6)
        got = F.conv2d(x, wt, b, s, p, g, res=r, act=act)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-6 * np.abs(want).max())


def test_identity_and_delta_kernels():
    x = RNG.normal(size=(3, 6, 7)).astype(np.float32)
    eye = np.eye(3, dtype=np.float32).reshape(3, 3, 1, 1)
    np.testing.assert_array_equal(F.conv2d(x, eye), x)
    centre = np.zeros((3, 3, 3, 3), np.float32)
    for c in range(3):
        centre[c, c, 1, 1] = 1
    np.testing.assert_array_equal(F.conv2d(x, centre, pad=1), x)
    # tap (ky=0, kx=2): Y[y,x] = X[y-1, x+1]  -> shifted input with a zero border
    off = np.zeros((3, 3, 3, 3), np.float32)
    for c in range(3):
        off[c, c, 0, 2] = 1
    y = F.conv2d(x, off, pad=1)
    want = np.zeros_like(x)
    want[:, 1:, :-1] = x[:, :-1, 1:]
    np.testing.assert_array_equal(y, want)


def test_all_ones_closed_form():
    cin = 5
    x = np.ones((cin, 6, 6), np.float32)
    w = np.ones((2, cin, 3, 3), np.float32)
    y = F.conv2d(x, w, pad=1)
    assert y[0, 2, 3] == 9 * cin and y[1, 0, 3] == 6 * cin and y[0, 5, 0] == 4 * cin and y[1, 5, 5] == 4 * cin


def test_linearity_and_output_size():
    x, z = (RNG.normal(size=(4, 9, 9)).astype(np.float32) for _ in range(2))
    w = RNG.normal(size=(6, 4, 3, 3)).astype(np.float32)
    a, b = 0.5, -2.0   # exactly representable factors
    lhs = F.conv2d((a * x + b * z).astype(np.float32), w, stride=2, pad=1)
    rhs = a * F.conv2d(x, w, stride=2, pad=1) + b * F.conv2d(z, w, stride=2, pad=1)
    assert lhs.shape == (6, 5, 5)
    np.testing.assert_allclose(lhs, rhs, atol=2e-5)
    assert F.conv2d(np.zeros((1, 224, 224), np.float32), np.zeros((1, 1, 7, 7), np.float32), stride=2, pad=3).shape == (1, 112, 112)
    assert F.maxpool2d(np.zeros((1, 112, 112), np.float32), 3, 2, 1).shape == (1, 56, 56)


def test_depthwise_equals_block_diagonal_dense():
    c = 6
    x = RNG.normal(size=(c, 8, 8)).astype(np.float32)
    wd = RNG.normal(size=(c, 1, 3, 3)).astype(np.float32)
    dense = np.zeros((c, c, 3, 3), np.float32)
    for i in range(c):
        dense[i, i] = wd[i, 0]
    np.testing.assert_array_equal(F.conv2d(x, wd, stride=2, pad=1, groups=c), F.conv2d(x, dense, stride=2, pad=1))


def test_bn_fold_matches_unfused_conv_then_bn():
    c, co = 5, 7
    x = torch.from_numpy(RNG.normal(size=(1, c, 9, 9)))
    w = RNG.normal(size=(co, c, 3, 3))
    gamma, beta, mean, var = wl.tensors.make_bn(3, 0, co)
    conv = TF.conv2d(x, torch.from_numpy(w), None, padding=1)[0].numpy()
    unfused = F.batchnorm(conv, gamma, beta, mean, var, wl.tensors.BN_EPS)
    lib = TF.batch_norm(torch.from_numpy(conv)[None], torch.from_numpy(mean), torch.from_numpy(var), torch.from_numpy(gamma),
                        torch.from_numpy(beta), False, 0.0, wl.tensors.BN_EPS)[0].numpy()
    np.testing.assert_allclose(unfused, lib, rtol=1e-12, atol=1e-12)
    wf, bf = wl.fold_bn(w, gamma, beta, mean, var)
    folded = TF.conv2d(x, torch.from_numpy(wf), torch.from_numpy(bf), padding=1)[0].numpy()
    np.testing.assert_allclose(folded, unfused, rtol=1e-12, atol=1e-12)


def test_pools():
    x = np.full((3, 8, 8), 2.5, np.float32)
    assert np.all(F.maxpool2d(x, 2, 2) == 2.5) and np.all(F.maxpool2d(x, 3, 2, 1) == 2.5) and np.all(F.gavgpool(x) == 2.5)
    neg = -np.abs(RNG.normal(size=(2, 7, 7))).astype(np.float32) - 1   # padding must be -inf, not 0
    got = F.maxpool2d(neg, 3, 2, 1)
    want = TF.max_pool2d(torch.from_numpy(neg)[None], 3, 2, 1)[0].numpy()
    np.testing.assert_array_equal(got, want)
    assert got.max() < 0
    y = RNG.normal(size=(4, 10, 10)).astype(np.float32)
    np.testing.assert_array_equal(F.maxpool2d(y, 2, 2), TF.max_pool2d(torch.from_numpy(y)[None], 2, 2)[0].numpy())
    np.testing.assert_array_equal(F.maxpool2d(y, 1, 1), y)      # 1x1 windows: identity
    ramp = np.arange(49, dtype=np.float32).reshape(1, 7, 7)
    assert F.gavgpool(ramp)[0, 0, 0] == 24.0                      # mean of 0..48
    np.testing.assert_allclose(F.gavgpool(y).reshape(-1), y.astype(np.float64).mean(axis=(1, 2)), atol=1e-7)


def test_fc_matches_numpy_float64():
    w = RNG.normal(size=(10, 37)).astype(np.float32)
    x = RNG.normal(size=37).astype(np.float32)
    b = RNG.normal(size=10).astype(np.float32)
    want = w.astype(np.float64) @ x.astype(np.float64) + b
    np.testing.assert_allclose(F.fc(x, w, b), want, atol=1e-6)
    np.testing.assert_allclose(F.fc(x, w, b, act=1), np.maximum(want, 0), atol=1e-6)


def test_bf16_rounding_bit_patterns():
    def rt(bits):
        f = np.array([bits], np.uint32).view(np.float32)
        return int(F.bf16_round(f).view(np.uint32)[0])
    assert rt(0x3F800000) == 0x3F800000          # 1.0 exact
    assert rt(0x3F808000) == 0x3F800000          # tie, lower mantissa even -> down
    assert rt(0x3F818000) == 0x3F820000          # tie, lower mantissa odd -> up
    assert rt(0x3F808001) == 0x3F810000          # just above tie -> up
    assert rt(0x3F807FFF) == 0x3F800000          # just below tie -> down
    assert rt(0x00000000) == 0x00000000 and rt(0x80000000) == 0x80000000   # +-0
    assert rt(0x00008000) == 0x00000000          # subnormal tie to even (0)
    assert rt(0x00018000) == 0x00020000          # subnormal tie, odd -> up
    assert rt(0x7F7FFFFF) == 0x7F800000          # max float rounds to +inf
    assert rt(0xFF7FFFFF) == 0xFF800000
    assert rt(0x7F800000) == 0x7F800000          # inf stays
    v = RNG.normal(size=4096).astype(np.float32) * np.float32(1e3)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float32).numpy()   # library conversion
    np.testing.assert_array_equal(F.bf16_round(v), want)


def test_bf16_mode_equals_fp32_mode_on_exact_values():
    """Small integers and dyadic weights are exact in bfloat16, so both precision modes must agree bit for bit."""
    g = np.random.default_rng(5)
    N = wl.nets
    layers = [N.Layer(op=N.OP_CONV, c_in=3, c_out=4, k=3, stride=1, pad=1, act=N.ACT_RELU, in_from=-1),
              N.Layer(op=N.OP_MAXPOOL, c_in=4, c_out=4, k=2, stride=2, in_from=0),
              N.Layer(op=N.OP_FC, c_in=4 * 4 * 4, c_out=5, in_from=1)]
    weights = [(g.integers(-1, 2, size=(4, 3, 3, 3)).astype(np.float32), g.integers(-2, 3, size=4).astype(np.float32)),
               (None, None),
               (g.choice([-0.5, 0.0, 0.5], size=(5, 64)).astype(np.float32), g.integers(-2, 3, size=5).astype(np.float32))]
    x = g.integers(0, 2, size=(3, 8, 8)).astype(np.float32)
    y32, a32 = F.forward(layers, weights, x, "fp32", return_all=True)
    y16, a16 = F.forward(layers, weights, x, "bf16", return_all=True)
    assert np.abs(a32[0]).max() <= 29          # |sum| <= 27 + 2: exactly representable with 8 mantissa bits
    for p, q in zip(a32, a16):
        np.testing.assert_array_equal(p, q)
    # and a value that is not representable must differ between the modes
    x2 = x + np.float32(1 / 512)
    assert not np.array_equal(F.forward(layers, weights, x2, "fp32"), F.forward(layers, weights, x2, "bf16"))


def torch_forward(layers, weights, x, in_shape):
    """The same layer table run through PyTorch CPU float64 library routines."""
    outs = []
    x = torch.from_numpy(x).double()[None]
    for l, L in enumerate(layers):
        src = x if L.in_from < 0 else outs[L.in_from]
        w, b = weights[l]
        if L.op == wl.nets.OP_CONV:
            y = TF.conv2d(src, torch.from_numpy(w).double(), torch.from_numpy(b).double(), stride=L.stride, padding=L.pad,
                          groups=L.groups)
            if L.res_from >= 0:
                y = y + outs[L.res_from]
        elif L.op == wl.nets.OP_MAXPOOL:
            y = TF.max_pool2d(src, L.k, L.stride, L.pad)
        elif L.op == wl.nets.OP_GAVGPOOL:
            y = src.mean(dim=(2, 3), keepdim=True)
        else:
            y = (src.reshape(1, -1) @ torch.from_numpy(w).double().T + torch.from_numpy(b).double()).reshape(1, -1, 1, 1)
        if L.act == 1:
            y = torch.relu(y)
        elif L.act == 2:
            y = torch.clamp(y, 0, 6)
        outs.append(y)
    return outs[-1].reshape(-1).numpy()


@pytest.mark.parametrize("net,dist", [("tiny", "uniform"), ("resnet18", "normal"), ("mobilenet_v2", "normal"), ("resnet50", "normal")])
def test_whole_network_matches_torch_float64(net, dist):
    layers, shp = wl.build_net(net)
    weights = wl.make_weights(layers, 11)
    x = wl.make_inputs(shp, 11, 1, dist)[0]
    got = F.forward(layers, weights, x, "fp32")
    want = torch_forward(layers, weights, x, shp)
    # the oracle rounds every layer output to float32; the library path stays in float64
    assert np.abs(got - want).max() <= 2e-5 * np.abs(want).max()


def test_network_integer_totals():
    want = {"tiny": (12_279_808, 73_802, 86_026), "resnet18": (1_814_073_344, 11_684_712, 2_685_928),
            "resnet50": (4_089_184_256, 25_530_472, 11_317_736), "vgg16": (15_470_264_320, 138_357_544, 15_087_080),
            "mobilenet_v2": (300_774_272, 3_487_816, 6_680_392)}
    for net, (macs, params, acts) in want.items():
        layers, shp = wl.build_net(net)
        assert sum(wl.net_macs(layers, shp)) == macs
        assert wl.net_params(layers) == params
        assert sum(c * h * w for c, h, w in wl.layer_shapes(layers, shp)) == acts
    layers, shp = wl.build_net("mobilenet_v2")
    dw = sum(m for m, L in zip(wl.net_macs(layers, shp), layers) if L.groups > 1)
    assert dw == 20_716_416
    layers, shp = wl.build_net("vgg16")
    assert sum(m for m, L in zip(wl.net_macs(layers, shp), layers) if L.op == wl.nets.OP_FC) == 123_633_664


def test_bf16_mode_rounds_at_every_stated_point_hand_worked():
    """A 1-channel toy worked by hand (bfloat16 keeps 8 significant bits; nearest, ties to even).  Each rounding point of
    the bf16 mode -- input, weights, every layer output after bias + residual + activation, the residual operand being the
    STORED tensor, the pooled value, and the logits NOT rounded -- changes at least one of the numbers below.

    x = [2, 7, 3, 1+2^-8] (2x2).  Input rounding: 1+2^-8 is a tie between 1 and 1+2^-7 -> even -> 1.
    L0 conv1x1 w = 515/512 -> bf16 129/128 (515/512 lies 1/512 below 129/128, 3/512 above 1); b = 31/128 (kept fp32).
       2*129/128 + 31/128 = 144.5/64  tie, 144 even -> 2.25        (ties away would give 145/64)
       7*129/128 + 31/128 = 233.5/32  tie, 234 even -> 7.3125      (unrounded w: 233.06/32 -> 7.28125)
       3*129/128 + 31/128 = 209/64    exact         -> 3.265625
       1*129/128 + 31/128 = 160/128   exact         -> 1.25        (unrounded input: 160.5/128 -> 161/128)
    L1 conv1x1 w = 0.5, b = 0, residual = L0's stored output, ReLU: 1.5 * stored
       3.375 exact; 10.96875 = 175.5/16 tie, 176 even -> 11.0 (with the unrounded residual 7.296875: 175.25/16 -> 10.9375);
       4.8984375 = 156.75/32 -> 157/32 = 4.90625; 1.875 exact.
    L2 global average: (3.375 + 11 + 4.90625 + 1.875) / 4 = 5.2890625 = 169.25/32 -> 5.28125.
    L3 FC w = [515/512 -> 129/128, -2], b = [2^-8, 0]: logits = [129/128 * 169/32 + 1/256, -10.5625]
       = [21817/4096, -10.5625] = [5.326416015625, -10.5625], exact in fp32 and left unrounded (bf16 would give 5.3125)."""
    N = wl.nets
    layers = [N.Layer(op=N.OP_CONV, c_in=1, c_out=1, k=1, in_from=-1),
              N.Layer(op=N.OP_CONV, c_in=1, c_out=1, k=1, act=N.ACT_RELU, in_from=0, res_from=0),
              N.Layer(op=N.OP_GAVGPOOL, c_in=1, c_out=1, in_from=1),
              N.Layer(op=N.OP_FC, c_in=1, c_out=2, in_from=2)]
    f = np.float32
    weights = [(np.full((1, 1, 1, 1), 515 / 512, f), np.array([31 / 128], f)),
               (np.full((1, 1, 1, 1), 0.5, f), np.zeros(1, f)),
               (None, None),
               (np.array([[515 / 512], [-2.0]], f), np.array([2.0 ** -8, 0.0], f))]
    x = np.array([[[2.0, 7.0], [3.0, 1 + 2.0 ** -8]]], f)
    logits, outs = F.forward(layers, weights, x, "bf16", return_all=True)
    np.testing.assert_array_equal(outs[0].ravel(), np.array([2.25, 7.3125, 3.265625, 1.25], f))
    np.testing.assert_array_equal(outs[1].ravel(), np.array([3.375, 11.0, 4.90625, 1.875], f))
    np.testing.assert_array_equal(outs[2].ravel(), np.array([5.28125], f))
    np.testing.assert_array_equal(logits, np.array([21817 / 4096, -10.5625], f))
    # the same toy in fp32 mode rounds nowhere: 515/512 * x + 31/128 etc. stay as computed
    l32, o32 = F.forward(layers, weights, x, "fp32", return_all=True)
    np.testing.assert_array_equal(o32[0].ravel(), (np.array([2.0, 7.0, 3.0, 1 + 2.0 ** -8]) * (515 / 512) + 31 / 128).astype(f))
    assert l32[1] == f(-2.0) * o32[2].ravel()[0]
