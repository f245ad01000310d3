"""Pins of the stage-split oracle: legal cut points of small hand-checked graphs, and the per-stage MAC integers of the
benchmark networks worked out block by block from the architectures (not by running the split)."""
import workloads as wl
from oracle import staging

N = wl.nets


def _conv(i, r=-1):
    return N.Layer(op=N.OP_CONV, c_in=4, c_out=4, k=1, in_from=i, res_from=r)


def test_legal_cuts_of_a_residual_toy():
    """L0 -> L1 -> L2 (+ L0's output as residual) -> L3 -> L4.  After L0 only L0's output crosses: legal.  After L1 two
    tensors cross (L1's output and L0's, still needed by L2's residual add): illegal.  After L2 and after L3: legal."""
    layers = [_conv(-1), _conv(0), _conv(1, 0), _conv(2), _conv(3)]
    assert staging.legal_cuts(layers) == [0, 2, 3]


def test_legal_cuts_with_two_readers_and_with_the_network_input_as_residual():
    # L1 and L2 both read L0 (a block's first convolution and its shortcut), L3 adds L1's output to conv(L2)
    layers = [_conv(-1), _conv(0), _conv(0), _conv(2, 1), _conv(3)]
    assert staging.legal_cuts(layers) == [0, 3]
    # a plain chain: every boundary is legal; the last layer is never followed by a cut
    assert staging.legal_cuts([_conv(-1), _conv(0), _conv(1)]) == [0, 1]
    # a later layer reading the network input itself (in_from = -1) forbids every cut before it
    assert staging.legal_cuts([_conv(-1), _conv(0), _conv(-1), _conv(2)]) == [2]


def test_split_ties_go_to_the_earliest_cuts_and_k_is_bounded():
    macs = [5, 0, 5, 0, 5]                      # zero-MAC layers (pools) between equal blocks: several optimal cut sets
    assert staging.split(macs, [0, 1, 2, 3], 3) == [0, 1, 3]        # cuts (0, 2) before (0, 3), (1, 2), (1, 3)
    assert staging.split(macs, [0, 1, 2, 3], 1) == [0]
    assert staging.split(macs, [1, 3], 4) is None
    assert staging.split([9, 1, 1, 9], [0, 1, 2], 2) == [0, 2]      # 11 | 9 beats 9 | 11 only by order: both cost 11


def _stages(net, k):
    layers, shp = wl.build_net(net)
    macs = wl.net_macs(layers, shp)
    first = staging.split(macs, staging.legal_cuts(layers), k)
    bounds = first + [len(layers)]
    return [layers[f].name for f in first], [sum(macs[a:b]) for a, b in zip(bounds, bounds[1:])]


def test_stage_macs_of_the_benchmark_networks():
    """Stage contents and MAC totals at the configured stage counts, block arithmetic done by hand:

    ResNet-18 (k=3).  stem 112*112*64*3*49 = 118,013,952; a 3x3 conv at 56x56x64->64 = 115,605,504 and the same at every
    later width (halved side, doubled channels) except a block's first conv after a stride (57,802,752) and its 1x1
    shortcut (6,422,528).  layer1 = 4 * 115,605,504; layer2 = layer3 = layer4 = 6,422,528 + 57,802,752 + 3 * 115,605,504
    = 411,041,792; first block of a layer 179,830,784, second 231,211,008; fc 512,000.
      stage 1 = stem + pool + layer1                 = 580,435,968
      stage 2 = layer2 + layer3 block 0              = 590,872,576
      stage 3 = layer3 block 1 + layer4 + gap + fc   = 642,764,800
    VGG-16 (k=3): c1 224*224*64*27 = 86,704,128; a 3x3 conv costs 1,849,688,064 at every width from c2 to c10 except the
    first one at a new width (c3, c5, c8: 924,844,032); c11..c13 462,422,016 each; FC 102,760,448 + 16,777,216 + 4,096,000.
    Cuts fall after c4 and after c8, and because a pool has no MACs the earliest of the equally good cut positions is
    taken, so the pool opens the next stage.
    """
    names, m = _stages("resnet18", 3)
    assert names == ["stem", "l2b0.ds", "l3b1.c1"]
    assert m == [580_435_968, 590_872_576, 642_764_800] and sum(m) == 1_814_073_344
    names, m = _stages("vgg16", 3)
    assert names == ["c1", "pool4", "c9"]
    # c1..c4 = 86,704,128 + 1,849,688,064 + 924,844,032 + 1,849,688,064; c5..c8 = 924,844,032 + 2 * 1,849,688,064 + 924,844,032;
    # c9..c13 + FC = 2 * 1,849,688,064 + 3 * 462,422,016 + 102,760,448 + 16,777,216 + 4,096,000
    assert m == [4_710_924_288, 5_549_064_192, 5_210_275_840] and sum(m) == 15_470_264_320
    names, m = _stages("resnet50", 4)
    assert names == ["stem", "l2b1.c1", "l3b1.c1", "l3b5.c1"]
    assert sum(m) == 4_089_184_256 and [round(v / 1e6) for v in m] == [1158, 1028, 873, 1030]
    names, m = _stages("mobilenet_v2", 3)
    assert sum(m) == 300_774_272 and [round(v / 1e6) for v in m] == [102, 108, 91]
    names, m = _stages("tiny", 2)
    # c1 + c2 = 1024*16*27 + 1024*32*144; the cut after c2 ties with the one after the pool that follows: earliest wins
    assert names == ["c1", "p1"] and m == [5_160_960, 7_118_848]
