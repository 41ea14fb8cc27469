"""Layer tables of the CNN shapes the paper serves on gpu-lets.

The paper's Table 4 lists GoogLeNet, LeNet, ResNet50, SSD-MobileNet and
VGG-16 with their input dimensions; its measurements (Fig. 3, Fig. 6) sweep
batch 1-32 over gpu-let sizes of 20-100%.  The trained networks and datasets
are replaced here by seeded random tensors of the same shapes, which is
enough because dense convolution timing does not depend on values.

A model is plain data: an ordered list of nodes reading and writing named
tensors.  Nothing here computes a shape or an output value; the CPU oracle
and the HIP model runner each interpret the table on their own.

Node kinds (all convolutions and pools are square):

  conv     src -> dst   C, K, k, stride, pad, relu, optional residual tensor
                        that is added before the ReLU
  dwconv   src -> dst   C, k, stride, pad, relu: one k x k filter per channel
  maxpool  src -> dst   k, stride, pad (padding never wins the max)
  gavgpool src -> dst   mean over the whole H x W plane
  fc       src -> dst   In, Out, relu; In is flattened from (C, H, W)
  concat   srcs -> dst  along channels
"""

from collections import namedtuple

from . import inputs

Node = namedtuple("Node", "op name src dst attr")
Model = namedtuple("Model", "name in_shape in_dist nodes out")


def _conv(name, src, dst, C, K, k, stride=1, pad=0, relu=True, residual=None):
    return Node("conv", name, src, dst,
                dict(C=C, K=K, k=k, stride=stride, pad=pad, relu=relu, residual=residual))


def _dwconv(name, src, dst, C, k, stride=1, pad=0, relu=True):
    return Node("dwconv", name, src, dst, dict(C=C, k=k, stride=stride, pad=pad, relu=relu))


def _maxpool(name, src, dst, k, stride, pad=0):
    return Node("maxpool", name, src, dst, dict(k=k, stride=stride, pad=pad))


def _gavg(name, src, dst):
    return Node("gavgpool", name, src, dst, {})


def _fc(name, src, dst, In, Out, relu):
    return Node("fc", name, src, dst, dict(In=In, Out=Out, relu=relu))


def _concat(name, srcs, dst):
    return Node("concat", name, tuple(srcs), dst, {})


def single_conv(C=256, K=256, H=14, W=14, k=3, stride=1, pad=1, relu=True):
    """One ResNet-50-style 3x3 convolution layer with bias and ReLU."""
    nodes = [_conv("conv", "x", "y", C, K, k, stride, pad, relu)]
    return Model("conv%dx%d_%d_%d_%d" % (k, k, C, K, H), (C, H, W), "normal", nodes, "y")


def lenet5():
    """LeNet-5 shape: 1x28x28 input (Table 4); the first convolution pads by
    2 so that the flattened feature vector has 16*5*5 = 400 entries."""
    nodes = [
        _conv("conv1", "x", "c1", 1, 6, 5, 1, 2, True),
        _maxpool("pool1", "c1", "p1", 2, 2),
        _conv("conv2", "p1", "c2", 6, 16, 5, 1, 0, True),
        _maxpool("pool2", "c2", "p2", 2, 2),
        _fc("fc1", "p2", "f1", 400, 120, True),
        _fc("fc2", "f1", "f2", 120, 84, True),
        _fc("fc3", "f2", "y", 84, 10, False),
    ]
    return Model("lenet5", (1, 28, 28), "normal", nodes, "y")


def vgg16(width_div=1, in_hw=224, n_class=1000):
    """VGG-16 shape: thirteen 3x3 pad-1 convolutions in five groups, each
    group followed by a 2x2/2 max pool, then three FC layers.  ``width_div``
    and ``in_hw`` shrink the model for quick tests."""
    cfg = [(64, 2), (128, 2), (256, 3), (512, 3), (512, 3)]
    nodes, src, C, hw, t = [], "x", 3, in_hw, 0
    for g, (K, reps) in enumerate(cfg, 1):
        K //= width_div
        for i in range(1, reps + 1):
            dst = "t%d" % t
            t += 1
            nodes.append(_conv("conv%d_%d" % (g, i), src, dst, C, K, 3, 1, 1, True))
            src, C = dst, K
        dst = "t%d" % t
        t += 1
        nodes.append(_maxpool("pool%d" % g, src, dst, 2, 2))
        src, hw = dst, hw // 2
    hidden = 4096 // width_div
    nodes.append(_fc("fc6", src, "f6", C * hw * hw, hidden, True))
    nodes.append(_fc("fc7", "f6", "f7", hidden, hidden, True))
    nodes.append(_fc("fc8", "f7", "y", hidden, n_class, False))
    return Model("vgg16" if width_div == 1 and in_hw == 224 else "vgg16_w%d_%d" % (width_div, in_hw),
                 (3, in_hw, in_hw), "uniform", nodes, "y")


def resnet50(width_div=1, in_hw=224, n_class=1000, blocks=(3, 4, 6, 3)):
    """ResNet-50 shape: 7x7/2 stem, 3x3/2 max pool, bottleneck stages of
    (1x1, 3x3, 1x1) convolutions with the stride-2 step on the 3x3 of the
    first block of stages 2-4, a 1x1 projection on the first shortcut of each
    stage, global average pool and FC.  Batch norm is taken as folded into the
    convolution weight and bias."""
    nodes = []
    w0 = 64 // width_div
    nodes.append(_conv("stem", "x", "s0", 3, w0, 7, 2, 3, True))
    nodes.append(_maxpool("stem_pool", "s0", "s1", 3, 2, 1))
    src, C = "s1", w0
    for s, reps in enumerate(blocks, 1):
        mid = (64 << (s - 1)) // width_div
        out = 4 * mid
        for b in range(reps):
            p = "l%d_%d" % (s, b)
            stride = 2 if (s > 1 and b == 0) else 1
            nodes.append(_conv(p + "_a", src, p + "_ta", C, mid, 1, 1, 0, True))
            nodes.append(_conv(p + "_b", p + "_ta", p + "_tb", mid, mid, 3, stride, 1, True))
            if b == 0:
                nodes.append(_conv(p + "_proj", src, p + "_sc", C, out, 1, stride, 0, False))
                shortcut = p + "_sc"
            else:
                shortcut = src
            nodes.append(_conv(p + "_c", p + "_tb", p + "_o", mid, out, 1, 1, 0, True,
                               residual=shortcut))
            src, C = p + "_o", out
    nodes.append(_gavg("avgpool", src, "gap"))
    nodes.append(_fc("fc", "gap", "y", C, n_class, False))
    full = width_div == 1 and in_hw == 224 and tuple(blocks) == (3, 4, 6, 3)
    return Model("resnet50" if full else "resnet50_w%d_%d" % (width_div, in_hw),
                 (3, in_hw, in_hw), "uniform", nodes, "y")


_INCEPTION = [
    # name, 1x1, 3x3 reduce, 3x3, 5x5 reduce, 5x5, pool projection
    ("3a", 64, 96, 128, 16, 32, 32),
    ("3b", 128, 128, 192, 32, 96, 64),
    ("4a", 192, 96, 208, 16, 48, 64),
    ("4b", 160, 112, 224, 24, 64, 64),
    ("4c", 128, 128, 256, 24, 64, 64),
    ("4d", 112, 144, 288, 32, 64, 64),
    ("4e", 256, 160, 320, 32, 128, 128),
    ("5a", 256, 160, 320, 32, 128, 128),
    ("5b", 384, 192, 384, 48, 128, 128),
]


def googlenet(width_div=1, in_hw=224, n_class=1000, n_blocks=9):
    """GoogLeNet shape: 7x7/2 stem, 1x1 and 3x3 convolutions, then inception
    blocks of four parallel branches (1x1 | 1x1->3x3 | 1x1->5x5 | 3x3 max
    pool->1x1) concatenated along channels; 3x3/2 pad-1 max pools before
    blocks 3a, 4a and 5a; global average pool and FC.  No auxiliary
    classifiers, no local response normalisation."""
    d = width_div
    nodes = [
        _conv("stem1", "x", "g0", 3, 64 // d, 7, 2, 3, True),
        _maxpool("pool1", "g0", "g1", 3, 2, 1),
        _conv("stem2", "g1", "g2", 64 // d, 64 // d, 1, 1, 0, True),
        _conv("stem3", "g2", "g3", 64 // d, 192 // d, 3, 1, 1, True),
        _maxpool("pool2", "g3", "g4", 3, 2, 1),
    ]
    src, C = "g4", 192 // d
    for name, c1, r3, c3, r5, c5, pp in _INCEPTION[:n_blocks]:
        c1, r3, c3, r5, c5, pp = (v // d for v in (c1, r3, c3, r5, c5, pp))
        if name in ("4a", "5a"):
            nodes.append(_maxpool("pool_" + name, src, "i%s_in" % name, 3, 2, 1))
            src = "i%s_in" % name
        p = "i" + name
        nodes.append(_conv(p + "_1x1", src, p + "_b1", C, c1, 1, 1, 0, True))
        nodes.append(_conv(p + "_3x3r", src, p + "_r3", C, r3, 1, 1, 0, True))
        nodes.append(_conv(p + "_3x3", p + "_r3", p + "_b2", r3, c3, 3, 1, 1, True))
        nodes.append(_conv(p + "_5x5r", src, p + "_r5", C, r5, 1, 1, 0, True))
        nodes.append(_conv(p + "_5x5", p + "_r5", p + "_b3", r5, c5, 5, 1, 2, True))
        nodes.append(_maxpool(p + "_pool", src, p + "_mp", 3, 1, 1))
        nodes.append(_conv(p + "_poolproj", p + "_mp", p + "_b4", C, pp, 1, 1, 0, True))
        nodes.append(_concat(p + "_cat", [p + "_b1", p + "_b2", p + "_b3", p + "_b4"], p + "_o"))
        src, C = p + "_o", c1 + c3 + c5 + pp
    nodes.append(_gavg("avgpool", src, "gap"))
    nodes.append(_fc("fc", "gap", "y", C, n_class, False))
    full = width_div == 1 and in_hw == 224 and n_blocks == 9
    return Model("googlenet" if full else "googlenet_w%d_%d_%d" % (width_div, in_hw, n_blocks),
                 (3, in_hw, in_hw), "uniform", nodes, "y")


def ssd_mobilenet(width_div=1, in_hw=300, n_class=91):
    """SSD-MobileNet shape (Table 4: camera data, 3x300x300): a MobileNet-v1
    backbone (3x3 stride-2 stem, 13 depthwise-separable blocks), four extra
    1x1 + 3x3 stride-2 feature stages and, on each of six feature maps, a 1x1
    box head (4 values per anchor) and a 1x1 class head (``n_class`` scores
    per anchor; 3 anchors on the first map, 6 on the others), concatenated
    per map.  ReLU stands in for ReLU6 and no box decoding follows: the
    workload is the dense part of the network.  The model's output tensor is
    the head of the last (smallest) map; the other heads are the named
    tensors ``head1`` .. ``head5``.  ``width_div`` and ``in_hw`` shrink it for
    CPU-sized tests."""
    d = width_div
    ch = lambda c: max(8, c // d)
    nodes = [_conv("stem", "x", "s0", 3, ch(32), 3, 2, 1, True)]
    src, C = "s0", ch(32)
    blocks = [(64, 1), (128, 2), (128, 1), (256, 2), (256, 1), (512, 2), (512, 1), (512, 1), (512, 1), (512, 1),
              (512, 1), (1024, 2), (1024, 1)]
    feats = []
    for i, (K, stride) in enumerate(blocks, 1):
        nodes.append(_dwconv("dw%d" % i, src, "d%d" % i, C, 3, stride, 1, True))
        nodes.append(_conv("pw%d" % i, "d%d" % i, "b%d" % i, C, ch(K), 1, 1, 0, True))
        src, C = "b%d" % i, ch(K)
        if i in (11, 13):
            feats.append((src, C))
    for j, (mid, K) in enumerate([(256, 512), (128, 256), (128, 256), (64, 128)], 1):
        nodes.append(_conv("extra%d_a" % j, src, "e%da" % j, C, ch(mid), 1, 1, 0, True))
        nodes.append(_conv("extra%d_b" % j, "e%da" % j, "e%db" % j, ch(mid), ch(K), 3, 2, 1, True))
        src, C = "e%db" % j, ch(K)
        feats.append((src, C))
    for m, (f, fc) in enumerate(feats, 1):
        anchors = 3 if m == 1 else 6
        nodes.append(_conv("box%d" % m, f, "box%d" % m, fc, 4 * anchors, 1, 1, 0, False))
        nodes.append(_conv("cls%d" % m, f, "cls%d" % m, fc, n_class * anchors, 1, 1, 0, False))
        nodes.append(_concat("head%d" % m, ["box%d" % m, "cls%d" % m], "y" if m == len(feats) else "head%d" % m))
    full = width_div == 1 and in_hw == 300 and n_class == 91
    return Model("ssd_mobilenet" if full else "ssd_mobilenet_w%d_%d_%d" % (width_div, in_hw, n_class),
                 (3, in_hw, in_hw), "uniform", nodes, "y")


def parameters(model, seed=0):
    """Seeded weights and biases of ``model``: ``{node name: (w, b)}`` with
    ``w`` in the canonical (K, C, R, S) / (Out, In) order, bfloat16-exact
    float32, and ``b`` float32."""
    out = {}
    for nd in model.nodes:
        if nd.op == "conv":
            a = nd.attr
            shape = (a["K"], a["C"], a["k"], a["k"])
        elif nd.op == "dwconv":
            a = nd.attr
            shape = (a["C"], 1, a["k"], a["k"])
        elif nd.op == "fc":
            shape = (nd.attr["Out"], nd.attr["In"])
        else:
            continue
        tag = "%s/%s" % (model.name, nd.name)
        out[nd.name] = (inputs.he_normal(seed, tag + ".w", shape),
                        inputs.bias(seed, tag + ".b", shape[0]))
    return out


def batch_input(model, batch, seed=0):
    """Seeded input batch in (N, C, H, W) order, bfloat16-exact float32:
    N(0, 1) or U(0, 1) as the model states."""
    return inputs.tensor(seed, "%s/input" % model.name, (batch,) + tuple(model.in_shape),
                         model.in_dist)
