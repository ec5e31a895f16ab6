"""Layer lists and DSP(p; m) schedules of the synthetic workloads (plain data).

A block of the split CNN is a list of layer dicts.  Layer ``i`` produces tensor
``i``; ``"in": -1`` names the block input h_k.  Ops:

  conv        cin, cout, r, s, stride, pad [, groups]  (cross-correlation, no bias; ``groups`` > 1: group g maps input
              channels [g cin/groups, (g+1) cin/groups) to output channels [g cout/groups, (g+1) cout/groups))
  bn          c, res (tensor index, -1, or None), relu   y = [relu](BN(x) [+ res])
  add         res (tensor index or -1)               y = x + res
  maxpool     k, stride, pad
  gap         global average pool over H, W
  linear      cin, cout                              z = W h + c
  softmax_ce  mean softmax cross-entropy over the mini-batch (last block only)

The architectures are the ones the benchmark configurations name in words:
CIFAR-style ResNets (3 stages, widths 16/32/64, post-activation basic blocks,
1x1 stride-2 projection shortcuts), a ResNet-18-style ImageNet net, the
conv4_x stage of a bottleneck ResNet-50 (stride on the 3x3), VGG-19 with
batch norm for 32x32 inputs, and the pre-activation bottleneck ResNet-164.  The schedules are
the first rows of the paper's accuracy table for each K:
DSP(1,0;2,0), DSP(1,1,0;4,2,0), DSP(1,1,1,0;6,4,2,0).
"""
from __future__ import annotations

import copy


# ----------------------------------------------------------------------------- builders
class _B:
    """Appends layers to a list and returns the new tensor index."""

    def __init__(self):
        self.layers = []

    def add(self, **kw):
        self.layers.append(kw)
        return len(self.layers) - 1

    def conv(self, src, cin, cout, k, stride=1, pad=None, groups=1):
        pad = (k // 2) if pad is None else pad
        kw = {"groups": groups} if groups > 1 else {}
        return self.add(op="conv", **{"in": src}, cin=cin, cout=cout, r=k, s=k, stride=stride, pad=pad, **kw)

    def resnext_unit(self, src, cin, width, cout, stride, cardinality):
        """Aggregated-transform bottleneck: 1x1 -> grouped 3x3 (``cardinality`` groups) -> 1x1, each followed by batch
        norm, projection shortcut (1x1 conv + BN) when the shape changes, ReLU after the sum."""
        a = self.conv(src, cin, width, 1, 1, pad=0)
        a = self.bn(a, width, relu=True)
        a = self.conv(a, width, width, 3, stride, groups=cardinality)
        a = self.bn(a, width, relu=True)
        a = self.conv(a, width, cout, 1, 1, pad=0)
        if stride != 1 or cin != cout:
            sc = self.conv(src, cin, cout, 1, stride, pad=0)
            sc = self.bn(sc, cout, relu=False)
        else:
            sc = src
        return self.bn(a, cout, relu=True, res=sc)

    def bn(self, src, c, relu=True, res=None):
        return self.add(op="bn", **{"in": src}, c=c, relu=relu, res=res)

    def basic(self, src, cin, cout, stride):
        a = self.conv(src, cin, cout, 3, stride)
        a = self.bn(a, cout, relu=True)
        a = self.conv(a, cout, cout, 3, 1)
        if stride != 1 or cin != cout:
            sc = self.conv(src, cin, cout, 1, stride, pad=0)
            sc = self.bn(sc, cout, relu=False)
        else:
            sc = src
        return self.bn(a, cout, relu=True, res=sc)

    def bottleneck(self, src, cin, mid, cout, stride):
        a = self.conv(src, cin, mid, 1, 1, pad=0)
        a = self.bn(a, mid, relu=True)
        a = self.conv(a, mid, mid, 3, stride)
        a = self.bn(a, mid, relu=True)
        a = self.conv(a, mid, cout, 1, 1, pad=0)
        if stride != 1 or cin != cout:
            sc = self.conv(src, cin, cout, 1, stride, pad=0)
            sc = self.bn(sc, cout, relu=False)
        else:
            sc = src
        return self.bn(a, cout, relu=True, res=sc)

    def preact_bottleneck(self, src, cin, mid, cout, stride):
        """Pre-activation bottleneck unit: BN-ReLU-conv three times, the shortcut added to the last conv's output;
        a unit that changes shape takes its 1x1 projection shortcut from the first activation."""
        t = self.bn(src, cin, relu=True)
        a = self.conv(t, cin, mid, 1, 1, pad=0)
        a = self.bn(a, mid, relu=True)
        a = self.conv(a, mid, mid, 3, stride)
        a = self.bn(a, mid, relu=True)
        a = self.conv(a, mid, cout, 1, 1, pad=0)
        sc = self.conv(t, cin, cout, 1, stride, pad=0) if (stride != 1 or cin != cout) else src
        return self.add(op="add", **{"in": a}, res=sc)

    def head(self, src, c, classes):
        a = self.add(op="gap", **{"in": src})
        a = self.add(op="linear", **{"in": a}, cin=c, cout=classes)
        return self.add(op="softmax_ce", **{"in": a})


def _tiny2():
    b0 = _B()
    a = b0.conv(-1, 3, 8, 3)
    b0.bn(a, 8)
    b1 = _B()
    a = b1.conv(-1, 8, 8, 3)
    a = b1.bn(a, 8)
    b1.head(a, 8, 10)
    return [b0.layers, b1.layers]


def _resnet_cifar(per_block_units, classes, widths=(16, 32, 64), units_per_stage=3):
    """CIFAR ResNet.  ``per_block_units``: number of basic blocks per DSP block."""
    seq = []  # (cin, cout, stride) of every basic block in order
    cin = widths[0]
    for si, w in enumerate(widths):
        for u in range(units_per_stage):
            seq.append((cin, w, 2 if (si > 0 and u == 0) else 1))
            cin = w
    assert sum(per_block_units) == len(seq)
    blocks, pos = [], 0
    for bi, cnt in enumerate(per_block_units):
        b = _B()
        src = -1
        if bi == 0:
            src = b.conv(-1, 3, widths[0], 3)
            src = b.bn(src, widths[0])
        for (ci, co, st) in seq[pos:pos + cnt]:
            src = b.basic(src, ci, co, st)
        pos += cnt
        if bi == len(per_block_units) - 1:
            b.head(src, widths[-1], classes)
        blocks.append(b.layers)
    return blocks


def _preact_resnet_cifar(per_block_units, classes, units_per_stage=18, widths=(16, 32, 64)):
    """Pre-activation bottleneck ResNet for 32x32 inputs (ResNet-164 with 18 units per stage): 3x3 stem conv,
    three stages of bottleneck units with 4x expansion, final BN-ReLU, global average pool, linear."""
    seq, cin = [], widths[0]
    for si, w in enumerate(widths):
        for u in range(units_per_stage):
            seq.append((cin, w, 4 * w, 2 if (si > 0 and u == 0) else 1))
            cin = 4 * w
    assert sum(per_block_units) == len(seq)
    blocks, pos = [], 0
    for bi, cnt in enumerate(per_block_units):
        b = _B()
        src = -1
        if bi == 0:
            src = b.conv(-1, 3, widths[0], 3)
        for (ci, mid, co, st) in seq[pos:pos + cnt]:
            src = b.preact_bottleneck(src, ci, mid, co, st)
        pos += cnt
        if bi == len(per_block_units) - 1:
            src = b.bn(src, 4 * widths[-1], relu=True)
            b.head(src, 4 * widths[-1], classes)
        blocks.append(b.layers)
    return blocks


def _resnext29(per_block_units, classes=10, cardinality=8, base_width=64, units_per_stage=3, out0=256):
    """ResNeXt-29 (cardinality x base_width d, e.g. 8 x 64d) for 32x32 inputs: 3x3 stem of 64 channels, three stages of
    three aggregated bottleneck units (grouped 3x3 of width cardinality * base_width * 2^stage, outputs 256 / 512 /
    1024 channels), global average pool, linear.  ``per_block_units``: units per DSP block."""
    seq, cin = [], 64
    for si in range(3):
        width, cout = cardinality * base_width * 2 ** si, out0 * 2 ** si
        for u in range(units_per_stage):
            seq.append((cin, width, cout, 2 if (si > 0 and u == 0) else 1))
            cin = cout
    assert sum(per_block_units) == len(seq)
    blocks, pos = [], 0
    for bi, cnt in enumerate(per_block_units):
        b = _B()
        src = -1
        if bi == 0:
            src = b.conv(-1, 3, 64, 3)
            src = b.bn(src, 64)
        for (ci, wd, co, st) in seq[pos:pos + cnt]:
            src = b.resnext_unit(src, ci, wd, co, st, cardinality)
        pos += cnt
        if bi == len(per_block_units) - 1:
            b.head(src, seq[-1][2], classes)
        blocks.append(b.layers)
    return blocks


def _resnet18(classes=1000):
    widths = (64, 128, 256, 512)
    blocks = []
    cin = 64
    for si, w in enumerate(widths):
        b = _B()
        src = -1
        if si == 0:
            src = b.conv(-1, 3, 64, 7, 2, pad=3)
            src = b.bn(src, 64)
            src = b.add(op="maxpool", **{"in": src}, k=3, stride=2, pad=1)
        for u in range(2):
            src = b.basic(src, cin, w, 2 if (si > 0 and u == 0) else 1)
            cin = w
        if si == len(widths) - 1:
            b.head(src, w, classes)
        blocks.append(b.layers)
    return blocks


def _resnet50_conv4x():
    b = _B()
    src = b.bottleneck(-1, 512, 256, 1024, 2)
    for _ in range(5):
        src = b.bottleneck(src, 1024, 256, 1024, 1)
    return [b.layers]


def _vgg19(classes=10, cuts=(6, 10)):
    """VGG-19 with batch norm for 32x32 inputs (16 conv layers, a 2x2 max pool after layers 2, 4, 8, 12, 16, then
    global average pool + one linear layer); ``cuts`` = index of the first conv layer of each later DSP block."""
    plan = [64, 64, "M", 128, 128, "M", 256, 256, 256, 256, "M", 512, 512, 512, 512, "M", 512, 512, 512, 512, "M"]
    blocks, b, src, cin, n_conv = [], _B(), -1, 3, 0
    for item in plan:
        if item == "M":
            src = b.add(op="maxpool", **{"in": src}, k=2, stride=2, pad=0)
            continue
        if n_conv in cuts:
            blocks.append(b.layers)
            b, src = _B(), -1
        src = b.conv(src, cin, item, 3)
        src = b.bn(src, item)
        cin = item
        n_conv += 1
    b.head(src, cin, classes)
    blocks.append(b.layers)
    return blocks


def _bn_probe():
    """Two 1x1 conv + BN(+ReLU) layers, the second with an identity shortcut from the block input: a cheap
    block whose normalisation layers can be checked against the oracle at ImageNet-sized feature maps."""
    b = _B()
    a = b.conv(-1, 64, 64, 1, 1, pad=0)
    a = b.bn(a, 64, relu=True)
    a = b.conv(a, 64, 64, 1, 1, pad=0)
    b.bn(a, 64, relu=True, res=-1)
    return [b.layers]


def _c64_probe():
    """One ResNet-18 stage-1 basic block (two 3x3 convolutions of 64 channels, identity shortcut): a block whose
    convolutions are large enough for the persistent filters-in-registers kernel, small enough for the oracle."""
    b = _B()
    a = b.conv(-1, 64, 64, 3)
    a = b.bn(a, 64, relu=True)
    a = b.conv(a, 64, 64, 3)
    b.bn(a, 64, relu=True, res=-1)
    return [b.layers]


def _stem_probe():
    """The ImageNet stem alone (7x7 / stride-2 convolution of the 3-channel image, batch norm + ReLU, 3x3 / stride-2 max
    pool) at its real map size: large enough for the stem's own convolution kernel and for the pool kernels that fold
    the batch norm in, with a batch small enough for the oracle."""
    b = _B()
    a = b.conv(-1, 3, 64, 7, 2, pad=3)
    a = b.bn(a, 64)
    b.add(op="maxpool", **{"in": a}, k=3, stride=2, pad=1)
    return [b.layers]


# ----------------------------------------------------------------------------- configs
CONFIGS = {
    # name: blocks, input (N, C, H, W), classes, DSP(p; m), lr, momentum, weight decay, steps, seed, dtype
    "tiny2": dict(blocks=_tiny2, input=(8, 3, 16, 16), classes=10, p=(1, 0), m=(2, 0),
                  lr=0.01, beta=0.9, wd=0.0, steps=4, seed=0, dtypes=("fp32",)),
    "resnet20": dict(blocks=lambda: _resnet_cifar((3, 3, 3), 10), input=(128, 3, 32, 32), classes=10,
                     p=(1, 1, 0), m=(4, 2, 0), lr=0.01, beta=0.9, wd=0.0, steps=50, seed=1, dtypes=("fp32",)),
    "resnet56": dict(blocks=lambda: _resnet_cifar((6, 7, 7, 7), 100, units_per_stage=9), input=(128, 3, 32, 32),
                     classes=100, p=(1, 1, 1, 0), m=(6, 4, 2, 0), lr=0.01, beta=0.9, wd=0.0, steps=50, seed=2,
                     dtypes=("fp32", "bf16")),
    "resnet50_conv4x": dict(blocks=_resnet50_conv4x, input=(64, 512, 28, 28), classes=None, p=(0,), m=(3,),
                            lr=0.01, beta=0.9, wd=0.0, steps=20, seed=3, dtypes=("bf16",), grad_std=0.1,
                            data_input=False),
    # one of the further networks the paper's speed-up table names (CIFAR, K = 3)
    "vgg19": dict(blocks=_vgg19, input=(128, 3, 32, 32), classes=10, p=(1, 1, 0), m=(4, 2, 0), lr=0.01, beta=0.9,
                  wd=0.0, steps=50, seed=6, dtypes=("fp32", "bf16")),
    # the network of the paper's gradient-difference and straggler experiments (CIFAR, K = 3)
    "resnet164": dict(blocks=lambda: _preact_resnet_cifar((18, 18, 18), 10), input=(128, 3, 32, 32), classes=10,
                      p=(1, 1, 0), m=(4, 2, 0), lr=0.01, beta=0.9, wd=0.0, steps=50, seed=7, dtypes=("fp32", "bf16")),
    # ResNet-1001 (111 bottleneck units per stage) on CIFAR-100 shapes, K = 4; units per block chosen so that the
    # blocks take about the same time (the 32x32 stage moves the most bytes per unit, every unit costs the same launches)
    "resnet1001": dict(blocks=lambda: _preact_resnet_cifar((70, 70, 95, 98), 100, units_per_stage=111),
                       input=(128, 3, 32, 32), classes=100, p=(1, 1, 1, 0), m=(6, 4, 2, 0), lr=0.01, beta=0.9, wd=0.0,
                       steps=20, seed=8, dtypes=("fp32", "bf16")),
    # ResNeXt-29 (8 x 64d), the grouped-convolution network of the paper's speed-up table (CIFAR-10, K = 4, batch 128)
    "resnext29": dict(blocks=lambda: _resnext29((2, 2, 2, 3)), input=(128, 3, 32, 32), classes=10, p=(1, 1, 1, 0),
                      m=(6, 4, 2, 0), lr=0.01, beta=0.9, wd=0.0, steps=20, seed=9, dtypes=("bf16", "fp32")),
    # the same graph with narrow channels, for finite differences and torch-autograd checks of the oracle (tests only)
    "resnext_tiny": dict(blocks=lambda: _resnext29((1, 2), cardinality=2, base_width=4, units_per_stage=1, out0=16),
                         input=(8, 3, 16, 16), classes=10, p=(1, 0), m=(2, 0), lr=0.01, beta=0.9, wd=0.0, steps=4, seed=10,
                         dtypes=("fp32",)),
    # not one of the paper-shaped workloads: a parity probe for the streaming kernels at large M (tests only)
    "bn_probe": dict(blocks=_bn_probe, input=(128, 64, 56, 56), classes=None, p=(0,), m=(1,), lr=0.01, beta=0.9,
                     wd=0.0, steps=3, seed=5, dtypes=("fp32", "bf16"), grad_std=0.1, data_input=False),
    # the same for the convolution kernel that only large 64-channel 3x3 layers take (M = 65856 rows: 258 tiles, the last
    # one ragged; forward + recompute in one launch, fused batch-norm sums, accumulating backward-data)
    "c64_probe": dict(blocks=_c64_probe, input=(21, 64, 56, 56), classes=None, p=(0,), m=(1,), lr=0.01, beta=0.9,
                      wd=0.0, steps=3, seed=6, dtypes=("bf16",), grad_std=0.1, data_input=False),
    # the ImageNet stem on 6 full-size images (M = 75264 output pixels of the convolution: 588 tiles of 128 for 512
    # workgroups; twin launches, fused sums, the pool with the batch norm folded in, forward and backward)
    "stem_probe": dict(blocks=_stem_probe, input=(6, 3, 224, 224), classes=None, p=(0,), m=(1,), lr=0.01, beta=0.9,
                       wd=0.0, steps=3, seed=7, dtypes=("bf16",), grad_std=0.1),
    # the same on 130 x 250 images: the stem's map is 65 x 125 -- the widest row its convolution kernel holds, odd in both
    # directions (the paths that need an even map fall back to the separate kernels), a ragged last tile (M = 73125)
    "stem_probe_wide": dict(blocks=_stem_probe, input=(9, 3, 130, 250), classes=None, p=(0,), m=(1,), lr=0.01, beta=0.9,
                            wd=0.0, steps=3, seed=8, dtypes=("bf16",), grad_std=0.1),
    "resnet18": dict(blocks=_resnet18, input=(256, 3, 224, 224), classes=1000, p=(1, 1, 1, 0), m=(6, 4, 2, 0),
                     lr=0.01, beta=0.9, wd=0.0, steps=20, seed=4, dtypes=("bf16",)),
}


def get_config(name, batch=None, hw=None):
    """Returns a materialised copy of a config; ``batch`` / ``hw`` shrink it for tests."""
    c = dict(CONFIGS[name])
    c["name"] = name
    c["blocks"] = copy.deepcopy(c["blocks"]())
    n, ch, h, w = c["input"]
    if batch is not None:
        n = batch
    if hw is not None:
        h = w = hw
    c["input"] = (n, ch, h, w)
    c["K"] = len(c["blocks"])
    return c


# ----------------------------------------------------------------------------- shape bookkeeping
def infer_shapes(layers, in_shape):
    """Output shape of every layer; (N,C,H,W) for maps, (N,C) after gap/linear, () for the loss."""
    shapes = []

    def sh(i):
        return in_shape if i == -1 else shapes[i]

    for L in layers:
        s = sh(L["in"])
        op = L["op"]
        if op == "conv":
            n, c, h, w = s
            assert c == L["cin"], (c, L)
            ho = (h + 2 * L["pad"] - L["r"]) // L["stride"] + 1
            wo = (w + 2 * L["pad"] - L["s"]) // L["stride"] + 1
            shapes.append((n, L["cout"], ho, wo))
        elif op == "bn":
            assert s[1] == L["c"]
            if L["res"] is not None:
                assert sh(L["res"]) == s, (sh(L["res"]), s)
            shapes.append(s)
        elif op == "add":
            assert sh(L["res"]) == s, (sh(L["res"]), s)
            shapes.append(s)
        elif op == "maxpool":
            n, c, h, w = s
            ho = (h + 2 * L["pad"] - L["k"]) // L["stride"] + 1
            wo = (w + 2 * L["pad"] - L["k"]) // L["stride"] + 1
            shapes.append((n, c, ho, wo))
        elif op == "gap":
            shapes.append((s[0], s[1]))
        elif op == "linear":
            assert s[1] == L["cin"]
            shapes.append((s[0], L["cout"]))
        elif op == "softmax_ce":
            shapes.append(())
        else:
            raise ValueError(op)
    return shapes


def block_output_shape(layers, in_shape):
    """Shape of h_{k+1}: the last tensor that is not the loss."""
    shapes = infer_shapes(layers, in_shape)
    for L, s in zip(reversed(layers), reversed(shapes)):
        if L["op"] != "softmax_ce":
            return s
    return in_shape


def param_shapes(layers):
    """Per layer, the ordered list of (name, shape) of its parameters."""
    out = []
    for L in layers:
        if L["op"] == "conv":
            out.append([("w", (L["cout"], L["cin"] // L.get("groups", 1), L["r"], L["s"]))])
        elif L["op"] == "bn":
            out.append([("gamma", (L["c"],)), ("beta", (L["c"],))])
        elif L["op"] == "linear":
            out.append([("w", (L["cout"], L["cin"])), ("c", (L["cout"],))])
        else:
            out.append([])
    return out


def count_macs(layers, in_shape):
    """Forward multiply-accumulates per image of the convolutions and the linear layer."""
    shapes = infer_shapes(layers, in_shape)
    macs = 0
    for L, s in zip(layers, shapes):
        if L["op"] == "conv":
            macs += s[1] * s[2] * s[3] * (L["cin"] // L.get("groups", 1)) * L["r"] * L["s"]
        elif L["op"] == "linear":
            macs += L["cin"] * L["cout"]
    return macs
