"""Conv-layer shape lists for the synthetic workloads.

The paper evaluates whole trained CNNs (Table 4: MobileNetV2, ResNet-18,
ResNet-50, ... at 224x224 input, batch 1).  Only the *shapes* of their
convolution layers matter for the transform/execute trade-off (Section 3.1,
Table 2), so each workload here is the list of conv layers of such a network;
pooling, batch-norm, activations and residual adds are not modelled and every
layer gets its own random input of the right shape.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List


@dataclass(frozen=True)
class ConvLayer:
    """One 2-D convolution: x[n,c,h,w] (*) w[k,c/groups,r,s] -> y[n,k,p,q]."""
    name: str
    c: int
    h: int
    w: int
    k: int
    r: int
    s: int
    stride: int
    pad: int
    groups: int = 1
    n: int = 1

    @property
    def p(self) -> int:
        return (self.h + 2 * self.pad - self.r) // self.stride + 1

    @property
    def q(self) -> int:
        return (self.w + 2 * self.pad - self.s) // self.stride + 1

    @property
    def cg(self) -> int:
        """Input channels per group (second dim of the OIHW weight tensor)."""
        return self.c // self.groups

    @property
    def params(self) -> int:
        return self.k * self.cg * self.r * self.s

    @property
    def macs(self) -> int:
        return self.n * self.k * self.p * self.q * self.cg * self.r * self.s

    @property
    def is_depthwise(self) -> bool:
        return self.groups == self.c and self.groups == self.k and self.groups > 1

    @property
    def winograd_ok(self) -> bool:
        return (self.r == 3 and self.s == 3 and self.stride == 1 and self.groups == 1)


STACK_NAMES = ("single3x3", "resnet18", "mobilenetv2", "vgg16", "resnet50",
               "mobilenetv1", "squeezenet", "googlenet", "alexnet", "shufflenet_g3", "efficientnet_b0", "shufflenetv2_x1_5")


def _single() -> List[ConvLayer]:
    return [ConvLayer("conv3x3_16_32", 16, 32, 32, 16, 3, 3, 1, 1)]


def _resnet18() -> List[ConvLayer]:
    L = [ConvLayer("stem7x7", 3, 224, 224, 64, 7, 7, 2, 3)]
    # after the stem's 3x3/2 max-pool the feature map is 56x56
    for i in range(4):
        L.append(ConvLayer(f"l1_conv{i}", 64, 56, 56, 64, 3, 3, 1, 1))
    cin, hw = 64, 56
    for stage, width in ((2, 128), (3, 256), (4, 512)):
        L.append(ConvLayer(f"l{stage}_conv0_s2", cin, hw, hw, width, 3, 3, 2, 1))
        L.append(ConvLayer(f"l{stage}_down1x1_s2", cin, hw, hw, width, 1, 1, 2, 0))
        hw //= 2
        for i in range(1, 4):
            L.append(ConvLayer(f"l{stage}_conv{i}", width, hw, hw, width, 3, 3, 1, 1))
        cin = width
    return L


def _mobilenetv2() -> List[ConvLayer]:
    # (expansion t, output width c, repeats n, first stride s) of the published
    # inverted-residual schedule; 3x3/2 stem to 32 channels, final 1x1 to 1280.
    sched = ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
             (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1))
    L = [ConvLayer("stem3x3_s2", 3, 224, 224, 32, 3, 3, 2, 1)]
    cin, hw = 32, 112
    b = 0
    for t, cout, reps, s0 in sched:
        for i in range(reps):
            st = s0 if i == 0 else 1
            hid = cin * t
            if t != 1:
                L.append(ConvLayer(f"b{b}_expand", cin, hw, hw, hid, 1, 1, 1, 0))
            L.append(ConvLayer(f"b{b}_dw_s{st}", hid, hw, hw, hid, 3, 3, st, 1, groups=hid))
            hw = (hw + 2 - 3) // st + 1
            L.append(ConvLayer(f"b{b}_project", hid, hw, hw, cout, 1, 1, 1, 0))
            cin = cout
            b += 1
    L.append(ConvLayer("head1x1", cin, hw, hw, 1280, 1, 1, 1, 0))
    return L


def _vgg16() -> List[ConvLayer]:
    cfg = ((224, (64, 64)), (112, (128, 128)), (56, (256, 256, 256)),
           (28, (512, 512, 512)), (14, (512, 512, 512)))
    L, cin = [], 3
    for hw, widths in cfg:
        for i, wd in enumerate(widths):
            L.append(ConvLayer(f"conv{hw}_{i}", cin, hw, hw, wd, 3, 3, 1, 1))
            cin = wd
    return L


def _resnet50() -> List[ConvLayer]:
    # Bottleneck blocks; the stride of a stage's first block sits on its first
    # 1x1 conv, so every 3x3 conv has stride 1.
    L = [ConvLayer("stem7x7", 3, 224, 224, 64, 7, 7, 2, 3)]
    cin, hw = 64, 56
    for stage, (width, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3)), start=1):
        for b in range(blocks):
            st = 2 if (b == 0 and stage > 1) else 1
            hout = hw // st
            L.append(ConvLayer(f"s{stage}b{b}_reduce1x1", cin, hw, hw, width, 1, 1, st, 0))
            L.append(ConvLayer(f"s{stage}b{b}_conv3x3", width, hout, hout, width, 3, 3, 1, 1))
            L.append(ConvLayer(f"s{stage}b{b}_expand1x1", width, hout, hout, 4 * width, 1, 1, 1, 0))
            if b == 0:
                L.append(ConvLayer(f"s{stage}b{b}_down1x1", cin, hw, hw, 4 * width, 1, 1, st, 0))
            cin, hw = 4 * width, hout
    return L


def _mobilenetv1() -> List[ConvLayer]:
    # 3x3/2 stem to 32 channels, then 13 depthwise-separable blocks (output width, stride of
    # the depthwise 3x3), as published for the width-1.0, 224x224 network of Table 4.
    blocks = ((64, 1), (128, 2), (128, 1), (256, 2), (256, 1), (512, 2), (512, 1), (512, 1),
              (512, 1), (512, 1), (512, 1), (1024, 2), (1024, 1))
    L = [ConvLayer("stem3x3_s2", 3, 224, 224, 32, 3, 3, 2, 1)]
    cin, hw = 32, 112
    for b, (cout, st) in enumerate(blocks):
        L.append(ConvLayer(f"b{b}_dw_s{st}", cin, hw, hw, cin, 3, 3, st, 1, groups=cin))
        hw = (hw + 2 - 3) // st + 1
        L.append(ConvLayer(f"b{b}_pw", cin, hw, hw, cout, 1, 1, 1, 0))
        cin = cout
    return L


def _squeezenet() -> List[ConvLayer]:
    # The first published version (7x7/2 stem to 96 channels, eight fire modules, 1x1 classifier
    # conv), the one whose size matches Table 4's 1.4 M parameters; 3x3/2 max-pools (ceil mode)
    # after the stem, fire4 and fire8.  fire = 1x1 squeeze, then 1x1 and 3x3 expand side by side.
    fires = ((16, 64), (16, 64), (32, 128), None, (32, 128), (48, 192), (48, 192), (64, 256), None, (64, 256))
    L = [ConvLayer("conv1_7x7_s2", 3, 224, 224, 96, 7, 7, 2, 0)]
    hw = (224 - 7) // 2 + 1          # 109
    hw = -(-(hw - 3) // 2) + 1       # 54
    cin, f = 96, 2
    for spec in fires:
        if spec is None:
            hw = -(-(hw - 3) // 2) + 1
            continue
        sq, ex = spec
        L.append(ConvLayer(f"fire{f}_squeeze", cin, hw, hw, sq, 1, 1, 1, 0))
        L.append(ConvLayer(f"fire{f}_expand1x1", sq, hw, hw, ex, 1, 1, 1, 0))
        L.append(ConvLayer(f"fire{f}_expand3x3", sq, hw, hw, ex, 3, 3, 1, 1))
        cin, f = 2 * ex, f + 1
    L.append(ConvLayer("conv10_1x1", cin, hw, hw, 1000, 1, 1, 1, 0))
    return L


def _googlenet() -> List[ConvLayer]:
    # Stem (7x7/2, 1x1, 3x3) and nine inception modules with their published widths
    # (#1x1, #3x3 reduce, #3x3, #5x5 reduce, #5x5, pool projection); its 5x5 and 1x1 branches
    # are the shapes Fig. 5's kernel tree distinguishes by filter size.
    L = [ConvLayer("conv1_7x7_s2", 3, 224, 224, 64, 7, 7, 2, 3),
         ConvLayer("conv2_reduce", 64, 56, 56, 64, 1, 1, 1, 0),
         ConvLayer("conv2_3x3", 64, 56, 56, 192, 3, 3, 1, 1)]
    mods = (("3a", 28, 192, (64, 96, 128, 16, 32, 32)), ("3b", 28, 256, (128, 128, 192, 32, 96, 64)),
            ("4a", 14, 480, (192, 96, 208, 16, 48, 64)), ("4b", 14, 512, (160, 112, 224, 24, 64, 64)),
            ("4c", 14, 512, (128, 128, 256, 24, 64, 64)), ("4d", 14, 512, (112, 144, 288, 32, 64, 64)),
            ("4e", 14, 528, (256, 160, 320, 32, 128, 128)), ("5a", 7, 832, (256, 160, 320, 32, 128, 128)),
            ("5b", 7, 832, (384, 192, 384, 48, 128, 128)))
    for name, hw, cin, (n1, r3, n3, r5, n5, pp) in mods:
        L.append(ConvLayer(f"i{name}_1x1", cin, hw, hw, n1, 1, 1, 1, 0))
        L.append(ConvLayer(f"i{name}_3x3_reduce", cin, hw, hw, r3, 1, 1, 1, 0))
        L.append(ConvLayer(f"i{name}_3x3", r3, hw, hw, n3, 3, 3, 1, 1))
        L.append(ConvLayer(f"i{name}_5x5_reduce", cin, hw, hw, r5, 1, 1, 1, 0))
        L.append(ConvLayer(f"i{name}_5x5", r5, hw, hw, n5, 5, 5, 1, 2))
        L.append(ConvLayer(f"i{name}_pool_proj", cin, hw, hw, pp, 1, 1, 1, 0))
    return L


def _alexnet() -> List[ConvLayer]:
    # The single-tower variant (64, 192, 384, 256, 256 channels, no groups), the one whose size
    # matches Table 4's 61.3 M parameters and 1.4 GFLOPs: an 11x11/4 stem, a 5x5, three 3x3;
    # 3x3/2 max-pools after the first, second and fifth conv.
    return [ConvLayer("conv1_11x11_s4", 3, 224, 224, 64, 11, 11, 4, 2),
            ConvLayer("conv2_5x5", 64, 27, 27, 192, 5, 5, 1, 2),
            ConvLayer("conv3_3x3", 192, 13, 13, 384, 3, 3, 1, 1),
            ConvLayer("conv4_3x3", 384, 13, 13, 256, 3, 3, 1, 1),
            ConvLayer("conv5_3x3", 256, 13, 13, 256, 3, 3, 1, 1)]


def _shufflenet_g3() -> List[ConvLayer]:
    # The grouped-pointwise / depthwise units of the first ShuffleNet at width 1x with 3 groups:
    # 3x3/2 stem to 24 channels, max-pool, then stages of 4, 8, 4 units with 240, 480, 960
    # channels; a unit is 1x1 group conv to out/4 channels, 3x3 depthwise, 1x1 group conv; the
    # first unit of a stage has stride 2 and its second 1x1 produces out - in channels (the
    # rest comes from the pooled shortcut); the very first 1x1 is not grouped.
    L = [ConvLayer("stem3x3_s2", 3, 224, 224, 24, 3, 3, 2, 1)]
    cin, hw = 24, 56
    for stage, (cout, units) in enumerate(((240, 4), (480, 8), (960, 4)), start=2):
        mid = cout // 4
        for u in range(units):
            st = 2 if u == 0 else 1
            g1 = 1 if (stage == 2 and u == 0) else 3
            L.append(ConvLayer(f"s{stage}u{u}_pw1_g{g1}", cin, hw, hw, mid, 1, 1, 1, 0, groups=g1))
            L.append(ConvLayer(f"s{stage}u{u}_dw_s{st}", mid, hw, hw, mid, 3, 3, st, 1, groups=mid))
            hw = (hw + 2 - 3) // st + 1
            L.append(ConvLayer(f"s{stage}u{u}_pw2_g3", mid, hw, hw, cout - cin if u == 0 else cout, 1, 1, 1, 0, groups=3))
            cin = cout
    return L


def _efficientnet_b0() -> List[ConvLayer]:
    # Published B0 schedule (expansion, depthwise filter, stride, output width, repeats); every
    # block is [1x1 expand], k x k depthwise, squeeze-and-excitation (two 1x1 convs on the pooled
    # 1x1 map, squeezed to a quarter of the block's input width), 1x1 project; 1x1 head to 1280.
    sched = ((1, 3, 1, 16, 1), (6, 3, 2, 24, 2), (6, 5, 2, 40, 2), (6, 3, 2, 80, 3),
             (6, 5, 1, 112, 3), (6, 5, 2, 192, 4), (6, 3, 1, 320, 1))
    L = [ConvLayer("stem3x3_s2", 3, 224, 224, 32, 3, 3, 2, 1)]
    cin, hw, b = 32, 112, 0
    for t, k, s0, cout, reps in sched:
        for i in range(reps):
            st = s0 if i == 0 else 1
            hid = cin * t
            if t != 1:
                L.append(ConvLayer(f"b{b}_expand", cin, hw, hw, hid, 1, 1, 1, 0))
            L.append(ConvLayer(f"b{b}_dw{k}x{k}_s{st}", hid, hw, hw, hid, k, k, st, k // 2, groups=hid))
            hw = (hw + 2 * (k // 2) - k) // st + 1
            se = max(1, cin // 4)
            L.append(ConvLayer(f"b{b}_se_reduce", hid, 1, 1, se, 1, 1, 1, 0))
            L.append(ConvLayer(f"b{b}_se_expand", se, 1, 1, hid, 1, 1, 1, 0))
            L.append(ConvLayer(f"b{b}_project", hid, hw, hw, cout, 1, 1, 1, 0))
            cin = cout
            b += 1
    L.append(ConvLayer("head1x1", cin, hw, hw, 1280, 1, 1, 1, 0))
    return L


def _shufflenetv2_x1_5() -> List[ConvLayer]:
    # Second ShuffleNet at width 1.5x (the width whose size is closest to Table 4's 3.4 M
    # parameters): 3x3/2 stem to 24, max-pool, stages of 4, 8, 4 units with 176, 352, 704
    # channels, 1x1 conv to 1024.  A stride-1 unit splits the channels in two and runs
    # 1x1, 3x3 depthwise, 1x1 on one half; a stride-2 unit runs (3x3/2 depthwise, 1x1) on the
    # input and (1x1, 3x3/2 depthwise, 1x1) on the input again, each to half the output width.
    L = [ConvLayer("stem3x3_s2", 3, 224, 224, 24, 3, 3, 2, 1)]
    cin, hw = 24, 56
    for stage, (cout, units) in enumerate(((176, 4), (352, 8), (704, 4)), start=2):
        half = cout // 2
        L.append(ConvLayer(f"s{stage}u0_left_dw_s2", cin, hw, hw, cin, 3, 3, 2, 1, groups=cin))
        L.append(ConvLayer(f"s{stage}u0_left_pw", cin, hw // 2, hw // 2, half, 1, 1, 1, 0))
        L.append(ConvLayer(f"s{stage}u0_right_pw1", cin, hw, hw, half, 1, 1, 1, 0))
        L.append(ConvLayer(f"s{stage}u0_right_dw_s2", half, hw, hw, half, 3, 3, 2, 1, groups=half))
        hw //= 2
        L.append(ConvLayer(f"s{stage}u0_right_pw2", half, hw, hw, half, 1, 1, 1, 0))
        for u in range(1, units):
            L.append(ConvLayer(f"s{stage}u{u}_pw1", half, hw, hw, half, 1, 1, 1, 0))
            L.append(ConvLayer(f"s{stage}u{u}_dw", half, hw, hw, half, 3, 3, 1, 1, groups=half))
            L.append(ConvLayer(f"s{stage}u{u}_pw2", half, hw, hw, half, 1, 1, 1, 0))
        cin = cout
    L.append(ConvLayer("conv5_1x1", cin, hw, hw, 1024, 1, 1, 1, 0))
    return L


_BUILDERS = {"single3x3": _single, "resnet18": _resnet18, "mobilenetv2": _mobilenetv2,
             "vgg16": _vgg16, "resnet50": _resnet50, "mobilenetv1": _mobilenetv1,
             "squeezenet": _squeezenet, "googlenet": _googlenet, "alexnet": _alexnet,
             "shufflenet_g3": _shufflenet_g3, "efficientnet_b0": _efficientnet_b0,
             "shufflenetv2_x1_5": _shufflenetv2_x1_5}


def stack(name: str) -> List[ConvLayer]:
    """Layer list of one workload; `name` is one of STACK_NAMES."""
    return _BUILDERS[name]()


def table2_layer(hw: int = 56) -> ConvLayer:
    """A layer shaped like the one Table 2 times (3x3, stride 1, 64 -> 192
    channels); the paper does not state its spatial size, so `hw` is a guess."""
    return ConvLayer(f"table2_64to192_{hw}", 64, hw, hw, 192, 3, 3, 1, 1)
