"""Block descriptors and seeded synthetic inputs shared by the tests, the bench and the smoke run.

This module holds no arithmetic of the distillation method: it only *describes* blocks (which layers,
which shapes) and draws random tensors.  Both the CPU oracle and the HIP library receive the very same
fp32 arrays produced here, so input rounding never counts as an error between the two.

Recipe (one place, stated once):
  * block input x: standard normal, passed through max(.,0) where the workload says the input is a
    post-ReLU feature map; drawn from numpy default_rng(seed) as float64 and cast to float32;
  * teacher parameters: default_rng(1000 + seed); student parameters: default_rng(2000 + seed);
    draw order is layer by layer -- conv: W, gamma, beta; depthwise-separable: D, P, gamma, beta --
    then the shortcut W, gamma, beta;
  * weights are untruncated normal with variance 2 / fan_in (fan_in = 9*Cin for a full 3x3 conv,
    9 for a depthwise 3x3, Cin for a 1x1); gamma = 1 and beta = 0 unless `random_affine` asks for
    gamma ~ U(0.5, 1.5), beta ~ N(0, 0.1^2), which the tests use to exercise the affine terms.

The paper distils VGG16 / ResNet50 on CIFAR10 and ImageNet (section 4.1.3, 4.1.4); none of that data is
used here.  The workloads below take the *shapes* of those feature maps (32x32 and 224x224 images, the
VGG16 channel plan 64/128/256/512/512) and fill them with the random tensors just described.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence

import numpy as np

CONV3X3 = 0      # full 3x3 convolution, zero padding 1, + BatchNorm + ReLU
DWSEP3X3 = 1     # depthwise 3x3 (carries the stride) + pointwise 1x1, + BatchNorm + ReLU


@dataclass(frozen=True)
class Layer:
    kind: int
    cin: int
    cout: int
    stride: int = 1
    trainable: int = 1


@dataclass(frozen=True)
class Arch:
    """One block: input shape, layer list, optional 1x1 projection shortcut and 2x2 max-pool."""
    n: int
    c: int
    h: int
    w: int
    layers: Sequence[Layer]
    shortcut: int = 0           # 1: 1x1 conv (stride shortcut_stride) + BN, 2: the block input itself (identity
                                # skip, needs equal shapes); added before the last ReLU
    shortcut_stride: int = 1
    pool: int = 0               # 2: 2x2 max-pool, stride 2, after the last ReLU
    bn_eps: float = 1e-5

    def with_batch(self, n: int) -> "Arch":
        return replace(self, n=n)


def out_hw(h: int, w: int, stride: int):
    return (h - 1) // stride + 1, (w - 1) // stride + 1


def layer_shapes(arch: Arch):
    """[(cin, hin, win, cout, hout, wout)] per layer."""
    res = []
    c, h, w = arch.c, arch.h, arch.w
    for L in arch.layers:
        assert L.cin == c, "layer channel chain broken"
        ho, wo = out_hw(h, w, L.stride)
        res.append((c, h, w, L.cout, ho, wo))
        c, h, w = L.cout, ho, wo
    return res


def output_shape(arch: Arch):
    _, _, _, c, h, w = layer_shapes(arch)[-1]
    if arch.pool == 2:
        h, w = h // 2, w // 2
    return (arch.n, c, h, w)


def param_shapes(arch: Arch):
    """Per layer the list of parameter shapes, then the shortcut's (if any)."""
    res = []
    for L in arch.layers:
        if L.kind == CONV3X3:
            res.append([(L.cout, L.cin, 3, 3), (L.cout,), (L.cout,)])
        else:
            res.append([(L.cin, 1, 3, 3), (L.cout, L.cin), (L.cout,), (L.cout,)])
    if arch.shortcut == 1:
        co = arch.layers[-1].cout
        res.append([(co, arch.c), (co,), (co,)])
    return res


def _he(rng, shape, fan_in):
    return (rng.standard_normal(shape) * np.sqrt(2.0 / fan_in)).astype(np.float32)


def _affine(rng, c, random_affine):
    if random_affine:
        g = rng.uniform(0.5, 1.5, size=(c,)).astype(np.float32)
        b = (0.1 * rng.standard_normal((c,))).astype(np.float32)
    else:
        g = np.ones((c,), np.float32)
        b = np.zeros((c,), np.float32)
    return g, b


def make_params(arch: Arch, rng_seed: int, random_affine: bool = False) -> List[List[np.ndarray]]:
    rng = np.random.default_rng(rng_seed)
    out = []
    for L in arch.layers:
        if L.kind == CONV3X3:
            W = _he(rng, (L.cout, L.cin, 3, 3), 9 * L.cin)
            g, b = _affine(rng, L.cout, random_affine)
            out.append([W, g, b])
        else:
            D = _he(rng, (L.cin, 1, 3, 3), 9)
            P = _he(rng, (L.cout, L.cin), L.cin)
            g, b = _affine(rng, L.cout, random_affine)
            out.append([D, P, g, b])
    if arch.shortcut == 1:
        co = arch.layers[-1].cout
        Ws = _he(rng, (co, arch.c), arch.c)
        g, b = _affine(rng, co, random_affine)
        out.append([Ws, g, b])
    return out


def make_input(arch: Arch, seed: int, relu_input: bool = True) -> np.ndarray:
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((arch.n, arch.c, arch.h, arch.w))
    if relu_input:
        x = np.maximum(x, 0.0)
    return x.astype(np.float32)


@dataclass
class Workload:
    name: str
    teacher: Arch
    student: Arch
    seed: int
    relu_input: bool = True
    lr: float = 0.01
    momentum: float = 0.9
    steps: int = 10
    copy_shortcut: bool = False   # student shortcut = frozen copy of the teacher's

    def tensors(self, random_affine: bool = False):
        x = make_input(self.teacher, self.seed, self.relu_input)
        tp = make_params(self.teacher, 1000 + self.seed, random_affine)
        sp = make_params(self.student, 2000 + self.seed, random_affine)
        if self.copy_shortcut and self.teacher.shortcut == 1 and self.student.shortcut == 1:
            sp[-1] = [a.copy() for a in tp[-1]]
        return x, tp, sp

    def with_batch(self, n: int) -> "Workload":
        return replace(self, teacher=self.teacher.with_batch(n), student=self.student.with_batch(n))


def _convs(chans, stride0=1, trainable=0):
    return [Layer(CONV3X3, ci, co, stride0 if i == 0 else 1, trainable)
            for i, (ci, co) in enumerate(zip(chans[:-1], chans[1:]))]


def _dws(chans, stride0=1):
    return [Layer(DWSEP3X3, ci, co, stride0 if i == 0 else 1, 1)
            for i, (ci, co) in enumerate(zip(chans[:-1], chans[1:]))]


def cfg1_tiny() -> Workload:
    t = Arch(4, 16, 16, 16, _convs([16, 16, 16]))
    s = Arch(4, 16, 16, 16, _dws([16, 16, 16]))
    return Workload("cfg1_tiny_block", t, s, seed=0)


def cfg2_vgg_block2(n: int = 128) -> Workload:
    t = Arch(n, 64, 16, 16, _convs([64, 128, 128]), pool=2)
    s = Arch(n, 64, 16, 16, _dws([64, 128, 128]), pool=2)
    return Workload("cfg2_cifar_vgg16_block2", t, s, seed=1)


def cfg3_resnet_down(n: int = 128) -> Workload:
    t = Arch(n, 128, 16, 16, _convs([128, 256, 256], stride0=2), shortcut=1, shortcut_stride=2)
    s = Arch(n, 128, 16, 16, _dws([128, 256, 256], stride0=2), shortcut=1, shortcut_stride=2)
    return Workload("cfg3_cifar_resnet18_down", t, s, seed=2, copy_shortcut=True)


def cfg4_imagenet_vgg_block1(n: int = 32, hw: int = 224) -> Workload:
    t = Arch(n, 3, hw, hw, _convs([3, 64, 64]), pool=2)
    s = Arch(n, 3, hw, hw, [Layer(CONV3X3, 3, 64, 1, 1), Layer(DWSEP3X3, 64, 64, 1, 1)], pool=2)
    return Workload("cfg4_imagenet_vgg16_block1", t, s, seed=3, relu_input=False)


def degenerate_variants() -> List[Workload]:
    """The smallest shapes a block can have: 1x1 feature maps (a 3x3 window that sees only its centre), single
    rows, one channel, one image, a pool that leaves one pixel (and one that drops a row and a column to get there),
    a stride-2 layer whose output is one pixel wide."""
    v = []
    t = Arch(2, 3, 1, 1, _convs([3, 5, 4]))
    s = Arch(2, 3, 1, 1, _dws([3, 5, 4]))
    v.append(Workload("maps_1x1", t, s, seed=31))
    # (two channels, not one: a single-channel pointwise weight in front of a BatchNorm has an exactly zero gradient,
    # which leaves nothing to compare but rounding noise)
    t = Arch(1, 2, 5, 3, _convs([2, 2]))
    s = Arch(1, 2, 5, 3, _dws([2, 2, 2]))
    v.append(Workload("one_image_two_channels", t, s, seed=32))
    t = Arch(3, 2, 1, 7, _convs([2, 6, 6], stride0=2), shortcut=1, shortcut_stride=2)
    s = Arch(3, 2, 1, 7, _dws([2, 6, 6], stride0=2), shortcut=1, shortcut_stride=2)
    v.append(Workload("single_row_residual_s2", t, s, seed=33, copy_shortcut=True))
    t = Arch(4, 3, 3, 3, _convs([3, 4]), pool=2)
    s = Arch(4, 3, 3, 3, _dws([3, 4, 4]), pool=2)
    v.append(Workload("pool_3x3_to_1x1", t, s, seed=34))
    t = Arch(5, 4, 2, 1, _convs([4, 4], stride0=2))
    s = Arch(5, 4, 2, 1, _dws([4, 4], stride0=2), shortcut=0)
    v.append(Workload("column_s2_to_one_pixel", t, s, seed=35))
    return v


VGG16_PLAN = [[3, 64, 64], [64, 128, 128], [128, 256, 256, 256], [256, 512, 512, 512], [512, 512, 512, 512]]


def cfg5_vgg16_blocks(n: int = 128, hw: int = 32) -> List[Workload]:
    """The five VGG16 stages as five workloads; block k's input is block k-1's teacher output, so only
    block 1 draws an input -- the others' `tensors()` x is a placeholder of the right shape that callers
    replace with the teacher prefix output."""
    res = []
    h = hw
    for b, chans in enumerate(VGG16_PLAN):
        t = Arch(n, chans[0], h, h, _convs(chans), pool=2)
        if b == 0:
            sl = [Layer(CONV3X3, chans[0], chans[1], 1, 1)] + _dws(chans[1:])
        else:
            sl = _dws(chans)
        s = Arch(n, chans[0], h, h, sl, pool=2)
        res.append(Workload(f"cfg5_vgg16_block{b + 1}", t, s, seed=4 + 10 * b, relu_input=(b > 0)))
        h //= 2
    return res


def paper_granularity_vgg16_tasks(n: int = 128, hw: int = 32) -> List[Workload]:
    """One task per 3x3 convolution (13 for VGG16, section 3.3 / 4.4): the teacher task is a single
    conv + BN + ReLU, the student two depthwise-separable layers (section 3.2, candidate (a))."""
    res = []
    h = hw
    k = 0
    for b, chans in enumerate(VGG16_PLAN):
        for ci, co in zip(chans[:-1], chans[1:]):
            t = Arch(n, ci, h, h, _convs([ci, co]))
            s = Arch(n, ci, h, h, _dws([ci, co, co]))
            res.append(Workload(f"vgg16_conv{k + 1}", t, s, seed=100 + k, relu_input=(k > 0)))
            k += 1
        h //= 2
    return res


def small_variants() -> List[Workload]:
    """Small ragged blocks for element-by-element parity: sizes that are not multiples of any tile,
    stride 2, shortcut, pool, a trainable full first conv, odd channel counts."""
    v = []
    t = Arch(3, 5, 12, 12, _convs([5, 7, 6]), pool=2)
    s = Arch(3, 5, 12, 12, _dws([5, 7, 6]), pool=2)
    v.append(Workload("ragged_pool", t, s, seed=11))
    t = Arch(5, 6, 9, 11, _convs([6, 10, 10], stride0=2), shortcut=1, shortcut_stride=2)
    s = Arch(5, 6, 9, 11, _dws([6, 10, 10], stride0=2), shortcut=1, shortcut_stride=2)
    v.append(Workload("ragged_residual_s2", t, s, seed=12, copy_shortcut=True))
    t = Arch(2, 3, 20, 20, _convs([3, 8, 8]), pool=2)
    s = Arch(2, 3, 20, 20, [Layer(CONV3X3, 3, 8, 1, 1), Layer(DWSEP3X3, 8, 8, 1, 1)], pool=2)
    v.append(Workload("fullconv_first", t, s, seed=13, relu_input=False))
    t = Arch(7, 33, 6, 6, _convs([33, 40, 40, 17]))
    s = Arch(7, 33, 6, 6, _dws([33, 40, 40, 17]))
    v.append(Workload("three_layers_oddc", t, s, seed=14))
    t = Arch(9, 20, 2, 2, _convs([20, 24]))
    s = Arch(9, 20, 2, 2, _dws([20, 24, 24]))
    v.append(Workload("paper_task_2x2", t, s, seed=15))
    t = Arch(2, 4, 40, 36, _convs([4, 4]))
    s = Arch(2, 4, 40, 36, _dws([4, 4, 4]))
    v.append(Workload("wide_rows", t, s, seed=16))
    # section 3.2's candidates (c) and (d): two / three depthwise-separable layers with a skip connection
    t = Arch(6, 12, 10, 8, _convs([12, 12]))
    s = Arch(6, 12, 10, 8, _dws([12, 12, 12]), shortcut=2)
    v.append(Workload("two_layers_skip", t, s, seed=17))
    t = Arch(4, 8, 8, 8, _convs([8, 8]), pool=2)
    s = Arch(4, 8, 8, 8, _dws([8, 8, 8, 8]), shortcut=2, pool=2)
    v.append(Workload("three_layers_skip_pool", t, s, seed=18))
    # stride 2 on maps whose width is a multiple of 8 (the register-window stride-2 kernels): as the first layer of a
    # residual block, and as a later layer behind a BatchNorm
    t = Arch(3, 5, 6, 8, _convs([5, 7, 7], stride0=2), shortcut=1, shortcut_stride=2)
    s = Arch(3, 5, 6, 8, _dws([5, 7, 7], stride0=2), shortcut=1, shortcut_stride=2)
    v.append(Workload("residual_s2_w8", t, s, seed=19, copy_shortcut=True))
    # a trainable full first convolution with two and with seven input channels (9*Cin = 18 and 63 columns in the
    # matrix-core weight gradient; the first also takes the first-layer forward kernel), odd heights
    t = Arch(3, 2, 5, 12, _convs([2, 5, 5]))
    s = Arch(3, 2, 5, 12, [Layer(CONV3X3, 2, 5, 1, 1), Layer(DWSEP3X3, 5, 5, 1, 1)])
    v.append(Workload("fullconv_first_2ch", t, s, seed=21, relu_input=False))
    t = Arch(2, 7, 7, 8, _convs([7, 9, 9]), pool=2)
    s = Arch(2, 7, 7, 8, [Layer(CONV3X3, 7, 9, 1, 1), Layer(DWSEP3X3, 9, 9, 1, 1)], pool=2)
    v.append(Workload("fullconv_first_7ch", t, s, seed=22, relu_input=False))
    # three input channels on maps the first-layer forward kernel takes in pieces or not at all: a width of 36 (one
    # full tile column and a four-pixel rest) with 70 output channels (a second, ragged channel block), and an odd
    # width (the general kernel's case)
    t = Arch(2, 3, 9, 36, _convs([3, 70, 8]))
    s = Arch(2, 3, 9, 36, [Layer(CONV3X3, 3, 70, 1, 1), Layer(DWSEP3X3, 70, 8, 1, 1)])
    v.append(Workload("fullconv_first_w36_70ch", t, s, seed=23, relu_input=False))
    t = Arch(2, 3, 7, 11, _convs([3, 8, 8]))
    s = Arch(2, 3, 7, 11, [Layer(CONV3X3, 3, 8, 1, 1), Layer(DWSEP3X3, 8, 8, 1, 1)])
    v.append(Workload("fullconv_first_w11", t, s, seed=24, relu_input=False))
    t = Arch(5, 4, 4, 16, [Layer(CONV3X3, 4, 6, 1, 0), Layer(CONV3X3, 6, 6, 2, 0)])
    s = Arch(5, 4, 4, 16, [Layer(DWSEP3X3, 4, 6, 1, 1), Layer(DWSEP3X3, 6, 6, 2, 1)])
    v.append(Workload("second_layer_s2_w16", t, s, seed=20))
    # shapes the teacher's bf16-split convolution takes (width a multiple of 4, more than 8 input channels): stride 2 as
    # first and as second layer with ragged channel counts and a projection shortcut; a 40-wide map whose rows take two
    # tiles (the staged rows then start four columns left of a tile), 5 images so that the last tile holds one
    t = Arch(5, 12, 10, 12, _convs([12, 20, 20], stride0=2), shortcut=1, shortcut_stride=2)
    s = Arch(5, 12, 10, 12, _dws([12, 20, 20], stride0=2), shortcut=1, shortcut_stride=2)
    v.append(Workload("split_s2_first_w12", t, s, seed=25, copy_shortcut=True))
    t = Arch(3, 9, 8, 16, [Layer(CONV3X3, 9, 17, 1, 0), Layer(CONV3X3, 17, 11, 2, 0)])
    s = Arch(3, 9, 8, 16, [Layer(DWSEP3X3, 9, 17, 1, 1), Layer(DWSEP3X3, 17, 11, 2, 1)])
    v.append(Workload("split_s2_second_w16", t, s, seed=26))
    t = Arch(5, 10, 6, 40, _convs([10, 12, 9]))
    s = Arch(5, 10, 6, 40, _dws([10, 12, 9]))
    v.append(Workload("split_two_tiles_w40", t, s, seed=27))
    return v


def fused_forward_variants() -> List[Workload]:
    """Small blocks whose depthwise-separable layers have shapes the one-kernel depthwise + pointwise forward accepts
    (stride 1, height a multiple of 4, width 4, 8, 16 or a multiple of 32), chosen to be ragged in everything else:
    batches that leave a tile's last images empty, channel counts that are multiples of no stage, more than one tile
    of output channels, both workgroup shapes (at most 64 output channels / more)."""
    v = []
    t = Arch(3, 5, 8, 8, _convs([5, 7, 6]))
    s = Arch(3, 5, 8, 8, _dws([5, 7, 6]))
    v.append(Workload("fused_8x8_ragged_batch", t, s, seed=41))
    t = Arch(2, 37, 12, 32, _convs([37, 130, 40]), pool=2)
    s = Arch(2, 37, 12, 32, _dws([37, 130, 40]), pool=2)
    v.append(Workload("fused_12x32_two_channel_tiles", t, s, seed=42))
    t = Arch(9, 12, 4, 4, _convs([12, 12]))
    s = Arch(9, 12, 4, 4, _dws([12, 12, 12]), shortcut=2)
    v.append(Workload("fused_4x4_skip", t, s, seed=43))
    t = Arch(2, 3, 16, 16, _convs([3, 8, 8]), pool=2)
    s = Arch(2, 3, 16, 16, [Layer(CONV3X3, 3, 8, 1, 1), Layer(DWSEP3X3, 8, 8, 1, 1)], pool=2)
    v.append(Workload("fused_16x16_fullconv_first", t, s, seed=44, relu_input=False))
    t = Arch(3, 70, 8, 64, _convs([70, 96]))
    s = Arch(3, 70, 8, 64, _dws([70, 66, 96]))
    v.append(Workload("fused_8x64_three_stages", t, s, seed=45))
    return v
