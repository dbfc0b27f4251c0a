"""GPU parity: the HIP library (through its C ABI) against the CPU fp64 oracle, element by element, on the
same seeded inputs.

Tolerances (stated by the benchmark spec): activations and loss within 1e-4, gradients and weights after 10 steps
within 1e-3, as max|gpu - ref| / max|ref| per tensor; the loss as a relative difference.

Sub-gradient choices.  ReLU and max-pool are kinks: an element whose pre-activation is closer to zero than
fp32 can resolve (a few 1e-6 after a K=500..4600 accumulation) may fall on either side, and with only
512..32768 elements per channel one such element moves that channel's gradient by 1/sqrt(count), far more
than 1e-3.  Both outcomes are correct gradients of the same continuous loss.  So the forward quantities are
compared directly, and for the backward pass the oracle is told which side the GPU took for every element
(rebuilt here bit for bit from the z, scale and shift tensors the library exposes: the kernels decide on
b = fmaf(z, scale, shift)); the oracle verifies that every choice differing from its own lies within 1e-4
of max|b| -- the activation tolerance -- and refuses anything else, then differentiates with those choices.
The tests bound what that lets through far below that margin: at most max(4, 4e-6 of all decisions) may differ
(none at all on the small blocks), and the farthest differing element must lie within 1e-5 of max|b| of the
kink, so a kernel whose b were off systematically would fail here long before the oracle's own margin.
Where 4e-6 comes from: an fp32 accumulation over K terms leaves z with a relative error of about sqrt(K) * 2^-24
(1.4e-6 for the 512-channel pointwise layers, K = 512 + 9), and over ten steps the two sides' weights drift apart
by a few 1e-6 relative, which moves b by as much; b is close to standard normal, so it lies within +-e of zero
with probability 0.8 e: up to about 0.8 * (1.4e-6 + 3e-6) = 3.5e-6 of the decisions.  Measured: at most 2.0e-6
(the 2x2x512 block of the five-block schedule after ten steps; 7e-8 on the 16x16 block), farthest 2.7e-6 of max|b|.
"""
from dataclasses import replace

import numpy as np
import pytest

from oracle import block as ob
from paper_2012_03096_amd import workloads as wl

pytestmark = pytest.mark.gpu

ACT_TOL = 1e-4
GRAD_TOL = 1e-3


def relerr(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if not np.all(np.isfinite(got)):
        return float("inf")
    d = np.abs(got - ref).max() if ref.size else 0.0
    return float(d / max(np.abs(ref).max(), 1e-30)) if ref.size else 0.0


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2012_03096_amd import binding
    binding.lib()
    return torch, binding


def _ref_block(w, tp, sp, **kw):
    return ob.RefBlock(w.teacher, tp, w.student, sp, momentum=w.momentum, **kw)


def _layer_act_shapes(arch):
    res = []
    for (ci, hi, wi, co, ho, wo), L in zip(wl.layer_shapes(arch), arch.layers):
        res.append(((arch.n, ci, ho, wo), (arch.n, co, ho, wo), L.kind))
    return res


def gpu_decisions(pb, blk, arch, x=None):
    """ReLU masks per layer and pool argmax as the GPU took them in its last student forward.
    x: the block input (fp32), needed when the block has an identity skip."""
    relu = []
    nl = len(arch.layers)
    b = None
    for l, (ushape, zshape, kind) in enumerate(_layer_act_shapes(arch)):
        c = zshape[1]

        def bn(layer):
            z = blk.get_tensor(pb.STUDENT_ACT, layer, 1, zshape).astype(np.float64)
            sc = blk.get_tensor(pb.STUDENT_ACT, layer, 4, (c,)).astype(np.float64)[None, :, None, None]
            sh = blk.get_tensor(pb.STUDENT_ACT, layer, 5, (c,)).astype(np.float64)[None, :, None, None]
            return (z * sc + sh).astype(np.float32)      # product exact in fp64: the sign is fmaf's sign

        b = bn(l)
        if l == nl - 1 and arch.shortcut == 1:
            b = b + bn(nl)                                # fp32 add, as in the kernel
        elif l == nl - 1 and arch.shortcut == 2:
            b = b + x.astype(np.float32)                  # identity skip: fmaf(x, 1, 0) = x, then the fp32 add
        relu.append(b > 0)
    pool_arg = None
    if arch.pool == 2:
        y = np.maximum(b, np.float32(0))
        N, C, H, W = y.shape
        Hp, Wp = H // 2, W // 2
        win = y[:, :, :2 * Hp, :2 * Wp].reshape(N, C, Hp, 2, Wp, 2).transpose(0, 1, 2, 4, 3, 5).reshape(N, C, Hp, Wp, 4)
        pool_arg = np.argmax(win, axis=-1)                # first maximum, like the kernel's strict '>'
    return {"relu": relu, "pool_arg": pool_arg}


DECISION_LOG = []
BN_DECAY = float(np.float32(0.9))
DIFFERING_FRACTION = 4e-6      # of all ReLU / pool decisions of a run may be taken differently from the oracle's own
DIFFERING_FLOOR = 4
DIFFERING_WORST_REL = 1e-5     # and each of those lies this close to the kink, as a fraction of max|b|


class DecisionTally:
    """Sums, over the steps of one run, what the oracle reports about the decisions it was handed."""

    def __init__(self):
        self.total = self.differing = 0
        self.worst_rel = 0.0

    def add(self, cache):
        self.total += cache["decisions_total"]
        self.differing += cache["decisions_differing"]
        self.worst_rel = max(self.worst_rel, cache["decisions_worst_rel"])

    def failures(self, none_allowed=False):
        out = {}
        allowed = 0 if none_allowed else max(DIFFERING_FLOOR, int(DIFFERING_FRACTION * self.total))
        if self.differing > allowed:
            out["decisions.differing"] = (self.differing, self.total, allowed)
        if self.worst_rel > DIFFERING_WORST_REL:
            out["decisions.worst_rel"] = self.worst_rel
        return out


def run_parity(gpu, w, steps, random_affine=True, loss_reduction=0, check_intermediates=True, x_override=None,
               no_differing_decisions=False):
    """Runs teacher forward + `steps` student steps on both sides and returns a dict of failures."""
    torch, pb = gpu
    x, tp, sp = w.tensors(random_affine=random_affine)
    if x_override is not None:
        x = x_override
    # a short memory for the running statistics, so that ten steps outweigh their starting values
    ref = _ref_block(w, tp, sp, loss_reduction=loss_reduction, bn_decay=BN_DECAY)
    blk = pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum, loss_reduction=loss_reduction, bn_decay=BN_DECAY)
    fails = {}

    def check(name, got, want, tol):
        e = relerr(got, want)
        if not e <= tol:
            fails[name] = e

    xd = torch.from_numpy(x).cuda()
    td = torch.empty(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda")
    t_ref, tcache = ob.block_forward(w.teacher, ref.tp, x, keep=True)
    blk.teacher_forward(xd, td)
    torch.cuda.synchronize()
    if check_intermediates:
        for l, (ushape, zshape, kind) in enumerate(_layer_act_shapes(w.teacher)):
            rec = tcache["layers"][l]
            check(f"teacher.z{l}", blk.get_tensor(pb.TEACHER_ACT, l, 1, zshape), rec["z"], ACT_TOL)
            check(f"teacher.mean{l}", blk.get_tensor(pb.TEACHER_ACT, l, 2, (zshape[1],)), rec["mean"], ACT_TOL)
            check(f"teacher.rstd{l}", blk.get_tensor(pb.TEACHER_ACT, l, 3, (zshape[1],)), rec["rstd"], ACT_TOL)
        if w.teacher.shortcut == 1:
            nl = len(w.teacher.layers)
            zs = tcache["layers"][-1]["zs"]
            check("teacher.zs", blk.get_tensor(pb.TEACHER_ACT, nl, 1, zs.shape), zs, ACT_TOL)
    check("teacher.target", td.cpu().numpy(), t_ref, ACT_TOL)

    # the student trains against the oracle's target rounded to fp32 on both sides, so that a teacher
    # discrepancy does not leak into the student comparison
    t32 = t_ref.astype(np.float32)
    td.copy_(torch.from_numpy(t32))
    out = torch.empty_like(td)
    blk.student_forward(xd, out)
    torch.cuda.synchronize()
    check("student.forward_out", out.cpu().numpy(), ref.student_forward(x), ACT_TOL)

    tally = DecisionTally()
    for step in range(steps):
        l_gpu = blk.student_step(xd, td, w.lr)
        l_ref = ref.student_step(x, t32, w.lr, decisions=gpu_decisions(pb, blk, w.student, x))
        tally.add(ref.cache)
        e = abs(l_gpu - l_ref) / max(abs(l_ref), 1e-30)
        if not e <= ACT_TOL:
            fails[f"loss[{step}]"] = (e, l_gpu, l_ref)
        if step == 0:
            assert abs(blk.last_loss() - l_gpu) == 0.0
            if check_intermediates:
                for l, (ushape, zshape, kind) in enumerate(_layer_act_shapes(w.student)):
                    rec = ref.cache["layers"][l]
                    if kind == wl.DWSEP3X3:
                        check(f"student.u{l}", blk.get_tensor(pb.STUDENT_ACT, l, 0, ushape), rec["u"], ACT_TOL)
                    check(f"student.z{l}", blk.get_tensor(pb.STUDENT_ACT, l, 1, zshape), rec["z"], ACT_TOL)
                    check(f"student.mean{l}", blk.get_tensor(pb.STUDENT_ACT, l, 2, (zshape[1],)), rec["mean"], ACT_TOL)
                    check(f"student.rstd{l}", blk.get_tensor(pb.STUDENT_ACT, l, 3, (zshape[1],)), rec["rstd"], ACT_TOL)
            grads = blk.student_grads()
            for l, L in enumerate(w.student.layers):
                if not L.trainable:
                    continue
                for k, (g_gpu, g_ref) in enumerate(zip(grads[l], ref.grads[l])):
                    check(f"grad[{l}][{k}]", g_gpu, g_ref, GRAD_TOL)
    params = blk.student_params()
    for l, (lp, lr_) in enumerate(zip(params, ref.sp)):
        for k, (a, b) in enumerate(zip(lp, lr_)):
            check(f"weights_after_{steps}[{l}][{k}]", a, b, GRAD_TOL)
    # running statistics: moved once per student step (not by the plain forward passes above), the teacher's never
    for l, (rm, rv) in enumerate(ref.s_running):
        c = rm.shape
        check(f"running_mean_after_{steps}[{l}]", blk.get_tensor(pb.STUDENT_BN_RUNNING, l, 0, c), rm, ACT_TOL)
        check(f"running_var_after_{steps}[{l}]", blk.get_tensor(pb.STUDENT_BN_RUNNING, l, 1, c), rv, ACT_TOL)
    for l, (rm, rv) in enumerate(ref.t_running):
        if not (np.all(blk.get_tensor(pb.TEACHER_BN_RUNNING, l, 0, rm.shape) == 0) and
                np.all(blk.get_tensor(pb.TEACHER_BN_RUNNING, l, 1, rm.shape) == 1)):
            fails[f"teacher_running[{l}]"] = "moved"
    blk.close()
    fails.update(tally.failures(none_allowed=no_differing_decisions))
    DECISION_LOG.append((w.name, steps, tally.differing, tally.total, tally.worst_rel))
    print(f"[parity] {w.name}: {steps} steps, {tally.differing} of {tally.total} decisions taken differently, "
          f"farthest from the kink {tally.worst_rel:.2e} of max|b|", flush=True)
    return fails


def test_cfg1_tiny_block_ten_steps(gpu):
    fails = run_parity(gpu, wl.cfg1_tiny(), steps=10, random_affine=False, no_differing_decisions=True)
    assert not fails, fails


@pytest.mark.parametrize("name", [w.name for w in wl.small_variants()])
def test_small_ragged_variants_ten_steps(gpu, name):
    w = {v.name: v for v in wl.small_variants()}[name]
    fails = run_parity(gpu, w, steps=10, no_differing_decisions=True)
    assert not fails, fails


@pytest.mark.parametrize("name", [w.name for w in wl.degenerate_variants()])
def test_degenerate_shapes_three_steps(gpu, name):
    """1x1 maps, single rows and columns, two channels, one image, pools and strides that end in one pixel."""
    w = {v.name: v for v in wl.degenerate_variants()}[name]
    fails = run_parity(gpu, w, steps=3, no_differing_decisions=True)
    assert not fails, fails


@pytest.mark.parametrize("fused", [1, 0])
@pytest.mark.parametrize("name", [w.name for w in wl.fused_forward_variants()])
def test_fused_depthwise_pointwise_forward(gpu, monkeypatch, name, fused):
    """The one-kernel depthwise + pointwise forward (PBKD_DWPW=1 takes it wherever the shape allows, 0 never) on small
    blocks ragged in batch and channels; depthwise outputs, pre-BatchNorm outputs, statistics, loss, gradients, weights."""
    monkeypatch.setenv("PBKD_DWPW", str(fused))
    w = {v.name: v for v in wl.fused_forward_variants()}[name]
    fails = run_parity(gpu, w, steps=5, no_differing_decisions=True)
    assert not fails, fails


def test_eq3_loss_reduction(gpu):
    w = wl.small_variants()[0]
    fails = run_parity(gpu, w, steps=3, loss_reduction=1)
    assert not fails, fails


def test_cfg2_vgg_block2_full_size(gpu):
    fails = run_parity(gpu, wl.cfg2_vgg_block2(), steps=10, random_affine=False)
    assert not fails, fails


def test_cfg3_resnet_down_full_size(gpu):
    fails = run_parity(gpu, wl.cfg3_resnet_down(), steps=10, random_affine=False)
    assert not fails, fails


def test_cfg4_imagenet_block_batch4_ten_steps(gpu):
    fails = run_parity(gpu, wl.cfg4_imagenet_vgg_block1(n=4), steps=10, random_affine=False)
    assert not fails, fails


def test_cfg4_imagenet_block_full_size_one_step(gpu):
    fails = run_parity(gpu, wl.cfg4_imagenet_vgg_block1(), steps=1, random_affine=False)
    assert not fails, fails


@pytest.mark.parametrize("k", range(13))
def test_paper_granularity_tasks(gpu, k):
    """Each of the thirteen per-convolution VGG16 tasks (one conv teacher, two DS layers student; section 4.4), batch 16."""
    tasks = wl.paper_granularity_vgg16_tasks(n=16)
    assert len(tasks) == 13
    fails = run_parity(gpu, tasks[k], steps=3)
    assert not fails, (tasks[k].name, fails)


def test_cfg4_shape_with_four_row_depthwise_strips_three_steps(gpu):
    """The ImageNet-shaped block at batch 11: the smallest batch at which the depthwise kernels take four rows per
    thread (N * H/4 * W/4 >= 32768 strips per channel), over several steps."""
    w = wl.cfg4_imagenet_vgg_block1(n=11)
    assert w.teacher.n * (w.teacher.h // 4) * (w.teacher.w // 4) >= 32768
    fails = run_parity(gpu, w, steps=3, random_affine=True)
    assert not fails, fails


@pytest.mark.parametrize("name", ["cfg2_batch16", "ragged_pool", "ragged_residual_s2", "fullconv_first"])
def test_large_mean_channels(gpu, name):
    """Block input 30 + N(0,1) instead of a post-ReLU map: every pre-BatchNorm channel of the first layers then has
    |mean| of the order of 30 standard deviations, where a one-pass variance E[z^2] - mean^2 loses (mean/sigma)^2 ~ 1e3
    times the rounding error of its sums.  The statistics, activations, loss and gradients must still meet the bounds."""
    w = wl.cfg2_vgg_block2(n=16) if name == "cfg2_batch16" else {v.name: v for v in wl.small_variants()}[name]
    rng = np.random.default_rng(30)
    x = (30.0 + rng.standard_normal((w.teacher.n, w.teacher.c, w.teacher.h, w.teacher.w))).astype(np.float32)
    fails = run_parity(gpu, w, steps=3, x_override=x)
    assert not fails, fails


FORCED = ([("PBKD_PW_VARIANT", v) for v in range(13)] + [("PBKD_CONV_TILE", v) for v in range(4)] +
          [("PBKD_WGRAD_VARIANT", v) for v in range(4)] + [("PBKD_CONV_KSPLIT", v) for v in (2, 3)])


@pytest.mark.parametrize("var,value", FORCED, ids=[f"{k[5:].lower()}{v}" for k, v in FORCED])
def test_every_tile_variant_on_ragged_blocks(gpu, monkeypatch, var, value):
    """The library picks tile shapes and kernel variants from the layer's shape; the benchmark shapes reach only some of
    them.  Its tuning overrides (read when a block is created) force each one in turn onto small blocks whose sizes are
    multiples of no tile: odd channel counts, 2x2 to 12x12 maps, pixel counts that leave ragged tails."""
    monkeypatch.setenv(var, str(value))
    by_name = {v.name: v for v in wl.small_variants()}
    for name in ("ragged_pool", "three_layers_oddc", "paper_task_2x2", "fullconv_first", "ragged_residual_s2"):
        fails = run_parity(gpu, by_name[name], steps=2, check_intermediates=(name == "three_layers_oddc"))
        assert not fails, (var, value, name, fails)


FIRST_LAYER_SWITCHES = [("PBKD_CF_TH", 4), ("PBKD_CF_TH", 8), ("PBKD_CF_OCC", 1), ("PBKD_CF_OCC", 6), ("PBKD_DW_EDGE", 0),
                        ("PBKD_DW_EDGE", 2), ("PBKD_WGRAD_BN_FUSED", 0)]


@pytest.mark.parametrize("var,value", FIRST_LAYER_SWITCHES, ids=[f"{k[5:].lower()}{v}" for k, v in FIRST_LAYER_SWITCHES])
def test_first_layer_and_depthwise_switches(gpu, monkeypatch, var, value):
    """Both tile heights and several grid sizes of the first-layer convolution, both ways the depthwise kernels get
    their edge columns on widths that do not fill 16-lane rows (12, 20, 36), and the first layer's weight gradient
    with and without its BatchNorm backward folded in (the default folds): each against the oracle on the blocks with a
    full first convolution (one, two and three input channels, a ragged second channel block, widths 12 to 36) and on
    two depthwise-only blocks."""
    monkeypatch.setenv(var, str(value))
    by_name = {v.name: v for v in wl.small_variants()}
    for name in ("fullconv_first", "fullconv_first_2ch", "fullconv_first_w36_70ch", "fullconv_first_w11", "ragged_pool", "wide_rows"):
        fails = run_parity(gpu, by_name[name], steps=3)
        assert not fails, (var, value, name, fails)


@pytest.mark.parametrize("split", [0, 1], ids=["fp32_mfma", "bf16_split"])
def test_teacher_convolution_both_arithmetics(gpu, monkeypatch, split):
    """The teacher's 3x3 convolutions through the fp32 MFMA kernel (PBKD_CONV_SPLIT=0) and through the bf16 MFMA
    kernel that splits every fp32 operand three ways (the default), each against the oracle at the activation
    tolerance: ragged channel counts (5, 7, 33, 40, 70: chunks of 8 with a zero-weight tail), stride 2, several images
    per pixel tile (2x2, 6x6, 8x8 maps), a K split (2x2 maps), tiles that end inside the image (9x11, 12x12), a
    projection shortcut beside it; stride 2 and rows of two tiles on widths the split kernel takes (12, 16, 40)."""
    monkeypatch.setenv("PBKD_CONV_SPLIT", str(split))
    by_name = {v.name: v for v in wl.small_variants()}
    for name in ("ragged_pool", "ragged_residual_s2", "three_layers_oddc", "paper_task_2x2", "two_layers_skip",
                 "second_layer_s2_w16", "fullconv_first_w36_70ch", "fullconv_first_7ch", "split_s2_first_w12",
                 "split_s2_second_w16", "split_two_tiles_w40"):
        fails = run_parity(gpu, by_name[name], steps=1)
        assert not fails, (split, name, fails)
    fails = run_parity(gpu, wl.cfg1_tiny(), steps=1)
    assert not fails, (split, fails)


def test_split_convolution_on_drawn_shapes(gpu):
    """Teacher forward of two-layer 3x3 blocks whose shapes are drawn (fixed seed) from what the bf16-split kernel takes:
    widths that are multiples of 4 up to 72 (rows of one to three tiles), heights 2 to 20, whole-image maps whose H*W is a
    multiple of 4 while the width is not (6x6, 2x14, 10x10), batches that leave the last pixel tile partly empty, 9 to 70
    input channels (ragged last chunk), stride 2 in either layer, with and without a projection shortcut."""
    torch, pb = gpu
    rng = np.random.default_rng(2024)
    shapes = [(6, 6), (2, 14), (10, 10)]
    while len(shapes) < 14:
        shapes.append((int(rng.integers(2, 21)), 4 * int(rng.integers(1, 19))))
    for k, (h, w_) in enumerate(shapes):
        n = int(rng.integers(1, 8))
        c0, c1, c2 = (int(rng.integers(9, 71)) for _ in range(3))
        s0 = 2 if (k % 4 == 1 and h >= 4 and w_ >= 8 and w_ % 8 == 0) else 1
        s1 = 2 if (k % 4 == 3 and h >= 4 and w_ >= 8 and w_ % 8 == 0) else 1
        sc = 1 if (k % 3 == 0) else 0
        layers = [wl.Layer(wl.CONV3X3, c0, c1, s0, 0), wl.Layer(wl.CONV3X3, c1, c2, s1, 0)]
        slayers = [wl.Layer(wl.DWSEP3X3, c0, c1, s0, 1), wl.Layer(wl.DWSEP3X3, c1, c2, s1, 1)]
        t = wl.Arch(n, c0, h, w_, layers, shortcut=sc, shortcut_stride=s0 * s1)
        s = wl.Arch(n, c0, h, w_, slayers, shortcut=sc, shortcut_stride=s0 * s1)
        wk = wl.Workload(f"drawn_{k}", t, s, seed=100 + k, copy_shortcut=bool(sc))
        x, tp, sp = wk.tensors(random_affine=True)
        t_ref, tcache = ob.block_forward(t, tp, x, keep=True)
        blk = pb.Block(t, tp, s, sp)
        xd = torch.from_numpy(x).cuda()
        td = torch.empty(wl.output_shape(t), dtype=torch.float32, device="cuda")
        blk.teacher_forward(xd, td)
        torch.cuda.synchronize()
        what = (k, n, c0, c1, c2, h, w_, s0, s1, sc)
        for l in range(2):
            rec = tcache["layers"][l]
            z = blk.get_tensor(pb.TEACHER_ACT, l, 1, rec["z"].shape)
            assert relerr(z, rec["z"]) <= ACT_TOL, (what, l, relerr(z, rec["z"]))
            assert relerr(blk.get_tensor(pb.TEACHER_ACT, l, 2, rec["mean"].shape), rec["mean"]) <= ACT_TOL, (what, l, "mean")
            assert relerr(blk.get_tensor(pb.TEACHER_ACT, l, 3, rec["rstd"].shape), rec["rstd"]) <= ACT_TOL, (what, l, "rstd")
        assert relerr(td.cpu().numpy(), t_ref) <= ACT_TOL, (what, "target")
        blk.close()


def test_teacher_weights_replaced_after_creation(gpu):
    """pbkd_block_set_tensor on a teacher's convolution weights re-packs them for whichever kernel the layer runs (the
    bf16-split kernel keeps three bf16 images of them): the forward pass then follows the new weights."""
    torch, pb = gpu
    w = wl.cfg1_tiny()
    x, tp, sp = w.tensors(random_affine=True)
    _, tp2, _ = replace(w, seed=w.seed + 7).tensors(random_affine=True)
    blk = pb.Block(w.teacher, tp, w.student, sp)
    for l in range(len(tp2)):
        blk.set_tensor(pb.TEACHER_PARAM, l, 0, tp2[l][0])           # the convolution weights only
    mixed = [[tp2[l][0]] + [a for a in tp[l][1:]] for l in range(len(tp))]
    t_ref = ob.block_forward(w.teacher, mixed, x)
    xd = torch.from_numpy(x).cuda()
    td = torch.empty(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda")
    blk.teacher_forward(xd, td)
    torch.cuda.synchronize()
    assert relerr(td.cpu().numpy(), t_ref) <= ACT_TOL
    blk.close()


def test_split_convolution_is_as_accurate_as_fp32(gpu, monkeypatch):
    """Six bf16 products of three-way split operands leave out terms of at most 2^-24 of each product, so against the fp64
    oracle the split kernel must not be worse than the fp32 MFMA kernel by more than rounding noise.  Two layers with
    long dot products (K = 9*128 and 9*256), BatchNorm between them, several workgroup tiles in a persistent grid."""
    torch, pb = gpu
    t = wl.Arch(24, 128, 16, 16, wl._convs([128, 256, 96]))
    s = wl.Arch(24, 128, 16, 16, wl._dws([128, 256, 96]))
    w = wl.Workload("accuracy_probe", t, s, seed=11)
    x, tp, sp = w.tensors(random_affine=True)
    t_ref, tcache = ob.block_forward(w.teacher, [[a.astype(np.float64) for a in lp] for lp in tp], x.astype(np.float64), keep=True)
    xd = torch.from_numpy(x).cuda()
    errs = {}
    for split in (0, 1):
        monkeypatch.setenv("PBKD_CONV_SPLIT", str(split))
        blk = pb.Block(w.teacher, tp, w.student, sp)
        td = torch.empty(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda")
        blk.teacher_forward(xd, td)
        torch.cuda.synchronize()
        e = []
        for l in range(2):
            z = blk.get_tensor(pb.TEACHER_ACT, l, 1, tcache["layers"][l]["z"].shape)
            e.append(relerr(z, tcache["layers"][l]["z"]))
        e.append(relerr(td.cpu().numpy(), t_ref))
        errs[split] = e
        blk.close()
    print(f"[split accuracy] max|err|/max|ref| of z0, z1, target: fp32 MFMA {errs[0]}, bf16 split {errs[1]}")
    for a, b in zip(errs[0], errs[1]):
        assert a <= ACT_TOL and b <= ACT_TOL, errs
        assert b <= 2.0 * a + 2e-7, errs


def test_zero_loss_when_student_is_the_factored_teacher(gpu):
    torch, pb = gpu
    chans = [6, 8, 5]
    t_arch = wl.Arch(3, 6, 8, 8, [wl.Layer(wl.CONV3X3, ci, co, 2 if i == 0 else 1, 0) for i, (ci, co) in enumerate(zip(chans[:-1], chans[1:]))],
                     shortcut=1, shortcut_stride=2, pool=2)
    s_arch = wl.Arch(3, 6, 8, 8, [wl.Layer(wl.DWSEP3X3, ci, co, 2 if i == 0 else 1, 1) for i, (ci, co) in enumerate(zip(chans[:-1], chans[1:]))],
                     shortcut=1, shortcut_stride=2, pool=2)
    sp = wl.make_params(s_arch, 1, True)
    tp = []
    for l in range(2):
        D, P, g, b = sp[l]
        tp.append([(P[:, :, None, None] * D[None, :, 0]).astype(np.float32), g.copy(), b.copy()])
    tp.append([q.copy() for q in sp[2]])
    x = wl.make_input(t_arch, 5)
    blk = pb.Block(t_arch, tp, s_arch, sp)
    xd = torch.from_numpy(x).cuda()
    td = torch.empty(wl.output_shape(t_arch), dtype=torch.float32, device="cuda")
    blk.teacher_forward(xd, td)
    loss = blk.student_step(xd, td, 0.1)
    # fp32 rounding of P*D and of two differently ordered sums: activations are O(1), so the mean squared
    # difference sits at the fp32 epsilon squared times a modest factor
    assert 0.0 <= loss < 1e-10, loss
    after = blk.student_params()
    for lp, lq in zip(after, sp):
        for a, b in zip(lp, lq):
            assert np.abs(a - b).max() < 1e-5
    blk.close()


def test_checkpoint_resume_is_bit_exact(gpu):
    torch, pb = gpu
    w = wl.small_variants()[1]
    x, tp, sp = w.tensors(random_affine=True)
    xd = torch.from_numpy(x).cuda()
    td = torch.empty(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda")
    a = pb.Block(w.teacher, tp, w.student, sp, momentum=0.9)
    a.teacher_forward(xd, td)
    for _ in range(10):
        a.student_step(xd, td, 0.02)
    ten = a.student_params()
    b = pb.Block(w.teacher, tp, w.student, sp, momentum=0.9)
    for _ in range(5):
        b.student_step(xd, td, 0.02)
    shapes = wl.param_shapes(w.student)
    saved_p = b.student_params()
    saved_v = [[b.get_tensor(pb.STUDENT_MOMENTUM, l, k, shp) for k, shp in enumerate(lp)] for l, lp in enumerate(shapes)]
    c = pb.Block(w.teacher, tp, w.student, sp, momentum=0.9)
    for l, lp in enumerate(shapes):
        for k, _ in enumerate(lp):
            c.set_tensor(pb.STUDENT_PARAM, l, k, saved_p[l][k])
            c.set_tensor(pb.STUDENT_MOMENTUM, l, k, saved_v[l][k])
    for _ in range(5):
        c.student_step(xd, td, 0.02)
    for lp, lq in zip(c.student_params(), ten):
        for p, q in zip(lp, lq):
            np.testing.assert_array_equal(p, q)
    for blk in (a, b, c):
        blk.close()


def test_create_errors(gpu):
    torch, pb = gpu
    import ctypes
    w = wl.cfg1_tiny()
    x, tp, sp = w.tensors()
    ta, sa = pb.make_arch(w.teacher), pb.make_arch(w.student)
    need = pb.workspace_bytes(w.teacher, w.student)
    ws = torch.empty(need + 512, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) & ~255
    tpa, k1 = pb._params_array(tp)
    spa, k2 = pb._params_array(sp)
    train = pb.TrainDesc(0.9, 0)
    h = ctypes.c_void_p()
    L = pb.lib()
    st = L.pbkd_block_create(ctypes.byref(ta), tpa, ctypes.byref(sa), spa, ctypes.byref(train), ctypes.c_void_p(base), need - 256,
                             None, ctypes.byref(h))
    assert st == pb.ENOMEM and "smaller" in pb.last_error()
    st = L.pbkd_block_create(ctypes.byref(ta), tpa, ctypes.byref(sa), spa, ctypes.byref(train), ctypes.c_void_p(base + 4), need,
                             None, ctypes.byref(h))
    assert st == pb.ENOMEM
    bad_train = pb.TrainDesc(1.5, 0)
    st = L.pbkd_block_create(ctypes.byref(ta), tpa, ctypes.byref(sa), spa, ctypes.byref(bad_train), ctypes.c_void_p(base), need,
                             None, ctypes.byref(h))
    assert st == pb.EINVAL
    st = L.pbkd_block_create(ctypes.byref(ta), tpa, ctypes.byref(sa), spa, ctypes.byref(train), ctypes.c_void_p(base), need,
                             None, ctypes.byref(h))
    assert st == pb.OK
    loss = ctypes.c_float()
    assert L.pbkd_block_last_loss(h, ctypes.byref(loss)) == pb.ESTATE
    assert L.pbkd_teacher_forward(h, None, None, None) == pb.EINVAL
    buf = np.empty(3, np.float32)
    assert L.pbkd_block_get_tensor(h, pb.STUDENT_PARAM, 0, 0, buf.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), 3) == pb.ESHAPE
    assert L.pbkd_block_get_tensor(h, pb.STUDENT_PARAM, 9, 0, buf.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), 3) == pb.EINVAL
    # running statistics have two slots; activations and gradients cannot be set
    c = np.empty(16, np.float32)
    cp = c.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
    assert L.pbkd_block_get_tensor(h, pb.STUDENT_BN_RUNNING, 0, 1, cp, 16) == pb.OK and np.all(c == 1)
    assert L.pbkd_block_get_tensor(h, pb.TEACHER_BN_RUNNING, 0, 2, cp, 16) == pb.EINVAL
    assert L.pbkd_block_set_tensor(h, pb.STUDENT_ACT, 0, 2, cp, 16) == pb.EINVAL
    assert L.pbkd_block_set_tensor(h, pb.STUDENT_GRAD, 0, 2, cp, 16) == pb.EINVAL
    # device tensors must be 16-byte aligned: refused before anything is launched
    xd = torch.zeros(4 * 16 * 16 * 16 + 4, dtype=torch.float32, device="cuda")
    td = torch.zeros(4 * 16 * 16 * 16 + 4, dtype=torch.float32, device="cuda")
    xp, tpd = ctypes.c_void_p(xd.data_ptr()), ctypes.c_void_p(td.data_ptr())
    xo, to = ctypes.c_void_p(xd.data_ptr() + 4), ctypes.c_void_p(td.data_ptr() + 4)
    assert L.pbkd_teacher_forward(h, xo, tpd, None) == pb.EINVAL and "aligned" in pb.last_error()
    assert L.pbkd_student_step(h, xp, to, ctypes.c_float(0.1), None, None) == pb.EINVAL
    assert L.pbkd_distill_step(h, xo, tpd, ctypes.c_float(0.1), None, None, None) == pb.EINVAL
    assert L.pbkd_block_last_loss(h, ctypes.byref(loss)) == pb.ESTATE      # none of the refused calls ran a step
    assert L.pbkd_teacher_forward(h, xp, tpd, None) == pb.OK
    torch.cuda.synchronize()
    L.pbkd_block_destroy(h)
    bad_decay = pb.TrainDesc(0.9, 0, 1.0)
    st = L.pbkd_block_create(ctypes.byref(ta), tpa, ctypes.byref(sa), spa, ctypes.byref(bad_decay), ctypes.c_void_p(base), need,
                             None, ctypes.byref(h))
    assert st == pb.EINVAL and "bn_decay" in pb.last_error()


def _all_blocks_setup(gpu, ws, tensors, n_streams, policy):
    torch, pb = gpu
    blocks = [pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum) for w, (x, tp, sp) in zip(ws, tensors)]
    x0 = torch.from_numpy(tensors[0][0]).cuda()
    ts = [torch.empty(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda") for w in ws]
    xs = [x0] + ts[:-1]
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    tstream = torch.cuda.Stream()
    sob, order, load = pb.schedule_blocks(None, n_streams, policy, blocks=blocks)
    torch.cuda.synchronize()
    return blocks, xs, ts, streams, tstream, sob, order


def test_all_vgg16_blocks_concurrently(gpu):
    """The whole CIFAR-shaped VGG16 at batch 128: the teacher chain feeds every block, the five student
    blocks train independently on three streams assigned by worst-fit-decreasing; ten steps against the
    oracle, and the result must not depend on the number of streams or the policy (blocks share nothing)."""
    torch, pb = gpu
    from oracle import schedule as osched
    ws = wl.cfg5_vgg16_blocks()
    tensors = [w.tensors() for w in ws]
    steps, lr = 10, 0.01
    tallies = [DecisionTally() for _ in ws]
    blocks, xs, ts, streams, tstream, sob, order = _all_blocks_setup(gpu, ws, tensors, 3, 0)
    weights = [osched.block_weight(w.teacher, w.student) for w in ws]
    assert sob == osched.wfd(weights, 3)[0]
    # oracle chain: block k's input is the fp32-rounded oracle output of block k-1
    refs, x_ref, t_ref = [], [], []
    x = tensors[0][0]
    for w, (_, tp, sp) in zip(ws, tensors):
        ref = ob.RefBlock(w.teacher, tp, w.student, sp, momentum=w.momentum)
        t = ref.teacher_forward(x)
        refs.append(ref); x_ref.append(x); t_ref.append(t)
        x = t.astype(np.float32)
    fails = {}
    losses = []
    for s in range(steps):
        pb.distill_step_all(blocks, xs, ts, lr, streams, sob, order, True, tstream)
        torch.cuda.synchronize()
        losses.append([b.last_loss() for b in blocks])
        for b, (w, ref) in enumerate(zip(ws, refs)):
            if s == 0:
                e = relerr(ts[b].cpu().numpy(), t_ref[b])
                if not e <= ACT_TOL:
                    fails[f"block{b}.target"] = e
            l_ref = ref.student_step(x_ref[b], t_ref[b].astype(np.float32), lr, decisions=gpu_decisions(pb, blocks[b], w.student))
            tallies[b].add(ref.cache)
            e = abs(losses[s][b] - l_ref) / abs(l_ref)
            if not e <= ACT_TOL:
                fails[f"block{b}.loss[{s}]"] = (e, losses[s][b], l_ref)
    params = [b.student_params() for b in blocks]
    for b, ref in enumerate(refs):
        for l, (lp, lr_) in enumerate(zip(params[b], ref.sp)):
            for k, (a, r) in enumerate(zip(lp, lr_)):
                e = relerr(a, r)
                if not e <= GRAD_TOL:
                    fails[f"block{b}.weights[{l}][{k}]"] = e
    for b in blocks:
        b.close()
    for b, tally in enumerate(tallies):
        print(f"[parity] cfg5 block {b}: {steps} steps, {tally.differing} of {tally.total} decisions taken differently, "
              f"farthest from the kink {tally.worst_rel:.2e} of max|b|", flush=True)
        for k, v in tally.failures().items():
            fails[f"block{b}.{k}"] = v
    assert not fails, fails
    # same work on one stream, round robin: bit-identical (deterministic reductions, no shared state)
    blocks1, xs1, ts1, streams1, tstream1, sob1, order1 = _all_blocks_setup(gpu, ws, tensors, 1, 1)
    losses1 = []
    for s in range(steps):
        pb.distill_step_all(blocks1, xs1, ts1, lr, streams1, sob1, order1, True, tstream1)
        losses1.append([b.last_loss() for b in blocks1])
    assert losses1 == losses
    for pa, blk1 in zip(params, blocks1):
        for lp, lq in zip(pa, blk1.student_params()):
            for a, c in zip(lp, lq):
                np.testing.assert_array_equal(a, c)
    for b in blocks1:
        b.close()
    # two sets of target buffers taken in turn and no host synchronisation between the steps: the next step's teacher
    # chain then runs ahead of this step's students (a teacher launch waits only for the steps that read the buffer it
    # overwrites); same bits again
    blocks2, xs2, ts2, streams2, tstream2, sob2, order2 = _all_blocks_setup(gpu, ws, tensors, 3, 0)
    ts2b = [torch.empty_like(t) for t in ts2]
    sets = [(xs2, ts2), ([xs2[0]] + ts2b[:-1], ts2b)]
    for s in range(steps):
        xs_, ts_ = sets[s % 2]
        pb.distill_step_all(blocks2, xs_, ts_, lr, streams2, sob2, order2, True, tstream2)
    torch.cuda.synchronize()
    assert [b.last_loss() for b in blocks2] == losses[-1]
    for pa, blk2 in zip(params, blocks2):
        for lp, lq in zip(pa, blk2.student_params()):
            for a, c in zip(lp, lq):
                np.testing.assert_array_equal(a, c)
    for b in blocks2:
        b.close()


def test_distill_step_on_two_streams_is_bit_identical(gpu, monkeypatch):
    """pbkd_distill_step overlaps teacher and student on two streams; its results must be those of
    pbkd_teacher_forward + pbkd_student_step on one stream, bit for bit, over several consecutive steps
    (the teacher of step i+1 runs while the student of step i is still in its backward pass), also with the teacher
    held back until the student step before the previous one has ended (PBKD_TEACHER_LAG=1)."""
    torch, pb = gpu
    w = wl.cfg2_vgg_block2()
    x, tp, sp = w.tensors()
    xd = torch.from_numpy(x).cuda()
    results = []
    for mode in ("one_stream", "two_streams", "two_streams_teacher_lag"):
        if mode == "two_streams_teacher_lag":
            monkeypatch.setenv("PBKD_TEACHER_LAG", "1")
        else:
            monkeypatch.delenv("PBKD_TEACHER_LAG", raising=False)
        blk = pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum)
        td = torch.zeros(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda")
        s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        if mode == "two_streams":
            blk.set_aux_stream(s3)      # weight gradients on a third stream
        torch.cuda.synchronize()
        losses = []
        for step in range(6):
            if mode != "one_stream":
                blk.distill_step(xd, td, w.lr, want_loss=False, student_stream=s1, teacher_stream=s2)
            else:
                blk.teacher_forward(xd, td, stream=s1)
                blk.student_step(xd, td, w.lr, want_loss=False, stream=s1)
            if step in (2, 5):
                losses.append(blk.last_loss())
        torch.cuda.synchronize()
        results.append((losses, [np.concatenate([a.ravel() for a in lp]) for lp in blk.student_params()], td.cpu().numpy()))
        blk.close()
    monkeypatch.delenv("PBKD_TEACHER_LAG", raising=False)
    l0, p0, t0 = results[0]
    for l1, p1, t1 in results[1:]:
        assert l0 == l1
        assert np.array_equal(t0, t1)
        for a, b in zip(p0, p1):
            assert np.array_equal(a, b)


@pytest.mark.parametrize("name", ["cfg1", "ragged_residual_s2", "three_layers_skip_pool", "cfg2"])
def test_graph_mode_replays_are_bit_identical_to_eager_steps(gpu, name):
    """pbkd_block_set_graph_mode: the captured step is replayed several times, with the program's own eager work and
    synchronisations between the replays, and every replay must leave exactly what the eager step leaves: losses, the
    teacher's target, and all weights.  One-stream steps (pbkd_teacher_forward + pbkd_student_step), the two-stream
    pbkd_distill_step, and a change of learning rate (a second capture) are all covered."""
    torch, pb = gpu
    w = {"cfg1": wl.cfg1_tiny(), "cfg2": wl.cfg2_vgg_block2(n=32)}.get(name) or {v.name: v for v in wl.small_variants()}[name]
    x, tp, sp = w.tensors(random_affine=True)
    xd = torch.from_numpy(x).cuda()
    lrs = [0.01, 0.01, 0.01, 0.02, 0.02, 0.01, 0.01]
    results = []
    for mode in ("eager", "graph_one_stream", "graph_two_streams"):
        blk = pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum)
        td = torch.zeros(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda")
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        blk.set_graph_mode(mode != "eager")
        torch.cuda.synchronize()
        losses, targets = [], []
        for step, lr in enumerate(lrs):
            if mode == "graph_two_streams":
                blk.distill_step(xd, td, lr, want_loss=False, student_stream=s1, teacher_stream=s2)
            else:
                blk.teacher_forward(xd, td, stream=s1)
                blk.student_step(xd, td, lr, want_loss=False, stream=s1)
            # eager work and a synchronisation between the replays
            losses.append(blk.last_loss())
            with torch.cuda.stream(s1):
                targets.append(float(td.double().sum().item()))
        torch.cuda.synchronize()
        results.append((losses, targets, [np.concatenate([a.ravel() for a in lp]) for lp in blk.student_params()],
                        [blk.get_tensor(pb.STUDENT_BN_RUNNING, 0, k, (w.student.layers[0].cout,)) for k in (0, 1)]))
        blk.close()
    ref = results[0]
    assert ref[0][0] != ref[0][-1]                      # the steps did train
    for got in results[1:]:
        assert got[0] == ref[0]
        assert got[1] == ref[1]
        for a, b in zip(got[2], ref[2]):
            assert np.array_equal(a, b)
        for a, b in zip(got[3], ref[3]):
            assert np.array_equal(a, b)


def test_graph_mode_all_block_step_is_bit_identical(gpu):
    """pbkd_distill_step_all with every block in graph mode: the whole teacher chain + five student steps as one
    graph, replayed with eager work between the replays, against the same steps issued eagerly (batch 16)."""
    torch, pb = gpu
    ws = wl.cfg5_vgg16_blocks(n=16)
    tensors = [w.tensors() for w in ws]
    out = []
    for graph in (False, True):
        blocks, xs, ts, streams, tstream, sob, order = _all_blocks_setup(gpu, ws, tensors, 3, 0)
        for b in blocks:
            b.set_graph_mode(graph)
        losses = []
        for s in range(5):
            pb.distill_step_all(blocks, xs, ts, 0.01, streams, sob, order, True, tstream)
            losses.append([b.last_loss() for b in blocks])
            with torch.cuda.stream(tstream):
                losses.append(float(ts[-1].double().sum().item()))
        torch.cuda.synchronize()
        out.append((losses, [[np.concatenate([a.ravel() for a in lp]) for lp in b.student_params()] for b in blocks]))
        # without a chain (every block its own stream, round robin), graph against eager as well
        xs2 = [x.clone() for x in xs]
        sob2, order2, _ = pb.schedule_blocks(None, 3, 1, blocks=blocks)
        for s in range(3):
            pb.distill_step_all(blocks, xs2, ts, 0.01, streams, sob2, order2, False, None)
        torch.cuda.synchronize()
        out[-1] = out[-1] + ([b.last_loss() for b in blocks],)
        for b in blocks:
            b.close()
    (l0, p0, n0), (l1, p1, n1) = out
    assert l0 == l1 and n0 == n1
    for pa, pb_ in zip(p0, p1):
        for a, b in zip(pa, pb_):
            assert np.array_equal(a, b)


def test_work_stealing_runs_every_task_once_with_identical_results(gpu):
    """pbkd_run_tasks_work_stealing (section 3.3): all tasks start in worker 0's queue, so the other workers
    must steal; whoever runs a task, its block ends with exactly the weights of the same steps run statically."""
    torch, pb = gpu
    ws = wl.small_variants()
    steps = [(3, 1, 4, 2, 5, 2, 1, 3)[i % 8] for i in range(len(ws))]

    def make():
        blocks, xs, ts = [], [], []
        for w in ws:
            x, tp, sp = w.tensors()
            blocks.append(pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum))
            xs.append(torch.from_numpy(x).cuda())
            ts.append(torch.empty(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda"))
        return blocks, xs, ts

    # static reference: every task on one stream, in order
    blocks, xs, ts = make()
    s0 = torch.cuda.Stream()
    for b, x, t, k, w in zip(blocks, xs, ts, steps, ws):
        for _ in range(k):
            b.teacher_forward(x, t, stream=s0)
            b.student_step(x, t, w.lr, want_loss=False, stream=s0)
    torch.cuda.synchronize()
    ref = [[np.concatenate([a.ravel() for a in lp]) for lp in b.student_params()] for b in blocks]
    ref_loss = [b.last_loss() for b in blocks]
    for b in blocks:
        b.close()

    blocks, xs, ts = make()
    streams = [torch.cuda.Stream() for _ in range(3)]
    torch.cuda.synchronize()
    ran_on, n_steals = pb.run_tasks_work_stealing(blocks, xs, ts, ws[0].lr, steps, streams, [0] * len(ws))
    assert all(0 <= r < 3 for r in ran_on)
    assert n_steals >= 1 and len(set(ran_on)) >= 2
    for b, r, rl in zip(blocks, ref, ref_loss):
        got = [np.concatenate([a.ravel() for a in lp]) for lp in b.student_params()]
        for a, c in zip(got, r):
            assert np.array_equal(a, c)
        assert b.last_loss() == rl
        b.close()


def test_reassembled_network_forward_and_feature_error(gpu):
    """pbkd_network_forward / pbkd_feature_mse (Algorithm 1's reassembly and its evaluation, label free): the five
    VGG16 blocks at batch 16 with their seeded weights on both sides; the network with no, some and all blocks
    replaced -- every block output and the feature error against the oracle."""
    torch, pb = gpu
    ws = wl.cfg5_vgg16_blocks(n=16)
    blocks, refs, ts = [], [], []
    x0 = None
    for i, w in enumerate(ws):
        x, tp, sp = w.tensors(random_affine=True)
        blocks.append(pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum))
        refs.append(_ref_block(w, tp, sp))
        if i == 0:
            x0 = x
        ts.append(torch.empty(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda"))
    xd = torch.from_numpy(x0).cuda()
    s = torch.cuda.Stream()
    t_ref = ob.network_forward(refs, [0] * 5, x0)
    outs = [torch.empty_like(t) for t in ts]
    pb.network_forward(blocks, [0] * 5, xd, ts, stream=s)
    for mask in ([0, 0, 0, 0, 0], [1, 0, 1, 0, 1], [0, 1, 0, 0, 0], [1, 1, 1, 1, 1]):
        pb.network_forward(blocks, mask, xd, outs, stream=s)
        torch.cuda.synchronize()
        want = ob.network_forward(refs, mask, x0)
        for k, (o, r) in enumerate(zip(outs, want)):
            e = relerr(o.cpu().numpy(), r)
            assert e <= ACT_TOL, (mask, k, e)
        got = pb.feature_mse(blocks[0], outs[-1], ts[-1], stream=s)
        ref = ob.feature_mse(want[-1], t_ref[-1])
        if ref == 0.0:
            assert got == 0.0, mask
        else:
            assert abs(got - ref) <= 1e-3 * ref, (mask, got, ref)
    # shapes that do not chain are refused
    with pytest.raises(Exception):
        pb.network_forward([blocks[0], blocks[2]], [0, 0], xd, [ts[0], ts[2]], stream=s)
    # inference mode: seeded running statistics on both sides (the teacher's come with its weights; the students'
    # stand for what training would have left), every mask again
    rng = np.random.default_rng(2012)
    for blk, ref in zip(blocks, refs):
        for kind, pairs in ((pb.TEACHER_BN_RUNNING, ref.t_running), (pb.STUDENT_BN_RUNNING, ref.s_running)):
            for l, pair in enumerate(pairs):
                pair[0] = (rng.normal(size=pair[0].shape) * 0.3).astype(np.float32).astype(np.float64)
                pair[1] = rng.uniform(0.5, 2.0, pair[1].shape).astype(np.float32).astype(np.float64)
                blk.set_tensor(kind, l, 0, pair[0])
                blk.set_tensor(kind, l, 1, pair[1])
    for mask in ([0, 0, 0, 0, 0], [1, 0, 1, 0, 1], [1, 1, 1, 1, 1]):
        pb.network_forward(blocks, mask, xd, outs, stream=s, bn_mode=1)
        torch.cuda.synchronize()
        want = ob.network_forward(refs, mask, x0, bn_mode=1)
        for k, (o, r) in enumerate(zip(outs, want)):
            e = relerr(o.cpu().numpy(), r)
            assert e <= ACT_TOL, ("inference", mask, k, e)
    # the batch-statistics forward still gives what it gave before, and the running pairs were only read
    pb.network_forward(blocks, [1, 0, 1, 0, 1], xd, outs, stream=s)
    torch.cuda.synchronize()
    want = ob.network_forward(refs, [1, 0, 1, 0, 1], x0)
    assert relerr(outs[-1].cpu().numpy(), want[-1]) <= ACT_TOL
    for blk, ref in zip(blocks, refs):
        for l, pair in enumerate(ref.s_running):
            assert np.array_equal(blk.get_tensor(pb.STUDENT_BN_RUNNING, l, 0, pair[0].shape), pair[0].astype(np.float32))
            assert np.array_equal(blk.get_tensor(pb.STUDENT_BN_RUNNING, l, 1, pair[1].shape), pair[1].astype(np.float32))
    with pytest.raises(Exception):
        pb.network_forward(blocks, [0] * 5, xd, outs, stream=s, bn_mode=2)
    # Algorithm 1's selection in both modes: per-block errors, the choice at a threshold inside the widest gap between
    # consecutive sorted errors (far from both of its ends), and the error of the network reassembled from the chosen blocks
    for mode in (0, 1):
        _, errs_ref, _ = ob.select_blocks(refs, x0, threshold=0.0, bn_mode=mode)
        srt = sorted(errs_ref)
        i = max(range(4), key=lambda j: srt[j + 1] / srt[j])
        assert srt[i + 1] > 1.1 * srt[i] > 0, srt
        thr = float(np.sqrt(srt[i] * srt[i + 1]))
        use_ref, _, final_ref = ob.select_blocks(refs, x0, threshold=thr, bn_mode=mode)
        use, errs, final = pb.select_blocks(blocks, xd, ts, outs, thr, stream=s, bn_mode=mode)
        assert use == use_ref and sum(use) == i + 1, (mode, use, use_ref)
        for k in range(5):
            assert abs(errs[k] - errs_ref[k]) <= 1e-3 * errs_ref[k], (mode, k, errs[k], errs_ref[k])
        assert abs(final - final_ref) <= 1e-3 * final_ref, (mode, final, final_ref)
    for b in blocks:
        b.close()
