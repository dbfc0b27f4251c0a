"""CPU oracle for the per-block distillation step: block composition, loss, backward, SGD-momentum.

TEST INFRASTRUCTURE ONLY -- imported by tests/, by the smoke check and by the bench's cpu_baseline leg;
never by the product path.  It shares no code with the HIP library and does not import the package.

The method is an iteration (SGD on a local regression loss), so this file takes its steps in the
paper's order, in fp64, on the fp32-rounded inputs and weights the GPU receives:

  1. teacher block forward  t = f_k(x)                       (section 3.1, Eq. 1; the label of Eq. 3)
  2. student block forward  p = g_k(x) on the same input     (section 3.1; layer = depthwise separable
                                                              + batch norm + ReLU, section 3.2)
  3. local loss             L = mean (p - t)^2               (Eq. 3, see reading R1)
  4. backward through the student block only                 (section 3.3: only the replacement
                                                              block's few layers need gradients)
  5. v <- mu*v + g ; theta <- theta - lr*v                   (optimizer unspecified in the paper, R2/R3)

The convolution / BatchNorm loops are the C primitives of pbkd_ref.c (direct definitions); everything
elementwise (ReLU, add, max-pool, loss) is numpy.

Readings taken where the paper is silent, ambiguous or garbled (each is a descriptor field or an
argument, not a hidden assumption):
  R1  loss normalisation: Eq. 3 divides the summed squared norm by the number of images.  Default here
      is the mean over all N*C*H*W output elements ("MSE"); loss_reduction=1 gives Eq. 3's form
      sum/N.  They differ by the constant C*H*W.
  R2  optimizer: plain SGD with momentum; lr and momentum are arguments.
  R3  momentum form: v0 = 0; v <- mu*v + g; theta <- theta - lr*v; no dampening, Nesterov or decay;
      applied alike to every trainable tensor (conv/depthwise/pointwise weights, gamma, beta).
  R4  BatchNorm in training mode for teacher and student: batch mean, biased batch variance over
      (N,H,W), eps inside the square root; backward differentiates through mean and variance.
  R5  no convolution bias anywhere (train-mode BN cancels it).
  R6  3x3: cross-correlation, zero padding 1 on all sides at every stride; 1x1 shortcut: pad 0.
  R7  inside a depthwise-separable layer there is nothing between the depthwise and the pointwise
      convolution (no BN, no ReLU, no bias).
  R8  a block is a list of layers, each conv (full or depthwise-separable) + BN + ReLU; with a
      projection shortcut the branch 1x1 conv(stride) + BN is added to the last layer's BN output
      before the last ReLU; an optional 2x2/stride-2 max-pool follows the last ReLU.
  R9  a frozen layer (trainable=0) takes part in forward and backward but receives no update.
  R10 ReLU'(b) = 1 for b > 0 and 0 otherwise; the max-pool gradient goes to the first maximum of the
      window in row-major order; odd spatial sizes under the pool drop the last row/column.
  R11 depthwise convolution acts on the layer's input channels, the pointwise maps Cin -> Cout.
  R13 sub-gradient choice at the kinks.  ReLU and max-pool make the loss piecewise smooth; an element
      whose pre-activation b (or whose gap between the two largest window entries) is smaller than the
      accuracy to which b itself is required (1e-4 of max|b|, the activation tolerance) can legitimately
      fall on either side in an fp32 implementation, and each side gives a different, equally valid
      gradient.  Forward values and the loss are unaffected (they are continuous).  For the backward
      pass the caller may therefore pass `decisions` = the ReLU on/off mask per layer and the pool
      argmax; the oracle VERIFIES that every entry differing from its own fp64 decision lies within
      that margin (it raises otherwise) and then differentiates with the given choices.  Without
      `decisions` it uses its own (R10).
  R12 scheduler weight of a block = teacher forward FLOPs + student step FLOPs, counting 2*MACs of
      the convolutions only (see schedule.py).
  R14 the candidate blocks with residual-style skip connections (section 3.2, candidates
      (c) and (d); their figure is missing): the block input itself is added to the last layer's
      BatchNorm output before the last ReLU (`shortcut = 2`); it needs equal input and output shapes
      and has no parameters.  The block input needs no gradient, so the skip changes the backward pass
      only through the last ReLU's mask.
  R15 inference-mode BatchNorm for the reassembled network (Algorithm 1's last loop runs the network to
      evaluate it; the paper's TensorFlow layers then use moving averages, about which it says nothing):
      every BatchNorm keeps a running mean (starts at 0) and a running variance (starts at 1); each
      student step moves those of EVERY student BatchNorm (frozen layers and the projection shortcut
      included, since they too normalise with batch statistics while training, R4) by
      running <- decay*running + (1-decay)*batch, with the batch mean and the BIASED batch variance of
      that step's forward pass; the teacher's are given with its weights.  In inference mode
      b = gamma*(z - running_mean)/sqrt(running_var + eps) + beta.  decay is an argument (0.99 by default).

Parity pins (tests/test_oracle_*.py): brute-force 7-loop convolutions on tiny shapes, torch CPU fp64
conv2d / batch_norm / autograd / optim.SGD as library cross-checks, central finite differences of the
whole block loss, the depthwise-separable == rank-structured full conv identity, zero loss and zero
gradient when the student reproduces the teacher, BN zero-mean / unit-variance, closed forms for
momentum.  The multi-step trajectory itself is "parity unpinned" beyond these per-step pins: the paper
prints no loss value, weight or activation for any block.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence

import numpy as np

CONV3X3 = 0
DWSEP3X3 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpbkd_ref.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile pbkd_ref.c with gcc into oracle/libpbkd_ref.so."""
    src = os.path.join(_HERE, "pbkd_ref.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB_PATH, src, "-lm"]
        subprocess.check_call(cmd)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB_PATH)
    return _lib


def num_threads() -> int:
    return int(_load().ref_num_threads())


def _p(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _c(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def out_dim(n: int, s: int) -> int:
    return (n - 1) // s + 1


# ---------------------------------------------------------------- layer primitives (C loops, fp64)

def conv3x3_fwd(a, W, s=1):
    a, W = _c(a), _c(W)
    N, Ci, H, Wd = a.shape
    Co = W.shape[0]
    assert W.shape == (Co, Ci, 3, 3)
    z = np.empty((N, Co, out_dim(H, s), out_dim(Wd, s)))
    _load().ref_conv3x3_fwd(_p(a), _p(W), _p(z), N, Ci, Co, H, Wd, s)
    return z


def conv3x3_wgrad(dz, a, s=1):
    dz, a = _c(dz), _c(a)
    N, Ci, H, Wd = a.shape
    Co = dz.shape[1]
    dW = np.empty((Co, Ci, 3, 3))
    _load().ref_conv3x3_wgrad(_p(dz), _p(a), _p(dW), N, Ci, Co, H, Wd, s)
    return dW


def conv3x3_dgrad(dz, W, in_hw, s=1):
    dz, W = _c(dz), _c(W)
    N, Co = dz.shape[:2]
    Ci = W.shape[1]
    H, Wd = in_hw
    da = np.empty((N, Ci, H, Wd))
    _load().ref_conv3x3_dgrad(_p(dz), _p(W), _p(da), N, Ci, Co, H, Wd, s)
    return da


def dw3x3_fwd(a, D, s=1):
    a, D = _c(a), _c(D)
    N, C, H, Wd = a.shape
    assert D.shape == (C, 1, 3, 3)
    u = np.empty((N, C, out_dim(H, s), out_dim(Wd, s)))
    _load().ref_dw3x3_fwd(_p(a), _p(D), _p(u), N, C, H, Wd, s)
    return u


def dw3x3_wgrad(du, a, s=1):
    du, a = _c(du), _c(a)
    N, C, H, Wd = a.shape
    dD = np.empty((C, 1, 3, 3))
    _load().ref_dw3x3_wgrad(_p(du), _p(a), _p(dD), N, C, H, Wd, s)
    return dD


def dw3x3_dgrad(du, D, in_hw, s=1):
    du, D = _c(du), _c(D)
    N, C = du.shape[:2]
    H, Wd = in_hw
    da = np.empty((N, C, H, Wd))
    _load().ref_dw3x3_dgrad(_p(du), _p(D), _p(da), N, C, H, Wd, s)
    return da


def conv1x1_fwd(a, P, s=1):
    a, P = _c(a), _c(P)
    N, Ci, H, Wd = a.shape
    Co = P.shape[0]
    assert P.shape == (Co, Ci)
    z = np.empty((N, Co, out_dim(H, s), out_dim(Wd, s)))
    _load().ref_conv1x1_fwd(_p(a), _p(P), _p(z), N, Ci, Co, H, Wd, s)
    return z


def conv1x1_wgrad(dz, a, s=1):
    dz, a = _c(dz), _c(a)
    N, Ci, H, Wd = a.shape
    Co = dz.shape[1]
    dP = np.empty((Co, Ci))
    _load().ref_conv1x1_wgrad(_p(dz), _p(a), _p(dP), N, Ci, Co, H, Wd, s)
    return dP


def conv1x1_dgrad(dz, P, in_hw, s=1):
    dz, P = _c(dz), _c(P)
    N, Co = dz.shape[:2]
    Ci = P.shape[1]
    H, Wd = in_hw
    da = np.empty((N, Ci, H, Wd))
    _load().ref_conv1x1_dgrad(_p(dz), _p(P), _p(da), N, Ci, Co, H, Wd, s)
    return da


def bn_fwd(z, gamma, beta, eps):
    z, gamma, beta = _c(z), _c(gamma), _c(beta)
    N, C, H, Wd = z.shape
    xhat = np.empty_like(z)
    b = np.empty_like(z)
    mean = np.empty((C,))
    rstd = np.empty((C,))
    _load().ref_bn_fwd(_p(z), _p(gamma), _p(beta), ctypes.c_double(eps), _p(xhat), _p(b), _p(mean), _p(rstd),
                       N, C, H * Wd)
    return xhat, b, mean, rstd


def bn_bwd(g, xhat, gamma, rstd):
    g, xhat, gamma, rstd = _c(g), _c(xhat), _c(gamma), _c(rstd)
    N, C, H, Wd = g.shape
    dz = np.empty_like(g)
    dgamma = np.empty((C,))
    dbeta = np.empty((C,))
    _load().ref_bn_bwd(_p(g), _p(xhat), _p(gamma), _p(rstd), _p(dz), _p(dgamma), _p(dbeta), N, C, H * Wd)
    return dz, dgamma, dbeta


def bn_inference(z, gamma, beta, rmean, rvar, eps):
    """BatchNorm with fixed statistics (R15): per channel an affine map of z."""
    z = _c(z)
    sh = (1, -1, 1, 1)
    return _c(gamma).reshape(sh) * (z - _c(rmean).reshape(sh)) / np.sqrt(_c(rvar).reshape(sh) + eps) + _c(beta).reshape(sh)


def batch_moments(z):
    """Per-channel batch mean and biased batch variance over (N, H, W), the two numbers R15 averages."""
    z = _c(z)
    return z.mean(axis=(0, 2, 3)), z.var(axis=(0, 2, 3))


# ---------------------------------------------------------------- elementwise pieces (numpy)

def maxpool2x2_fwd(y):
    """p[n,c,i,j] = max of the 2x2 window; also the index (0..3, row-major) of its first maximum."""
    N, C, H, W = y.shape
    Hp, Wp = H // 2, W // 2
    win = y[:, :, :2 * Hp, :2 * Wp].reshape(N, C, Hp, 2, Wp, 2).transpose(0, 1, 2, 4, 3, 5).reshape(N, C, Hp, Wp, 4)
    arg = np.argmax(win, axis=-1)          # numpy returns the first maximum
    p = np.take_along_axis(win, arg[..., None], axis=-1)[..., 0]
    return p, arg


class DecisionOutsideMargin(ValueError):
    """A ReLU / max-pool decision handed to the oracle differs from the oracle's own although the
    element is not within the stated margin of the kink."""


def check_relu_decisions(b, given, margin_rel):
    own = b > 0.0
    given = np.asarray(given, dtype=bool)
    if given.shape != own.shape:
        raise ValueError("relu decision mask has the wrong shape")
    diff = given != own
    n = int(diff.sum())
    worst_rel = 0.0
    if n:
        bmax = np.abs(b).max()
        margin = margin_rel * bmax
        worst = float(np.abs(b[diff]).max())
        if worst > margin:
            raise DecisionOutsideMargin(f"{n} ReLU decisions differ; |b| up to {worst:.3e} exceeds the margin {margin:.3e}")
        worst_rel = worst / bmax
    return n, worst_rel


def check_pool_decisions(y, own_arg, given_arg, margin_rel):
    N, C, H, W = y.shape
    Hp, Wp = H // 2, W // 2
    given_arg = np.asarray(given_arg)
    if given_arg.shape != own_arg.shape:
        raise ValueError("pool argmax has the wrong shape")
    diff = given_arg != own_arg
    n = int(diff.sum())
    worst_rel = 0.0
    if n:
        win = y[:, :, :2 * Hp, :2 * Wp].reshape(N, C, Hp, 2, Wp, 2).transpose(0, 1, 2, 4, 3, 5).reshape(N, C, Hp, Wp, 4)
        y_own = np.take_along_axis(win, own_arg[..., None], axis=-1)[..., 0]
        y_giv = np.take_along_axis(win, given_arg[..., None].astype(np.int64), axis=-1)[..., 0]
        ymax = np.abs(y).max()
        margin = margin_rel * ymax
        worst = float((y_own - y_giv)[diff].max())
        if worst > margin:
            raise DecisionOutsideMargin(f"{n} pool decisions differ; gap up to {worst:.3e} exceeds the margin {margin:.3e}")
        worst_rel = worst / ymax if ymax > 0 else 0.0
    return n, worst_rel


def maxpool2x2_bwd(dp, arg, in_hw):
    N, C, Hp, Wp = dp.shape
    H, W = in_hw
    win = np.zeros((N, C, Hp, Wp, 4))
    np.put_along_axis(win, arg[..., None], dp[..., None], axis=-1)
    dy = np.zeros((N, C, H, W))
    dy[:, :, :2 * Hp, :2 * Wp] = win.reshape(N, C, Hp, Wp, 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(N, C, 2 * Hp, 2 * Wp)
    return dy


def local_loss(p, t, loss_reduction=0):
    """Eq. 3 on one batch.  reduction 0: mean over every element; 1: summed squared norm / batch size."""
    cnt = p.size if loss_reduction == 0 else p.shape[0]
    d = p - t
    return float(np.sum(d * d) / cnt), cnt


# ---------------------------------------------------------------- block forward / backward

def block_forward(arch, params: Sequence[Sequence[np.ndarray]], x, keep: bool = False, running=None):
    """Forward of one block (teacher or student).  Returns the block output and, if keep, the cache.
    running: None = BatchNorm with batch statistics (R4); else one (running_mean, running_var) pair per layer,
    then the projection shortcut's if there is one: inference mode (R15; not together with keep)."""
    x = _c(x)
    assert not (keep and running is not None)
    layers = list(arch.layers)
    nl = len(layers)
    a = x
    cache = []
    for l, L in enumerate(layers):
        pr = [_c(q) for q in params[l]]
        rec = {"a": a}
        if L.kind == CONV3X3:
            W, gamma, beta = pr
            z = conv3x3_fwd(a, W, L.stride)
        else:
            D, P, gamma, beta = pr
            u = dw3x3_fwd(a, D, L.stride)
            z = conv1x1_fwd(u, P, 1)
            rec["u"] = u
        if running is None:
            xhat, b, mean, rstd = bn_fwd(z, gamma, beta, arch.bn_eps)
            rec.update(z=z, xhat=xhat, mean=mean, rstd=rstd)
        else:
            b = bn_inference(z, gamma, beta, running[l][0], running[l][1], arch.bn_eps)
        if l == nl - 1 and arch.shortcut == 1:
            Ws, gs, bs = [_c(q) for q in params[nl]]
            zs = conv1x1_fwd(x, Ws, arch.shortcut_stride)
            if running is None:
                xhs, bsc, ms, rs = bn_fwd(zs, gs, bs, arch.bn_eps)
                rec.update(zs=zs, xhat_s=xhs, mean_s=ms, rstd_s=rs)
            else:
                bsc = bn_inference(zs, gs, bs, running[nl][0], running[nl][1], arch.bn_eps)
            b = b + bsc
        elif l == nl - 1 and arch.shortcut == 2:
            b = b + x                      # identity skip (R14): the block input, added before the last ReLU
        rec["b"] = b
        a = np.maximum(b, 0.0)
        cache.append(rec)
    out = a
    pool_arg = None
    if arch.pool == 2:
        out, pool_arg = maxpool2x2_fwd(a)
    if keep:
        return out, {"layers": cache, "pool_arg": pool_arg, "y_hw": a.shape[2:], "x": x}
    return out


def block_backward(arch, params, cache, dout, decisions=None, margin_rel=1e-4):
    """Gradients of every parameter of the block given dL/d(block output).  Same nesting as params.
    decisions (optional, reading R13): {"relu": [bool mask per layer, shape of that layer's output],
    "pool_arg": int array [N,C,Hp,Wp] or None}; verified against the margin, then used."""
    layers = list(arch.layers)
    nl = len(layers)
    relu_on = [rec["b"] > 0.0 for rec in cache["layers"]]
    pool_arg = cache["pool_arg"]
    # what a caller needs to judge the given decisions: how many there were, how many differ from the oracle's own,
    # and how far from the kink the farthest differing one lies (as a fraction of max|b|, or of max y for the pool)
    cache["decisions_total"] = 0
    cache["decisions_differing"] = 0
    cache["decisions_worst_rel"] = 0.0
    if decisions is not None:
        for l in range(nl):
            n, worst = check_relu_decisions(cache["layers"][l]["b"], decisions["relu"][l], margin_rel)
            cache["decisions_total"] += int(cache["layers"][l]["b"].size)
            cache["decisions_differing"] += n
            cache["decisions_worst_rel"] = max(cache["decisions_worst_rel"], worst)
            relu_on[l] = np.asarray(decisions["relu"][l], dtype=bool)
        if arch.pool == 2 and decisions.get("pool_arg") is not None:
            y_last = np.maximum(cache["layers"][-1]["b"], 0.0)
            n, worst = check_pool_decisions(y_last, pool_arg, decisions["pool_arg"], margin_rel)
            cache["decisions_total"] += int(pool_arg.size)
            cache["decisions_differing"] += n
            cache["decisions_worst_rel"] = max(cache["decisions_worst_rel"], worst)
            pool_arg = np.asarray(decisions["pool_arg"]).astype(np.int64)
    if arch.pool == 2:
        dy = maxpool2x2_bwd(dout, pool_arg, cache["y_hw"])
    else:
        dy = dout
    grads = [None] * len(params)
    for l in range(nl - 1, -1, -1):
        L = layers[l]
        rec = cache["layers"][l]
        pr = [_c(q) for q in params[l]]
        g = dy * relu_on[l]
        if l == nl - 1 and arch.shortcut == 1:
            Ws, gs, bs = [_c(q) for q in params[nl]]
            dzs, dgs, dbs = bn_bwd(g, rec["xhat_s"], gs, rec["rstd_s"])
            dWs = conv1x1_wgrad(dzs, cache["x"], arch.shortcut_stride)
            grads[nl] = [dWs, dgs, dbs]
        gamma = pr[-2]
        dz, dgamma, dbeta = bn_bwd(g, rec["xhat"], gamma, rec["rstd"])
        a = rec["a"]
        if L.kind == CONV3X3:
            W = pr[0]
            dW = conv3x3_wgrad(dz, a, L.stride)
            grads[l] = [dW, dgamma, dbeta]
            if l > 0:
                dy = conv3x3_dgrad(dz, W, a.shape[2:], L.stride)
        else:
            D, P = pr[0], pr[1]
            dP = conv1x1_wgrad(dz, rec["u"], 1)
            du = conv1x1_dgrad(dz, P, rec["u"].shape[2:], 1)
            dD = dw3x3_wgrad(du, a, L.stride)
            grads[l] = [dD, dP, dgamma, dbeta]
            if l > 0:
                dy = dw3x3_dgrad(du, D, a.shape[2:], L.stride)
    return grads


class RefBlock:
    """One distillation task: frozen teacher block + trainable student block + SGD-momentum state."""

    def __init__(self, teacher, teacher_params, student, student_params, momentum=0.9, loss_reduction=0,
                 shortcut_trainable=0, bn_decay=0.99):
        self.teacher = teacher
        self.student = student
        self.tp = [[_c(q).copy() for q in lp] for lp in teacher_params]
        self.sp = [[_c(q).copy() for q in lp] for lp in student_params]
        self.vel = [[np.zeros_like(q) for q in lp] for lp in self.sp]
        self.momentum = float(momentum)
        self.loss_reduction = loss_reduction
        self.shortcut_trainable = shortcut_trainable
        self.bn_decay = float(bn_decay)
        # running (mean, variance) per BatchNorm, R15: start at (0, 1); the teacher's are set by the caller
        self.t_running = [[np.zeros(lp[-1].shape), np.ones(lp[-1].shape)] for lp in self.tp]
        self.s_running = [[np.zeros(lp[-1].shape), np.ones(lp[-1].shape)] for lp in self.sp]
        self.grads = None
        self.cache = None

    def teacher_forward(self, x, bn_mode=0):
        return block_forward(self.teacher, self.tp, x, running=self.t_running if bn_mode else None)

    def student_forward(self, x, bn_mode=0):
        return block_forward(self.student, self.sp, x, running=self.s_running if bn_mode else None)

    def _update_running(self, cache):
        """R15: every student BatchNorm's running pair moves toward this forward pass's batch moments."""
        nl = len(self.student.layers)
        zs = [rec["z"] for rec in cache["layers"]]
        if self.student.shortcut == 1:
            zs.append(cache["layers"][-1]["zs"])
        assert len(zs) == len(self.s_running) and len(zs) in (nl, nl + 1)
        d = self.bn_decay
        for pair, z in zip(self.s_running, zs):
            m, v = batch_moments(z)
            pair[0] = d * pair[0] + (1.0 - d) * m
            pair[1] = d * pair[1] + (1.0 - d) * v

    def loss_and_grads(self, x, t, decisions=None):
        p, cache = block_forward(self.student, self.sp, x, keep=True)
        loss, cnt = local_loss(p, _c(t), self.loss_reduction)
        dp = 2.0 * (p - _c(t)) / cnt
        grads = block_backward(self.student, self.sp, cache, dp, decisions)
        self.cache = cache
        self.grads = grads
        return loss, grads

    def _trainable(self, l):
        nl = len(self.student.layers)
        if l == nl:
            return bool(self.shortcut_trainable)
        return bool(self.student.layers[l].trainable)

    def student_step(self, x, t, lr, decisions=None):
        """One SGD-momentum step; returns the loss of this step's forward pass (before the update)."""
        loss, grads = self.loss_and_grads(x, t, decisions)
        self._update_running(self.cache)
        for l, lp in enumerate(self.sp):
            if not self._trainable(l):
                continue
            for k in range(len(lp)):
                self.vel[l][k] = self.momentum * self.vel[l][k] + grads[l][k]
                lp[k] -= lr * self.vel[l][k]
        return loss


# ------------------------------------------------------------------------------------------------
# Reassembly (Algorithm 1, the loop after the gather: a teacher block is replaced by its student block where the
# student passed the evaluation).  Readings: BatchNorm uses batch statistics (bn_mode 0, R4) or the running ones
# (bn_mode 1, R15), and the evaluation metric is label free -- the mean squared difference between the reassembled
# network's final features and the teacher's -- because the paper's accuracy needs its datasets and classifier.
def network_forward(blocks: Sequence["RefBlock"], use_student: Sequence[int], x, bn_mode=0):
    """Runs the chain of blocks on x: block k by its student g_k where use_student[k] is non-zero, by the
    teacher f_k otherwise (Eq. 1 and Eq. 2 are the two extremes).  Returns every block's output."""
    outs = []
    a = _c(x)
    for blk, u in zip(blocks, use_student):
        a = blk.student_forward(a, bn_mode) if u else blk.teacher_forward(a, bn_mode)
        outs.append(a)
    return outs


def feature_mse(a, b) -> float:
    a, b = _c(a), _c(b)
    return float(np.mean((a - b) ** 2))


def select_blocks(blocks: Sequence["RefBlock"], x, threshold: float, bn_mode=0):
    """Evaluates every student block on its own (the network with only that block replaced) and keeps those whose
    feature error stays below the threshold (the paper keeps those whose accuracy stays above one).
    Returns (use_student, per-block error, error of the reassembled network)."""
    n = len(blocks)
    ref = network_forward(blocks, [0] * n, x, bn_mode)[-1]
    errs = []
    for k in range(n):
        mask = [1 if j == k else 0 for j in range(n)]
        errs.append(feature_mse(network_forward(blocks, mask, x, bn_mode)[-1], ref))
    use = [1 if e < threshold else 0 for e in errs]
    final = feature_mse(network_forward(blocks, use, x, bn_mode)[-1], ref)
    return use, errs, final
