"""Pins for the oracle's block composition, loss, backward and SGD-momentum (CPU only).

Finite differences of the whole block loss, a torch CPU fp64 autograd re-statement built from library
ops, structural invariants (zero loss / zero gradient when the student is the teacher in factored form;
scale invariances that BatchNorm induces), and closed forms for momentum SGD.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import block as ob
from paper_2012_03096_amd import workloads as wl


def _loss_only(arch, sp, x, t, red=0):
    p = ob.block_forward(arch, sp, x)
    return ob.local_loss(p, t, red)[0]


def _variants():
    vs = {w.name: w for w in wl.small_variants() + wl.degenerate_variants()}
    vs["cfg1"] = wl.cfg1_tiny()
    return vs


VARIANTS = _variants()


def _setup(name, random_affine=True, shrink=True):
    w = VARIANTS[name]
    x, tp, sp = w.tensors(random_affine=random_affine)
    x = x.astype(np.float64)
    tp = [[q.astype(np.float64) for q in lp] for lp in tp]
    sp = [[q.astype(np.float64) for q in lp] for lp in sp]
    blk = ob.RefBlock(w.teacher, tp, w.student, sp, momentum=w.momentum, shortcut_trainable=1)
    t = blk.teacher_forward(x)
    return w, x, t, blk


@pytest.mark.parametrize("name", ["ragged_pool", "ragged_residual_s2", "fullconv_first", "three_layers_oddc", "paper_task_2x2",
                                  "two_layers_skip", "three_layers_skip_pool",
                                  "single_row_residual_s2", "pool_3x3_to_1x1", "column_s2_to_one_pixel"])
@pytest.mark.parametrize("red", [0, 1])
def test_block_gradients_finite_differences(name, red):
    """Directional central differences for every parameter tensor (shortcut included).  (The degenerate variants with
    two or fifteen values per BatchNorm channel are left to the autograd cross-check below: there BatchNorm is so
    curved, and a kink so likely within the probe, that a central difference is no measure of the gradient.)"""
    w, x, t, blk = _setup(name)
    blk.loss_reduction = red
    loss, grads = blk.loss_and_grads(x, t)
    rng = np.random.default_rng(7)
    worst = 0.0
    for l, lp in enumerate(blk.sp):
        for k, q in enumerate(lp):
            for trial in range(2):
                d = rng.standard_normal(q.shape)
                d /= np.linalg.norm(d)
                h = 1e-6
                keep = q.copy()
                q[...] = keep + h * d
                lp_ = _loss_only(w.student, blk.sp, x, t, red)
                q[...] = keep - h * d
                lm_ = _loss_only(w.student, blk.sp, x, t, red)
                q[...] = keep
                fd = (lp_ - lm_) / (2 * h)
                an = float(np.sum(grads[l][k] * d))
                scale = max(abs(an), np.linalg.norm(grads[l][k]) * 1e-3, 1e-12)
                worst = max(worst, abs(fd - an) / scale)
    # ReLU / max-pool kinks crossed by the +-h probe cost a little; a wrong term costs O(1)
    assert worst < 2e-4, worst


def test_block_gradients_per_parameter_tiny():
    """Every single parameter of a tiny block, one by one."""
    t_arch = wl.Arch(2, 2, 4, 4, [wl.Layer(wl.CONV3X3, 2, 3, 2, 0), wl.Layer(wl.CONV3X3, 3, 3, 1, 0)], shortcut=1, shortcut_stride=2)
    s_arch = wl.Arch(2, 2, 4, 4, [wl.Layer(wl.DWSEP3X3, 2, 3, 2, 1), wl.Layer(wl.DWSEP3X3, 3, 3, 1, 1)], shortcut=1, shortcut_stride=2)
    rng = np.random.default_rng(3)
    x = np.maximum(rng.standard_normal((2, 2, 4, 4)), 0)
    tp = [[q.astype(np.float64) for q in lp] for lp in wl.make_params(t_arch, 5, True)]
    sp = [[q.astype(np.float64) for q in lp] for lp in wl.make_params(s_arch, 6, True)]
    blk = ob.RefBlock(t_arch, tp, s_arch, sp, shortcut_trainable=1)
    t = blk.teacher_forward(x)
    loss, grads = blk.loss_and_grads(x, t)
    bad = 0
    total = 0
    for l, lp in enumerate(blk.sp):
        for k, q in enumerate(lp):
            flat = q.reshape(-1)
            gflat = grads[l][k].reshape(-1)
            for i in range(flat.size):
                keep = flat[i]
                h = 1e-6 * max(1.0, abs(keep))
                flat[i] = keep + h
                lp_ = _loss_only(s_arch, blk.sp, x, t)
                flat[i] = keep - h
                lm_ = _loss_only(s_arch, blk.sp, x, t)
                flat[i] = keep
                fd = (lp_ - lm_) / (2 * h)
                total += 1
                if abs(fd - gflat[i]) > 1e-6 * max(1.0, abs(gflat[i])) + 1e-5 * abs(gflat[i]):
                    bad += 1
    assert bad == 0, (bad, total)


def _torch_block(arch, params, x):
    a = x
    nl = len(arch.layers)
    for l, L in enumerate(arch.layers):
        pr = params[l]
        if L.kind == wl.CONV3X3:
            z = F.conv2d(a, pr[0], stride=L.stride, padding=1)
        else:
            u = F.conv2d(a, pr[0], stride=L.stride, padding=1, groups=L.cin)
            z = F.conv2d(u, pr[1][:, :, None, None])
        b = F.batch_norm(z, None, None, pr[-2], pr[-1], True, 0.1, arch.bn_eps)
        if l == nl - 1 and arch.shortcut == 1:
            ps = params[nl]
            zs = F.conv2d(x, ps[0][:, :, None, None], stride=arch.shortcut_stride)
            b = b + F.batch_norm(zs, None, None, ps[1], ps[2], True, 0.1, arch.bn_eps)
        elif l == nl - 1 and arch.shortcut == 2:
            b = b + x
        a = F.relu(b)
    if arch.pool == 2:
        a = F.max_pool2d(a, 2)
    return a


@pytest.mark.parametrize("name", list(VARIANTS))
def test_block_matches_torch_autograd(name):
    w, x, t, blk = _setup(name)
    loss, grads = blk.loss_and_grads(x, t)
    tx = torch.from_numpy(x)
    tparams = [[torch.from_numpy(q.copy()) for q in lp] for lp in blk.tp]
    sparams = [[torch.from_numpy(q.copy()).requires_grad_() for q in lp] for lp in blk.sp]
    with torch.no_grad():
        tt = _torch_block(w.teacher, tparams, tx)
    np.testing.assert_allclose(t, tt.numpy(), atol=1e-10)
    tl = F.mse_loss(_torch_block(w.student, sparams, tx), tt)
    tl.backward()
    assert np.isclose(loss, tl.item(), rtol=1e-11)
    for l, lp in enumerate(sparams):
        for k, q in enumerate(lp):
            ref = q.grad.numpy()
            np.testing.assert_allclose(grads[l][k], ref, atol=1e-9 * max(1.0, np.abs(ref).max()))


def test_zero_loss_and_gradient_when_student_reproduces_teacher():
    """Teacher convs built as W = P (x) D; the student holds the factors -> loss 0 and all gradients 0."""
    rng = np.random.default_rng(0)
    chans = [6, 8, 5]
    t_arch = wl.Arch(3, 6, 8, 8, [wl.Layer(wl.CONV3X3, ci, co, 2 if i == 0 else 1, 0) for i, (ci, co) in enumerate(zip(chans[:-1], chans[1:]))],
                     shortcut=1, shortcut_stride=2, pool=2)
    s_arch = wl.Arch(3, 6, 8, 8, [wl.Layer(wl.DWSEP3X3, ci, co, 2 if i == 0 else 1, 1) for i, (ci, co) in enumerate(zip(chans[:-1], chans[1:]))],
                     shortcut=1, shortcut_stride=2, pool=2)
    sp = [[q.astype(np.float64) for q in lp] for lp in wl.make_params(s_arch, 1, True)]
    tp = []
    for l in range(2):
        D, P, g, b = sp[l]
        tp.append([P[:, :, None, None] * D[None, :, 0], g.copy(), b.copy()])
    tp.append([q.copy() for q in sp[2]])
    x = np.maximum(rng.standard_normal((3, 6, 8, 8)), 0)
    blk = ob.RefBlock(t_arch, tp, s_arch, sp, shortcut_trainable=1)
    t = blk.teacher_forward(x)
    loss, grads = blk.loss_and_grads(x, t)
    assert loss < 1e-25
    for lg in grads:
        for g in lg:
            assert np.abs(g).max() < 1e-12
    # a step leaves the weights where they are
    before = [[q.copy() for q in lp] for lp in blk.sp]
    blk.student_step(x, t, 0.1)
    for lp, lb in zip(blk.sp, before):
        for q, qb in zip(lp, lb):
            np.testing.assert_allclose(q, qb, atol=1e-12)


def test_batchnorm_scale_invariance_identities():
    """BN after the pointwise conv makes z's scale irrelevant, so (up to the eps term)
    <P[o,:], dP[o,:]> = 0 for every o; and rescaling D[c] by s and P[:,c] by 1/s leaves z unchanged,
    which gives exactly <D[c], dD[c]> = <P[:,c], dP[:,c]> for every c."""
    w, x, t, blk = _setup("three_layers_oddc")
    loss, grads = blk.loss_and_grads(x, t)
    for l, L in enumerate(w.student.layers):
        D, P = blk.sp[l][0], blk.sp[l][1]
        dD, dP = grads[l][0], grads[l][1]
        lhs = np.sum(D * dD, axis=(1, 2, 3))
        rhs = np.sum(P * dP, axis=0)
        np.testing.assert_allclose(lhs, rhs, rtol=1e-9, atol=1e-13)
        row = np.sum(P * dP, axis=1)
        assert np.abs(row).max() < 1e-3 * np.abs(P * dP).sum(axis=1).max()


def test_sgd_momentum_closed_forms():
    """With a constant gradient g: v_k = g (1-mu^k)/(1-mu) and theta_k = theta_0 - lr * sum_j v_j.
    Checked by driving the RefBlock update loop with a pinned gradient."""
    w = wl.cfg1_tiny()
    x, tp, sp = w.tensors()
    blk = ob.RefBlock(w.teacher, tp, w.student, sp, momentum=0.9)
    g_const = [[np.full_like(q, 0.5) for q in lp] for lp in blk.sp]
    blk.loss_and_grads = lambda x_, t_, d_=None: (0.0, g_const)     # pin the gradient
    blk._update_running = lambda cache_: None                        # no forward pass, no batch moments
    theta0 = [[q.copy() for q in lp] for lp in blk.sp]
    lr, mu = 0.01, 0.9
    cum = 0.0
    for k in range(1, 6):
        blk.student_step(None, None, lr)
        vk = 0.5 * (1 - mu ** k) / (1 - mu)
        cum += vk
        np.testing.assert_allclose(blk.vel[0][0], vk, rtol=1e-13)
        np.testing.assert_allclose(blk.sp[0][0], theta0[0][0] - lr * cum, rtol=1e-13, atol=1e-15)
        if k == 1:       # the first step is plain SGD
            np.testing.assert_allclose(blk.sp[1][1], theta0[1][1] - lr * 0.5, rtol=1e-14)


def test_sgd_two_step_hand_example_and_torch_optim():
    """theta_2 = theta_0 - lr (g_0 (1+mu) + g_1); and three real steps equal torch.optim.SGD's."""
    w, x, t, blk = _setup("ragged_pool")
    blk.shortcut_trainable = 0
    lr, mu = 0.05, blk.momentum
    theta0 = [[q.copy() for q in lp] for lp in blk.sp]
    _, g0 = blk.loss_and_grads(x, t)
    g0 = [[g.copy() for g in lg] for lg in g0]
    blk.student_step(x, t, lr)
    _, g1 = blk.loss_and_grads(x, t)
    g1 = [[g.copy() for g in lg] for lg in g1]
    blk.student_step(x, t, lr)
    for l in range(len(theta0)):
        for k in range(len(theta0[l])):
            np.testing.assert_allclose(blk.sp[l][k], theta0[l][k] - lr * (g0[l][k] * (1 + mu) + g1[l][k]), rtol=1e-12, atol=1e-14)
    blk.student_step(x, t, lr)
    # library cross-check
    sparams = [[torch.from_numpy(q.copy()).requires_grad_() for q in lp] for lp in theta0]
    opt = torch.optim.SGD([q for lp in sparams for q in lp], lr=lr, momentum=mu)
    tt = torch.from_numpy(t)
    for _ in range(3):
        opt.zero_grad()
        F.mse_loss(_torch_block(w.student, sparams, torch.from_numpy(x)), tt).backward()
        opt.step()
    for lp, lt in zip(blk.sp, sparams):
        for q, qt in zip(lp, lt):
            np.testing.assert_allclose(q, qt.detach().numpy(), atol=1e-10)


def test_frozen_layers_do_not_move_and_loss_decreases():
    w = wl.cfg1_tiny()
    x, tp, sp = w.tensors()
    blk = ob.RefBlock(w.teacher, tp, w.student, sp, momentum=w.momentum)
    t = blk.teacher_forward(x)
    losses = [blk.student_step(x, t, w.lr) for _ in range(10)]
    assert all(b < a for a, b in zip(losses[:-1], losses[1:])), losses
    w3, x3, t3, blk3 = _setup("ragged_residual_s2")
    blk3.shortcut_trainable = 0
    before = [q.copy() for q in blk3.sp[-1]]
    blk3.student_step(x3, t3, 0.01)
    for q, qb in zip(blk3.sp[-1], before):
        np.testing.assert_array_equal(q, qb)


def test_eq3_reduction_is_a_constant_rescale():
    w, x, t, blk = _setup("ragged_pool")
    l0, g0 = blk.loss_and_grads(x, t)
    g0 = [[g.copy() for g in lg] for lg in g0]
    blk.loss_reduction = 1
    l1, g1 = blk.loss_and_grads(x, t)
    chw = np.prod(t.shape[1:])
    assert np.isclose(l1, l0 * chw, rtol=1e-13)
    np.testing.assert_allclose(g1[0][1], g0[0][1] * chw, rtol=1e-12)


def _torch_block_with_decisions(arch, params, x, relu_on, pool_arg):
    """The block with every ReLU replaced by a fixed 0/1 mask and the pool by a fixed gather: what
    'differentiate with the given sub-gradient choices' means, restated with torch autograd."""
    a = x
    nl = len(arch.layers)
    for l, L in enumerate(arch.layers):
        pr = params[l]
        if L.kind == wl.CONV3X3:
            z = F.conv2d(a, pr[0], stride=L.stride, padding=1)
        else:
            u = F.conv2d(a, pr[0], stride=L.stride, padding=1, groups=L.cin)
            z = F.conv2d(u, pr[1][:, :, None, None])
        b = F.batch_norm(z, None, None, pr[-2], pr[-1], True, 0.1, arch.bn_eps)
        if l == nl - 1 and arch.shortcut == 1:
            ps = params[nl]
            zs = F.conv2d(x, ps[0][:, :, None, None], stride=arch.shortcut_stride)
            b = b + F.batch_norm(zs, None, None, ps[1], ps[2], True, 0.1, arch.bn_eps)
        elif l == nl - 1 and arch.shortcut == 2:
            b = b + x
        # forward value: the true ReLU; derivative: the given mask
        a = F.relu(b).detach() + (b - b.detach()) * torch.from_numpy(relu_on[l].astype(np.float64))
    if arch.pool == 2:
        N, C, H, W = a.shape
        Hp, Wp = H // 2, W // 2
        win = a[:, :, :2 * Hp, :2 * Wp].reshape(N, C, Hp, 2, Wp, 2).permute(0, 1, 2, 4, 3, 5).reshape(N, C, Hp, Wp, 4)
        picked = torch.gather(win, -1, torch.from_numpy(pool_arg.astype(np.int64))[..., None])[..., 0]
        a = F.max_pool2d(a, 2).detach() + (picked - picked.detach())
    return a


@pytest.mark.parametrize("name", ["ragged_pool", "ragged_residual_s2"])
def test_backward_with_given_decisions(name):
    """Own decisions reproduce the plain backward; flipped near-kink decisions are accepted, change the
    gradient exactly as the masked network's autograd says; decisions away from the kink are refused."""
    w, x, t, blk = _setup(name)
    loss0, g0 = blk.loss_and_grads(x, t)
    g0 = [[g.copy() for g in lg] for lg in g0]
    cache = blk.cache
    own = {"relu": [rec["b"] > 0 for rec in cache["layers"]], "pool_arg": cache["pool_arg"]}
    loss1, g1 = blk.loss_and_grads(x, t, own)
    assert blk.cache["decisions_differing"] == 0 and loss1 == loss0
    for la, lb in zip(g0, g1):
        for a, b in zip(la, lb):
            np.testing.assert_array_equal(a, b)
    # move the block so that a few pre-activations sit within the margin: shift beta of each layer by
    # minus the value of its 3 smallest positive b's midpoint ... simpler: flip the k elements of smallest |b|
    # and widen the margin accordingly through margin_rel
    flipped = {"relu": [m.copy() for m in own["relu"]], "pool_arg": None}
    need = 0.0
    for l, rec in enumerate(cache["layers"]):
        b = rec["b"]
        idx = np.argsort(np.abs(b).ravel())[:3]
        flipped["relu"][l].reshape(-1)[idx] ^= True
        need = max(need, np.abs(b.ravel()[idx]).max() / np.abs(b).max())
    p, c2 = ob.block_forward(w.student, blk.sp, x, keep=True)
    _, cnt = ob.local_loss(p, t, 0)
    dp = 2.0 * (p - t) / cnt
    with pytest.raises(ob.DecisionOutsideMargin):
        ob.block_backward(w.student, blk.sp, c2, dp, flipped, margin_rel=need * 0.5)
    g2 = ob.block_backward(w.student, blk.sp, c2, dp, flipped, margin_rel=need * 1.01)
    assert c2["decisions_differing"] == 3 * len(cache["layers"])
    # the figures a caller judges the given decisions by: every mask element (and pool window) was counted, and
    # the farthest differing element's distance from the kink is the one planted above
    want_total = sum(rec["b"].size for rec in cache["layers"])
    assert c2["decisions_total"] == want_total            # flipped["pool_arg"] differs in nothing: still counted if given
    assert abs(c2["decisions_worst_rel"] - need) <= 1e-12 * need
    # library cross-check: autograd through the masked network, upstream gradient = the oracle's dp
    sparams = [[torch.from_numpy(q.copy()).requires_grad_() for q in lp] for lp in blk.sp]
    arg = own["pool_arg"] if own["pool_arg"] is not None else None
    out = _torch_block_with_decisions(w.student, sparams, torch.from_numpy(x), flipped["relu"], arg)
    out.backward(torch.from_numpy(dp))
    changed = False
    for l, lp in enumerate(sparams):
        for k, q in enumerate(lp):
            ref = q.grad.numpy()
            np.testing.assert_allclose(g2[l][k], ref, atol=1e-9 * max(1.0, np.abs(ref).max()))
            changed = changed or not np.allclose(g2[l][k], g0[l][k], rtol=1e-9, atol=0)
    assert changed
    # a far-away pool decision is refused too
    if own["pool_arg"] is not None:
        bad = {"relu": own["relu"], "pool_arg": (own["pool_arg"] + 1) % 4}
        with pytest.raises(ob.DecisionOutsideMargin):
            ob.block_backward(w.student, blk.sp, c2, dp, bad)


# ------------------------------------------------------------------ reassembly (Algorithm 1, last loop)
def _three_small_blocks():
    """A chain of three blocks whose shapes fit together: 5 -> 6 -> 6 -> 4 channels on a 6x6 map."""
    chans = [(5, 6), (6, 6), (6, 4)]
    blocks, rng = [], np.random.default_rng(77)
    for ci, co in chans:
        t = wl.Arch(3, ci, 6, 6, [wl.Layer(wl.CONV3X3, ci, co, 1, 0)])
        s = wl.Arch(3, ci, 6, 6, [wl.Layer(wl.DWSEP3X3, ci, co, 1, 1)])
        tp = [[rng.normal(size=(co, ci, 3, 3)) * 0.3, rng.uniform(0.5, 1.5, co), rng.normal(size=co) * 0.1]]
        sp = [[rng.normal(size=(ci, 1, 3, 3)) * 0.5, rng.normal(size=(co, ci)) * 0.4, rng.uniform(0.5, 1.5, co), rng.normal(size=co) * 0.1]]
        blocks.append(ob.RefBlock(t, tp, s, sp))
    x = np.maximum(rng.normal(size=(3, 5, 6, 6)), 0)
    return blocks, x


def test_network_forward_is_the_composition_of_the_chosen_blocks():
    blocks, x = _three_small_blocks()
    outs = ob.network_forward(blocks, [0, 1, 0], x)
    a = ob.block_forward(blocks[0].teacher, blocks[0].tp, x)
    b = ob.block_forward(blocks[1].student, blocks[1].sp, a)
    c = ob.block_forward(blocks[2].teacher, blocks[2].tp, b)
    for got, want in zip(outs, (a, b, c)):
        assert np.array_equal(got, want)
    # the two extremes are the teacher network (Eq. 1) and the student network (Eq. 2)
    assert ob.feature_mse(ob.network_forward(blocks, [0, 0, 0], x)[-1], c) > 0
    assert ob.feature_mse(ob.network_forward(blocks, [0, 0, 0], x)[-1], ob.network_forward(blocks, [0, 0, 0], x)[-1]) == 0.0


def test_select_blocks_keeps_exact_students_and_drops_bad_ones():
    """A student holding the teacher's factors reproduces its block exactly (error 0, kept at any positive
    threshold); a random student does not (error far above a small threshold, dropped); the reassembled
    network then differs from the teacher only through kept blocks, so its error is 0 as well."""
    blocks, x = _three_small_blocks()
    rng = np.random.default_rng(5)
    # make block 1's teacher rank-structured and give its student those factors
    ci, co = 6, 6
    D = rng.normal(size=(ci, 1, 3, 3)) * 0.5
    P = rng.normal(size=(co, ci)) * 0.4
    W = P[:, :, None, None] * D[None, :, 0]
    g, b = blocks[1].tp[0][1], blocks[1].tp[0][2]
    blocks[1].tp[0][0] = W
    blocks[1].sp = [[D, P, g.copy(), b.copy()]]
    use, errs, final = ob.select_blocks(blocks, x, threshold=1e-12)
    assert use == [0, 1, 0]
    assert errs[1] < 1e-24 and errs[0] > 1e-4 and errs[2] > 1e-4
    assert final < 1e-24
    # with a huge threshold everything is replaced and the error is that of the all-student network
    use2, errs2, final2 = ob.select_blocks(blocks, x, threshold=1e9)
    assert use2 == [1, 1, 1]
    ref = ob.network_forward(blocks, [0, 0, 0], x)[-1]
    assert final2 == ob.feature_mse(ob.network_forward(blocks, [1, 1, 1], x)[-1], ref)


def test_feature_mse_hand_value():
    a = np.array([[1.0, 2.0], [3.0, 4.0]])
    b = np.array([[1.0, 0.0], [0.0, 4.0]])
    assert ob.feature_mse(a, b) == (0 + 4 + 9 + 0) / 4


def test_identity_skip_adds_the_block_input_before_the_last_relu():
    """Candidates (c)/(d) of section 3.2: with an all-zero last pointwise layer and beta = 0 the stack contributes
    BatchNorm(0) = 0, so the block with a skip returns relu(x) = x for a post-ReLU input, and without one returns 0."""
    rng = np.random.default_rng(3)
    x = np.maximum(rng.normal(size=(2, 4, 5, 5)), 0)
    layers = [wl.Layer(wl.DWSEP3X3, 4, 4, 1, 1), wl.Layer(wl.DWSEP3X3, 4, 4, 1, 1)]
    sp = [[rng.normal(size=(4, 1, 3, 3)), rng.normal(size=(4, 4)), np.ones(4), np.zeros(4)],
          [rng.normal(size=(4, 1, 3, 3)), np.zeros((4, 4)), np.ones(4), np.zeros(4)]]
    with_skip = ob.block_forward(wl.Arch(2, 4, 5, 5, layers, shortcut=2), sp, x)
    without = ob.block_forward(wl.Arch(2, 4, 5, 5, layers), sp, x)
    assert np.array_equal(with_skip, x)
    assert np.array_equal(without, np.zeros_like(x))


# ------------------------------------------------------------------ inference-mode BatchNorm (reading R15)
def test_bn_inference_matches_torch_eval_batch_norm():
    rng = np.random.default_rng(11)
    z = rng.normal(size=(3, 5, 4, 6)) * 2 + 1
    g, b = rng.uniform(0.5, 1.5, 5), rng.normal(size=5)
    rm, rv = rng.normal(size=5), rng.uniform(0.3, 2.0, 5)
    got = ob.bn_inference(z, g, b, rm, rv, 1e-5)
    want = F.batch_norm(torch.from_numpy(z), torch.from_numpy(rm), torch.from_numpy(rv), torch.from_numpy(g),
                        torch.from_numpy(b), training=False, eps=1e-5).numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    # hand value: z = 3, mean 1, var 4 - eps, gamma 2, beta 0.5 -> 2 * (3 - 1) / 2 + 0.5
    one = ob.bn_inference(np.full((1, 1, 1, 1), 3.0), [2.0], [0.5], [1.0], [4.0 - 1e-5], 1e-5)
    assert abs(float(one[0, 0, 0, 0]) - 2.5) < 1e-14


def test_inference_forward_with_the_batch_moments_equals_the_training_forward():
    """With running statistics set to the batch's own moments both modes are the same function."""
    for name in ["ragged_residual_s2", "three_layers_skip_pool", "fullconv_first"]:
        w, x, t, blk = _setup(name)
        p, cache = ob.block_forward(w.student, blk.sp, x, keep=True)
        zs = [rec["z"] for rec in cache["layers"]]
        if w.student.shortcut == 1:
            zs.append(cache["layers"][-1]["zs"])
        running = [ob.batch_moments(z) for z in zs]
        q = ob.block_forward(w.student, blk.sp, x, running=running)
        np.testing.assert_allclose(q, p, rtol=0, atol=1e-11 * max(1.0, np.abs(p).max()))
        # and with other statistics it is a different function
        other = [(m + 0.3, v * 1.7) for m, v in running]
        assert np.abs(ob.block_forward(w.student, blk.sp, x, running=other) - p).max() > 1e-3


def test_running_statistics_follow_torch_and_the_closed_form():
    """Three steps of a one-layer student: the running mean equals torch BatchNorm2d's (momentum = 1 - decay), the
    running variance equals torch's once its unbiased batch variance is scaled back by (n-1)/n; with lr = 0 the
    batch moments repeat, so after k steps running = decay^k * start + (1 - decay^k) * moment."""
    w, x, t, blk = _setup("paper_task_2x2")
    decay = 0.9
    blk.bn_decay = decay
    k = 3
    nl = len(w.student.layers)
    p, cache = ob.block_forward(w.student, blk.sp, x, keep=True)
    z0 = cache["layers"][0]["z"]
    for _ in range(k):
        blk.student_step(x, t, 0.0)
    m, v = ob.batch_moments(z0)
    np.testing.assert_allclose(blk.s_running[0][0], (1 - decay ** k) * m, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(blk.s_running[0][1], decay ** k * 1.0 + (1 - decay ** k) * v, rtol=1e-12, atol=1e-14)
    bn = torch.nn.BatchNorm2d(z0.shape[1], eps=w.student.bn_eps, momentum=1 - decay).double()
    bn.train()
    for _ in range(k):
        bn(torch.from_numpy(z0))
    n = z0.size // z0.shape[1]
    np.testing.assert_allclose(blk.s_running[0][0], bn.running_mean.numpy(), rtol=1e-12, atol=1e-14)
    tv = decay ** k + (bn.running_var.numpy() - decay ** k) * (n - 1) / n
    np.testing.assert_allclose(blk.s_running[0][1], tv, rtol=1e-12, atol=1e-14)
    assert len(blk.s_running) == nl and len(blk.t_running) == len(blk.tp)
    # the teacher's pair is never touched by a student step
    assert all(np.all(a == 0) and np.all(b == 1) for a, b in blk.t_running)


def test_running_statistics_move_with_training_and_cover_the_shortcut():
    w, x, t, blk = _setup("ragged_residual_s2")
    nl = len(w.student.layers)
    assert len(blk.s_running) == nl + 1
    blk.student_step(x, t, 0.05)
    first = [[a.copy(), b.copy()] for a, b in blk.s_running]
    blk.student_step(x, t, 0.05)
    for (a0, b0), (a1, b1) in zip(first, blk.s_running):
        assert np.abs(a1 - a0).max() > 0 and np.abs(b1 - b0).max() > 0
    # step 1 of the first layer: 0.01 * batch moments of the first pre-BN output under the initial weights
    w2, x2, t2, fresh = _setup("ragged_residual_s2")
    _, cache = ob.block_forward(w2.student, fresh.sp, x2, keep=True)
    m, v = ob.batch_moments(cache["layers"][0]["z"])
    np.testing.assert_allclose(first[0][0], 0.01 * m, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(first[0][1], 0.99 + 0.01 * v, rtol=1e-12, atol=1e-15)


def test_network_forward_in_inference_mode_composes_the_inference_blocks():
    blocks, x = _three_small_blocks()
    rng = np.random.default_rng(3)
    for blk in blocks:
        for pair in blk.t_running + blk.s_running:
            pair[0] = rng.normal(size=pair[0].shape) * 0.2
            pair[1] = rng.uniform(0.5, 1.5, pair[1].shape)
    outs = ob.network_forward(blocks, [1, 0, 1], x, bn_mode=1)
    a = ob.block_forward(blocks[0].student, blocks[0].sp, x, running=blocks[0].s_running)
    b = ob.block_forward(blocks[1].teacher, blocks[1].tp, a, running=blocks[1].t_running)
    c = ob.block_forward(blocks[2].student, blocks[2].sp, b, running=blocks[2].s_running)
    for got, want in zip(outs, (a, b, c)):
        assert np.array_equal(got, want)
    assert np.abs(outs[-1] - ob.network_forward(blocks, [1, 0, 1], x)[-1]).max() > 1e-3
    # in inference mode an image's features do not depend on the rest of the batch
    solo = ob.network_forward(blocks, [1, 0, 1], x[1:2], bn_mode=1)[-1]
    np.testing.assert_allclose(solo[0], outs[-1][1], rtol=0, atol=1e-12)


def test_bn_backward_is_linear_in_g_and_z_for_the_weight_gradient():
    """The first layer's weight-gradient kernel folds its BatchNorm backward in by linearity (no dz is formed):
    dz = scale*g - scale/m*dbeta - scale/m*dgamma*rstd*(z - mean), hence
    dW = scale*W(g) - scale/m*dgamma*rstd*W(z - mean) - scale/m*dbeta*W(1), W(.) = the convolution's weight gradient
    of its argument.  Checked with the oracle's own BatchNorm backward and weight gradient on a ragged shape."""
    rng = np.random.default_rng(5)
    N, Ci, Co, H, Wd = 3, 3, 5, 7, 12
    x = rng.standard_normal((N, Ci, H, Wd))
    z = 4.0 + 0.5 * rng.standard_normal((N, Co, H, Wd))              # means several standard deviations from zero
    gamma, beta = 0.5 + rng.random(Co), rng.standard_normal(Co)
    g = rng.standard_normal((N, Co, H, Wd)) * (rng.random((N, Co, H, Wd)) > 0.4)   # masked, as behind a ReLU
    xhat, _, mean, rstd = ob.bn_fwd(z, gamma, beta, 1e-5)
    dz, dgamma, dbeta = ob.bn_bwd(g, xhat, gamma, rstd)
    direct = ob.conv3x3_wgrad(dz, x)
    m = N * H * Wd
    scale = gamma * rstd
    zc = z - mean[None, :, None, None]
    ones = np.ones_like(z)
    w_g, w_z, w_1 = ob.conv3x3_wgrad(g, x), ob.conv3x3_wgrad(zc, x), ob.conv3x3_wgrad(ones, x)
    s = lambda v: v[:, None, None, None]
    folded = s(scale) * w_g - s(scale / m * dgamma * rstd) * w_z - s(scale / m * dbeta) * w_1
    assert np.max(np.abs(folded - direct)) <= 1e-12 * max(1.0, np.max(np.abs(direct)))
