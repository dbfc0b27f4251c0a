"""Pins for the scheduler oracle and the FLOP weights (CPU only)."""
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import schedule as osched
from paper_2012_03096_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_wfd_hand_replay():
    g = json.load(open(os.path.join(GOLDEN, "wfd_hand_example.json")))
    bin_of, order, load = osched.wfd(g["weights"], g["n_bins"])
    assert bin_of == g["bin_of_item"]
    assert order == g["order_within_bin"]
    assert load == g["bin_load"]


def _brute_optimum(weights, m):
    best = None
    for assign in itertools.product(range(m), repeat=len(weights)):
        load = [0] * m
        for w, b in zip(weights, assign):
            load[b] += w
        mk = max(load)
        best = mk if best is None else min(best, mk)
    return best


@pytest.mark.parametrize("seed", range(12))
def test_wfd_partition_and_lpt_bound(seed):
    """The assignment is a partition, loads add up, and -- worst-fit-decreasing with unbounded bins being
    longest-processing-time-first list scheduling -- makespan <= (4/3 - 1/(3m)) * optimum (Graham 1969)."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 9))
    m = int(rng.integers(1, 5))
    weights = [int(v) for v in rng.integers(1, 100, n)]
    bin_of, order, load = osched.wfd(weights, m)
    # a partition: every item is placed exactly once, in an existing bin
    assert len(bin_of) == n and len(order) == n and len(load) == m
    assert all(isinstance(b, int) and 0 <= b < m for b in bin_of)
    assert sum(load) == sum(weights)
    for b in range(m):
        items = [i for i in range(n) if bin_of[i] == b]
        assert sum(weights[i] for i in items) == load[b]
        assert sorted(order[i] for i in items) == list(range(len(items)))
        # within a bin the placement order follows decreasing weight
        by_order = sorted(items, key=lambda i: order[i])
        assert all(weights[a] >= weights[c] for a, c in zip(by_order[:-1], by_order[1:]))
    opt = _brute_optimum(weights, m)
    assert Fraction(max(load)) <= (Fraction(4, 3) - Fraction(1, 3 * m)) * opt


def test_round_robin():
    bin_of, order, load = osched.round_robin([5, 1, 4, 2, 3], 2)
    assert bin_of == [0, 1, 0, 1, 0] and order == [0, 0, 1, 1, 2] and load == [12, 3]


def test_ds_cost_ratio_matches_paper_claim():
    g = json.load(open(os.path.join(GOLDEN, "ds_cost_ratio.json")))
    for case in g["cases"]:
        ci, co = case["cin"], case["cout"]
        full = wl.Arch(2, ci, 8, 8, [wl.Layer(wl.CONV3X3, ci, co, 1, 0)])
        ds = wl.Arch(2, ci, 8, 8, [wl.Layer(wl.DWSEP3X3, ci, co, 1, 1)])
        r = Fraction(osched.arch_flops(ds, False), osched.arch_flops(full, False))
        assert r == Fraction(case["ratio_num"], case["ratio_den"]) == Fraction(1, co) + Fraction(1, 9)


def test_flop_weights_spelled_out_for_vgg_block2():
    """CIFAR-shaped VGG16 block 2, batch 128, written out term by term."""
    w = wl.cfg2_vgg_block2()
    pix = 128 * 16 * 16
    teacher = 2 * 9 * 64 * 128 * pix + 2 * 9 * 128 * 128 * pix
    dw1, pw1 = 2 * 9 * 64 * pix, 2 * 64 * 128 * pix
    dw2, pw2 = 2 * 9 * 128 * pix, 2 * 128 * 128 * pix
    fwd = dw1 + pw1 + dw2 + pw2
    step = fwd + (dw1 + pw1 + dw2 + pw2) + (pw1 + pw2 + dw2)     # + weight grads + data grads (no dw1 dgrad)
    assert osched.arch_flops(w.teacher, False) == teacher == 14_495_514_624
    assert osched.arch_flops(w.student, False) == fwd
    assert osched.arch_flops(w.student, True) == step == 5_133_828_096
    assert osched.block_weight(w.teacher, w.student) == teacher + step


def test_vgg16_five_block_schedule():
    """The five VGG16 stages at batch 128: weights, and the WFD assignment for 2, 3, 4 streams checked
    against brute force (WFD is optimal for 3 and 4 bins here and within the LPT bound for 2)."""
    blocks = wl.cfg5_vgg16_blocks()
    weights = [osched.block_weight(b.teacher, b.student) for b in blocks]
    assert weights[1] == 19_629_342_720
    # block 1: conv 3->64 kept full and trainable (forward + weight gradient), then one DS layer
    pix = 128 * 32 * 32
    conv, dw, pw = 2 * 27 * 64 * pix, 2 * 9 * 64 * pix, 2 * 64 * 64 * pix
    assert weights[0] == (conv + 2 * 9 * 64 * 64 * pix) + (2 * conv + 3 * (dw + pw))
    for m in (2, 3, 4):
        bin_of, order, load = osched.wfd(weights, m)
        opt = _brute_optimum(weights, m)
        assert max(load) >= opt
        assert Fraction(max(load)) <= (Fraction(4, 3) - Fraction(1, 3 * m)) * opt
        if m >= 3:
            assert max(load) == opt
    bin_of, _, _ = osched.wfd(weights, 5)
    assert sorted(bin_of) == [0, 1, 2, 3, 4]


# ------------------------------------------------------------------ work stealing (section 3.3)
def test_work_stealing_hand_example():
    """Four tasks of durations 5, 1, 1, 1, all queued on worker 0, two workers.  t=0: worker 0 takes task 0
    from the front of its queue; worker 1 has nothing and steals task 3 from the tail.  t=1: worker 1 is idle
    again and steals task 2; t=2: steals task 1; worker 0 finishes at 5.  Makespan 5, three steals."""
    ran_on, start, makespan, steals = osched.work_stealing([5, 1, 1, 1], 2, [0, 0, 0, 0])
    assert ran_on == [0, 1, 1, 1]
    assert start == [0.0, 2.0, 1.0, 0.0]
    assert makespan == 5.0 and steals == 3


def test_work_stealing_no_steal_when_balanced():
    ran_on, start, makespan, steals = osched.work_stealing([2, 2, 2, 2], 2, [0, 1, 0, 1])
    assert ran_on == [0, 1, 0, 1] and steals == 0 and makespan == 4.0


def test_work_stealing_properties_random():
    rng = np.random.default_rng(5)
    for trial in range(200):
        n, m = int(rng.integers(1, 14)), int(rng.integers(1, 6))
        d = [float(v) for v in rng.integers(1, 20, size=n)]
        q = [int(v) for v in rng.integers(0, m, size=n)]
        ran_on, start, makespan, steals = osched.work_stealing(d, m, q)
        assert sorted(range(n)) == sorted(i for i in range(n) if 0 <= ran_on[i] < m)      # every task once
        # no worker runs two tasks at once, and none idles while any task is still waiting anywhere
        for w in range(m):
            iv = sorted((start[i], start[i] + d[i]) for i in range(n) if ran_on[i] == w)
            for (a0, a1), (b0, b1) in zip(iv[:-1], iv[1:]):
                assert b0 >= a1 - 1e-12
        assert makespan >= max(max(d), sum(d) / m) - 1e-12
        assert makespan <= sum(d) / m + max(d) + 1e-12                                    # greedy list-scheduling bound
        # a task that stays on its own worker keeps queue order
        for w in range(m):
            own = [i for i in range(n) if q[i] == w and ran_on[i] == w]
            assert [start[i] for i in own] == sorted(start[i] for i in own)
