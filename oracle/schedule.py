"""CPU oracle for the block scheduler and the FLOP weights it balances.

TEST INFRASTRUCTURE ONLY (see block.py).  Section 3.3 of the paper: tasks with unequal run times are
items, workers are bins of unlimited capacity; the bin-packing policy is worst-fit-decreasing -- sort the
items by decreasing weight, then put each one into the currently emptiest bin.  Round-robin deals the
tasks out in their given order.  Work stealing needs no weights: every worker owns a queue of tasks and
serves it from the front; a worker that runs out of work takes a task from the tail of another worker's
queue (`work_stealing` simulates this for given task durations).

Readings: ties in the sort keep the lower task index first; ties between bins take the lowest bin index;
`order` is the position a task gets inside its bin.  The paper weighs tasks by measured run time; here
the default weight is a FLOP count (2 * multiply-accumulates of the convolutions only):
teacher forward + student forward + student weight gradients + student data gradients, where the data
gradient of the depthwise (or full) convolution of a block's FIRST layer is not counted because the
block input needs no gradient, and frozen layers count forward only.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

CONV3X3 = 0
DWSEP3X3 = 1


def wfd(weights: Sequence[int], n_bins: int) -> Tuple[List[int], List[int], List[int]]:
    """Worst-fit-decreasing.  Returns (bin_of_item, order_within_bin, bin_load)."""
    idx = sorted(range(len(weights)), key=lambda i: (-weights[i], i))
    load = [0] * n_bins
    count = [0] * n_bins
    bin_of = [0] * len(weights)
    order = [0] * len(weights)
    for i in idx:
        b = min(range(n_bins), key=lambda k: (load[k], k))
        bin_of[i] = b
        order[i] = count[b]
        count[b] += 1
        load[b] += weights[i]
    return bin_of, order, load


def round_robin(weights: Sequence[int], n_bins: int) -> Tuple[List[int], List[int], List[int]]:
    load = [0] * n_bins
    bin_of, order = [], []
    for i, w in enumerate(weights):
        b = i % n_bins
        bin_of.append(b)
        order.append(i // n_bins)
        load[b] += w
    return bin_of, order, load


def work_stealing(durations: Sequence[float], n_workers: int, queue_of_task: Sequence[int]):
    """Event-driven simulation of the work-stealing policy (section 3.3) for known task durations.
    Every worker serves its own queue from the front (tasks in index order); an idle worker with an empty
    queue steals from the TAIL of the queue that holds the most waiting tasks (ties: lowest worker index).
    Idle workers act in the order they became idle (ties: lowest worker index).
    Returns (ran_on[task], start[task], makespan, n_steals)."""
    from collections import deque
    queues = [deque() for _ in range(n_workers)]
    for t, q in enumerate(queue_of_task):
        queues[q].append(t)
    free_at = [0.0] * n_workers
    ran_on = [-1] * len(durations)
    start = [0.0] * len(durations)
    steals = 0
    remaining = len(durations)
    while remaining:
        w = min(range(n_workers), key=lambda k: (free_at[k], k))
        if queues[w]:
            t = queues[w].popleft()
        else:
            victim = max(range(n_workers), key=lambda k: (len(queues[k]), -k))
            t = queues[victim].pop()
            steals += 1
        ran_on[t] = w
        start[t] = free_at[w]
        free_at[w] += durations[t]
        remaining -= 1
    return ran_on, start, max(free_at) if durations else 0.0, steals


def _out(n, s):
    return (n - 1) // s + 1


def arch_flops(arch, backward: bool) -> int:
    """2*MACs of the block's convolutions.  backward=False: forward only.  backward=True: a training
    step (forward + weight gradients + data gradients as described in the module docstring)."""
    total = 0
    h, w = arch.h, arch.w
    for l, L in enumerate(arch.layers):
        ho, wo = _out(h, L.stride), _out(w, L.stride)
        pix = arch.n * ho * wo
        if L.kind == CONV3X3:
            f = 2 * 9 * L.cin * L.cout * pix
            total += f
            if backward and L.trainable:
                total += f                      # weight gradient
                if l > 0:
                    total += f                  # data gradient
        else:
            fd = 2 * 9 * L.cin * pix
            fp = 2 * L.cin * L.cout * pix
            total += fd + fp
            if backward and L.trainable:
                total += fd + fp                # weight gradients of both convolutions
                total += fp                     # data gradient of the pointwise
                if l > 0:
                    total += fd                 # data gradient of the depthwise
        h, w = ho, wo
    if arch.shortcut == 1:
        co = arch.layers[-1].cout
        ho, wo = _out(arch.h, arch.shortcut_stride), _out(arch.w, arch.shortcut_stride)
        total += 2 * arch.c * co * arch.n * ho * wo
    return total


def block_weight(teacher, student) -> int:
    return arch_flops(teacher, False) + arch_flops(student, True)
