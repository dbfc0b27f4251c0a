"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and its host-side
logic (descriptor validation, workspace sizing, FLOP counts, the block scheduler) agrees with the
oracle.  No kernel is launched here."""
import os
import re

import numpy as np
import pytest

from oracle import schedule as osched
from paper_2012_03096_amd import binding as pb
from paper_2012_03096_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pbkd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(pbkd_[a-z_]+)\s*\(", header))
    assert declared == set(pb.EXPORTS), declared ^ set(pb.EXPORTS)
    L = pb.lib()
    for name in declared:
        assert getattr(L, name) is not None


def _all_workloads():
    return [wl.cfg1_tiny(), wl.cfg2_vgg_block2(), wl.cfg3_resnet_down(), wl.cfg4_imagenet_vgg_block1()] + \
        wl.cfg5_vgg16_blocks() + wl.small_variants() + wl.paper_granularity_vgg16_tasks()


def test_validate_accepts_all_workloads_and_sizes_workspace():
    for w in _all_workloads():
        assert pb.arch_validate(w.teacher, w.student) == pb.OK, (w.name, pb.last_error())
        nbytes = pb.workspace_bytes(w.teacher, w.student)
        assert nbytes > 0 and nbytes % 256 == 0
    # the ImageNet-shaped block: seven 411 MB activation-sized tensors (teacher z1 z2; student z1 u2 z2; gradient ping-pong gz du)
    big = pb.workspace_bytes(*(lambda w: (w.teacher, w.student))(wl.cfg4_imagenet_vgg_block1()))
    assert 2.5e9 < big < 4e9


def test_flops_match_oracle_definition():
    for w in _all_workloads():
        assert pb.arch_flops(w.teacher, False) == osched.arch_flops(w.teacher, False), w.name
        assert pb.arch_flops(w.student, False) == osched.arch_flops(w.student, False), w.name
        assert pb.arch_flops(w.student, True) == osched.arch_flops(w.student, True), w.name


def test_validation_errors():
    w = wl.cfg1_tiny()
    bad = wl.Arch(4, 16, 16, 16, [wl.Layer(wl.DWSEP3X3, 16, 16, 1, 1), wl.Layer(wl.DWSEP3X3, 8, 16, 1, 1)])
    assert pb.arch_validate(w.teacher, bad) == pb.ESHAPE and "cin" in pb.last_error()
    bad = wl.Arch(4, 16, 16, 16, [wl.Layer(wl.DWSEP3X3, 16, 16, 1, 1), wl.Layer(wl.DWSEP3X3, 16, 8, 1, 1)])
    assert pb.arch_validate(w.teacher, bad) == pb.ESHAPE
    bad = wl.Arch(4, 16, 16, 16, [wl.Layer(wl.DWSEP3X3, 16, 16, 3, 1), wl.Layer(wl.DWSEP3X3, 16, 16, 1, 1)])
    assert pb.arch_validate(w.teacher, bad) == pb.EINVAL
    bad = wl.Arch(4, 16, 16, 16, [wl.Layer(wl.DWSEP3X3, 16, 16, 1, 1), wl.Layer(wl.CONV3X3, 16, 16, 1, 1)])
    assert pb.arch_validate(w.teacher, bad) == pb.EUNSUPPORTED
    bad = wl.Arch(4, 16, 16, 16, [wl.Layer(wl.DWSEP3X3, 16, 16, 1, 1), wl.Layer(wl.DWSEP3X3, 16, 16, 1, 0)])
    assert pb.arch_validate(w.teacher, bad) == pb.EUNSUPPORTED
    bad = wl.Arch(4, 16, 16, 16, [])
    assert pb.arch_validate(w.teacher, bad) == pb.EINVAL
    bad = wl.Arch(4, 16, 16, 16, w.student.layers, pool=3)
    assert pb.arch_validate(w.teacher, bad) == pb.EINVAL
    bad = wl.Arch(2, 16, 16, 16, w.student.layers)
    assert pb.arch_validate(w.teacher, bad) == pb.ESHAPE
    bad = wl.Arch(4, 16, 16, 16, w.student.layers, shortcut=1, shortcut_stride=2)
    assert pb.arch_validate(w.teacher, bad) == pb.ESHAPE
    assert pb.workspace_bytes(w.teacher, bad) == 0
    bad = wl.Arch(4, 16, 1, 1, w.student.layers, pool=2)
    assert pb.arch_validate(bad, bad) in (pb.ESHAPE, pb.EUNSUPPORTED)


@pytest.mark.parametrize("seed", range(10))
@pytest.mark.parametrize("policy", [0, 1])
def test_scheduler_matches_oracle(seed, policy):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(0, 14))
    m = int(rng.integers(1, 6))
    weights = [int(v) for v in rng.integers(1, 50, n)]       # small range: many ties
    got = pb.schedule_blocks(weights, m, policy)
    ref = (osched.wfd if policy == 0 else osched.round_robin)(weights, m)
    assert got[0] == ref[0] and got[1] == ref[1] and got[2] == ref[2]


def test_scheduler_on_vgg16_blocks_and_errors():
    blocks = wl.cfg5_vgg16_blocks()
    weights = [pb.arch_flops(b.teacher, False) + pb.arch_flops(b.student, True) for b in blocks]
    for m in (1, 2, 3, 4, 5, 7):
        got = pb.schedule_blocks(weights, m, 0)
        ref = osched.wfd(weights, m)
        assert got[0] == ref[0] and got[2] == ref[2]
    with pytest.raises(pb.PbkdError) as e:
        pb.schedule_blocks(weights, 0, 0)
    assert e.value.status == pb.EINVAL
    with pytest.raises(pb.PbkdError):
        pb.schedule_blocks(weights, 2, 5)
