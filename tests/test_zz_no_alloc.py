"""GPU test of pbkd_feature_mse_noalloc, the entry point for callers that cannot allocate device memory: its
scratch is a static device array of the library instead of a block's workspace.  It must give what
pbkd_feature_mse gives (same kernels, same fixed summation order: the same bits) and what the plain fp64
definition mean((a - b)^2) gives, on two calls in a row, the second with a smaller input (the array keeps
the first call's contents).  Also: sizes beyond the stated maximum are refused before anything is launched.
"""
import ctypes

import numpy as np
import pytest

from paper_2012_03096_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_feature_mse_noalloc_matches_workspace_variant_twice():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2012_03096_amd import binding as pb
    pb.lib()
    w = wl.cfg1_tiny()
    x, tp, sp = w.tensors()
    blk = pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum)
    rng = np.random.default_rng(77)
    # two calls in a row: 1 000 003 elements (ragged against the 256 x 256 grid), then 4 099
    for n in (1_000_003, 4_099):
        a = rng.standard_normal(n).astype(np.float32)
        b = (a + 0.25 * rng.standard_normal(n)).astype(np.float32)
        ad, bd = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()
        torch.cuda.synchronize()
        print(f"feature_mse_noalloc n={n}", flush=True)
        got = pb.feature_mse_noalloc(ad, bd)
        ref_ws = pb.feature_mse(blk, ad, bd)
        exact = float(np.mean((a.astype(np.float64) - b.astype(np.float64)) ** 2))
        assert got == ref_ws, (n, got, ref_ws)
        assert abs(got - exact) <= 1e-12 * exact, (n, got, exact)
    # on a side stream as well
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        got = pb.feature_mse_noalloc(ad, bd, stream=s)
    assert got == ref_ws
    blk.close()


def test_feature_mse_noalloc_rejects_sizes_beyond_the_maximum():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2012_03096_amd import binding as pb
    L = pb.lib()
    ad = torch.zeros(16, dtype=torch.float32, device="cuda")
    out = ctypes.c_double(-1.0)
    st = L.pbkd_feature_mse_noalloc(ctypes.c_void_p(ad.data_ptr()), ctypes.c_void_p(ad.data_ptr()), (1 << 32) + 1,
                                    ctypes.byref(out), ctypes.c_void_p(0))
    assert st == pb.EINVAL and "maximum" in pb.last_error()
    assert out.value == -1.0
    st = L.pbkd_feature_mse_noalloc(ctypes.c_void_p(ad.data_ptr()), ctypes.c_void_p(ad.data_ptr()), 0, ctypes.byref(out),
                                    ctypes.c_void_p(0))
    assert st == pb.EINVAL
