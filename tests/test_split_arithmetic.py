"""The arithmetic the teacher's bf16-split convolution relies on, checked on the CPU with numpy: an fp32 number is
exactly the sum of three bf16 numbers obtained by rounding to nearest three times, and the six cross products the
kernel forms differ from the exact product by at most 2^-24 of it (2^-27 rms, no bias): no more than the rounding of
one fp32 operation.  (The GPU kernel and the host routine that splits
the weights do these steps in hardware / in C++; this file pins the claim itself, independent of both.)"""
import numpy as np


def bf16_rn(x):
    """Nearest bf16 (ties to even) of fp32 values, returned as fp32."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return r.astype(np.uint32).view(np.float32)


def split3(x):
    x = np.asarray(x, dtype=np.float32)
    x0 = bf16_rn(x)
    r1 = x - x0                      # exact in fp32
    x1 = bf16_rn(r1)
    x2 = r1 - x1                     # exact, and itself a bf16 number
    return x0, x1, x2


def samples(n, seed):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(n).astype(np.float32)
    b = (rng.standard_normal(n) * np.exp2(rng.integers(-30, 30, n))).astype(np.float32)
    c = np.array([1.0, -1.0, 3.0, 255.0, 256.0, 257.0, 1.0 + 2.0 ** -23, 1.0 - 2.0 ** -24, 0.0, 2.0 ** -100, 3.4e38 / 4,
                  np.float32(1.00390625), np.float32(1.01171875)], dtype=np.float32)     # ties of the first rounding among them
    return np.concatenate([a, b, c])


def test_three_bf16_terms_are_the_number():
    x = samples(200_000, 1)
    x0, x1, x2 = split3(x)
    # every piece is a bf16 number (its low 16 bits are zero) ...
    for p in (x0, x1, x2):
        assert np.all(p.view(np.uint32) & 0xFFFF == 0)
    # ... and the three add up to x exactly (in fp64, where the sum of three fp32 numbers of this spread is exact)
    assert np.array_equal(x0.astype(np.float64) + x1.astype(np.float64) + x2.astype(np.float64), x.astype(np.float64))
    # magnitudes the error bound rests on
    nz = x != 0
    assert np.all(np.abs(x1[nz]) <= np.abs(x[nz]) * 2.0 ** -8)
    assert np.all(np.abs(x2[nz]) <= np.abs(x[nz]) * 2.0 ** -17)


def test_two_terms_are_not_enough():
    # the reason for three: with two roundings a remainder of up to 2^-17 |x| is left
    x = samples(50_000, 2)
    x0, x1, x2 = split3(x)
    assert np.any(x2 != 0)
    nz = x != 0
    assert np.max(np.abs(x2[nz] / x[nz])) > 2.0 ** -19


def test_six_products_are_within_one_fp32_rounding_of_the_product():
    rng = np.random.default_rng(3)
    x = samples(100_000, 4)
    w = rng.permutation(samples(100_000, 5))
    keep = (np.abs(x.astype(np.float64) * w.astype(np.float64)) < 1e30) & (np.abs(x.astype(np.float64) * w.astype(np.float64)) > 1e-30)
    x, w = x[keep], w[keep]
    xs = [p.astype(np.float64) for p in split3(x)]
    ws = [p.astype(np.float64) for p in split3(w)]
    six = sum(xs[i] * ws[j] for i in range(3) for j in range(3) if i + j <= 2)
    exact = x.astype(np.float64) * w.astype(np.float64)
    rel = (six - exact) / np.abs(exact)
    # the three terms left out: |x1 w2| + |x2 w1| <= 2 * 2^-8 * 2^-17, |x2 w2| <= 2^-34
    assert np.abs(rel).max() <= 2.0 ** -24, np.abs(rel).max()
    assert np.sqrt(np.mean(rel ** 2)) < 2.0 ** -27
    assert abs(rel.mean()) < 2.0 ** -32                  # rounding to nearest: no bias
    # each kept term is a product of two 8-bit significands: exact in fp32, hence in the MFMA's fp32 accumulation
    for i in range(3):
        for j in range(3):
            if i + j <= 2:
                t = xs[i] * ws[j]
                assert np.array_equal(t.astype(np.float32).astype(np.float64), t)


def test_dot_product_by_six_bf16_products_matches_fp32_accuracy():
    # a K = 1152 dot product (nine taps x 128 channels): the split sum, accumulated in fp32 term by term, against fp64
    rng = np.random.default_rng(6)
    K, n = 1152, 256
    x = np.maximum(rng.standard_normal((n, K)), 0).astype(np.float32)          # post-ReLU activations
    w = (rng.standard_normal((n, K)) * np.sqrt(2.0 / K)).astype(np.float32)    # He-initialised weights
    exact = np.sum(x.astype(np.float64) * w.astype(np.float64), axis=1)
    xs, ws = split3(x), split3(w)
    acc = np.zeros(n, dtype=np.float32)
    plain = np.zeros(n, dtype=np.float32)
    for k in range(K):
        for i, j in ((1, 0), (1, 1), (2, 0), (0, 0), (0, 1), (0, 2)):          # the kernel's order of the six products
            acc = acc + xs[j][:, k] * ws[i][:, k]                               # each product exact, one fp32 rounding per add
        plain = plain + x[:, k] * w[:, k]                                       # fp32 multiply-add chain (two roundings per term)
    scale = np.abs(exact).max()
    e_split = np.abs(acc - exact).max() / scale
    e_plain = np.abs(plain - exact).max() / scale
    assert e_split < 2e-6 and e_plain < 2e-6
    assert e_split < 4 * e_plain + 1e-7, (e_split, e_plain)


def test_ninth_tap_pairing_covers_the_six_products_once():
    # The ninth tap's products are paired by piece, two per MFMA (the half-waves supply different pieces): the tables
    # the host packer and the kernel share must name every (weight piece, activation piece) with i + j <= 2 exactly once.
    import os
    import re
    here = os.path.dirname(os.path.abspath(__file__))
    text = open(os.path.join(here, "..", "paper_2012_03096_amd", "csrc", "pbkd_internal.h")).read()

    def table(name):
        m = re.search(name + r"\[3\]\[2\] = \{\{(\d), (\d)\}, \{(\d), (\d)\}, \{(\d), (\d)\}\}", text)
        assert m, name
        v = [int(g) for g in m.groups()]
        return [(v[0], v[1]), (v[2], v[3]), (v[4], v[5])]

    w, x = table("kSplitLastW"), table("kSplitLastX")
    pairs = sorted((w[c][h], x[c][h]) for c in range(3) for h in range(2))
    assert pairs == sorted((i, j) for i in range(3) for j in range(3) if i + j <= 2)
