"""The claims behind the split contraction arithmetic (fp32 operands as three bf16 pieces, six of
the nine partial products), checked in numpy on the CPU: the decomposition is exact, the pieces
shrink by 2^-8 each, and what the three omitted products amount to.  This is arithmetic of the
number formats only; the kernel itself is compared with fp64 in tests/test_gpu_kernels.py."""
import numpy as np


def bf16_rne(x):
    """fp32 -> nearest bf16 (ties to even), returned as fp32."""
    u = np.asarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def pieces(x):
    x = np.asarray(x, np.float32)
    h = bf16_rne(x)
    r = x - h                      # exact in fp32
    m = bf16_rne(r)
    l = bf16_rne(r - m)
    return h, m, l


def _samples():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(200000).astype(np.float32) * np.exp2(rng.integers(-60, 60, 200000)).astype(np.float32)
    edge = np.array([1.0, -1.0, 0.0, 1.0 + 2.0 ** -23, 2.0 - 2.0 ** -23, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -9,
                     1.0 + 3 * 2.0 ** -9, 255.5, 0.1, -0.3, 3.0e-30, 7.0e29], np.float32)
    return np.concatenate([x, edge])


def test_three_pieces_reproduce_every_fp32_value_exactly():
    x = _samples()
    h, m, l = pieces(x)
    assert np.array_equal(h.astype(np.float64) + m.astype(np.float64) + l.astype(np.float64), x.astype(np.float64))
    # each piece is a bf16 value: conversion leaves it unchanged
    for p in (h, m, l):
        assert np.array_equal(bf16_rne(p), p)
    nz = x != 0
    assert (np.abs(m[nz]) <= np.abs(x[nz]) * 2.0 ** -8).all()
    assert (np.abs(l[nz]) <= np.abs(x[nz]) * 2.0 ** -16).all()


def test_cut_off_pieces_are_exact_too_but_biased():
    """Pieces cut off instead of rounded also add up exactly; every piece then has the sign of the
    value, so the omitted products all pull a product towards zero (the reason they were rejected)."""
    x = _samples()
    cut = lambda v: (np.asarray(v, np.float32).view(np.uint32) & 0xFFFF0000).view(np.float32)
    h = cut(x); r = x - h; m = cut(r); l = r - m
    assert np.array_equal(h.astype(np.float64) + m.astype(np.float64) + l.astype(np.float64), x.astype(np.float64))
    assert (np.sign(m) * np.sign(x) >= 0).all() and (np.sign(l) * np.sign(x) >= 0).all()
    hr, mr, lr = pieces(x)
    assert (np.sign(mr) * np.sign(x) < 0).any()          # rounded pieces take both signs


def test_six_products_miss_at_most_2_to_minus_23_of_a_product():
    rng = np.random.default_rng(1)
    a = rng.standard_normal(100000).astype(np.float32)
    b = (rng.standard_normal(100000) * 3).astype(np.float32)
    pa, pb = [p.astype(np.float64) for p in pieces(a)], [p.astype(np.float64) for p in pieces(b)]
    kept = (pa[0] * pb[0] + pa[0] * pb[1] + pa[1] * pb[0] + pa[1] * pb[1] + pa[0] * pb[2] + pa[2] * pb[0])
    exact = a.astype(np.float64) * b.astype(np.float64)
    rel = np.abs(kept - exact) / np.abs(exact)
    assert rel.max() <= 2.0 ** -23, rel.max()           # |m| <= 2^-8 |x|, |l| <= 2^-16 |x|: m l' + l m' + l l'
    assert np.mean(rel) <= 2.0 ** -26, np.mean(rel)
    # unbiased: the omitted part is as often above as below
    assert abs(np.mean(np.sign(kept - exact) * np.sign(exact))) < 0.02
    # a bf16 x bf16 product has at most 16 significant bits: exact in an fp32 accumulator
    prod = (pa[0] * pb[0]).astype(np.float32).astype(np.float64)
    assert np.array_equal(prod, pa[0] * pb[0])


def test_a_dot_product_from_the_six_products_is_as_good_as_an_fp32_one():
    """K = 800 terms, the six kept partial products summed in fp32 (any order of an fp32
    accumulator) against a plain fp32 dot product, both measured on fp64."""
    rng = np.random.default_rng(2)
    n, K = 200, 800
    a = (rng.standard_normal((n, K)) * 0.05).astype(np.float32)
    b = (rng.standard_normal((n, K)) * 0.05).astype(np.float32)
    exact = (a.astype(np.float64) * b.astype(np.float64)).sum(axis=1)
    scale = (np.abs(a).astype(np.float64) * np.abs(b).astype(np.float64)).sum(axis=1)
    pa, pb = pieces(a), pieces(b)
    acc = np.zeros(n, np.float32)
    # (the kernel adds the six products of a k-tile one after the other; here piece pair by piece pair:
    # the error level is the same for either order)
    for i, j in ((2, 0), (0, 2), (1, 1), (1, 0), (0, 1), (0, 0)):
        prod = pa[i] * pb[j]                                           # exact: 16 significant bits
        for k0 in range(0, K, 16):                                     # one MFMA step of 16 k at a time
            acc = (acc + prod[:, k0:k0 + 16].sum(axis=1, dtype=np.float32)).astype(np.float32)
    plain = np.zeros(n, np.float32)
    for k in range(K):
        plain = (plain + a[:, k] * b[:, k]).astype(np.float32)
    err_split = np.abs(acc.astype(np.float64) - exact) / scale
    err_plain = np.abs(plain.astype(np.float64) - exact) / scale
    assert err_split.max() < 5e-7, err_split.max()
    assert err_split.mean() <= 2.0 * err_plain.mean() + 1e-9, (err_split.mean(), err_plain.mean())
