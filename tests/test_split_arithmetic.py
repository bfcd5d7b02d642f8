"""The arithmetic behind the fp32 tile kernels, checked on the CPU in numpy: an fp32 value is exactly the sum
of three bf16 values obtained by truncation, and the six leading partial products of two such triples miss
the exact product by less than 2^-23 of its magnitude.  (Host-side check of the derivation that the kernels'
comments and the tolerance of the fp32 tile path rest on; the kernels themselves are tested on the GPU.)"""
import numpy as np


def upper_half(x):
    """The bf16 value made of the upper 16 bits of an fp32 value (truncation), as fp32."""
    return (x.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)


def triple(x):
    h = upper_half(x)
    r = x - h                      # exact: the low 16 bits of the significand, renormalised
    m = upper_half(r)
    l = upper_half(r - m)
    return h, m, l


def sample(rng, n):
    mant = rng.integers(0, 1 << 23, n, dtype=np.uint32)
    expo = rng.integers(1 + 40, 255 - 40, n, dtype=np.uint32)          # normal numbers, remainders stay normal
    sign = rng.integers(0, 2, n, dtype=np.uint32)
    return ((sign << np.uint32(31)) | (expo << np.uint32(23)) | mant).view(np.float32)


def test_an_fp32_value_is_exactly_three_truncated_bf16_values():
    rng = np.random.default_rng(0)
    x = np.concatenate([sample(rng, 200000), np.float32([0.0, -0.0, 1.0, -1.0, 3.0, 1.0 + 2.0 ** -23,
                                                          np.finfo(np.float32).max, 2.0 ** -100])])
    h, m, l = triple(x)
    for part in (h, m, l):
        assert np.all((part.view(np.uint32) & np.uint32(0xFFFF)) == 0)           # each is a bf16 value
    assert np.array_equal(h.astype(np.float64) + m.astype(np.float64) + l.astype(np.float64), x.astype(np.float64))
    assert np.all(np.isfinite(h))                                                # truncation cannot overflow
    # magnitudes fall by at least 2^-8 per level (8 significant bits each), which is what bounds the dropped terms
    nz = x != 0
    assert np.all(np.abs(m[nz]) <= np.abs(x[nz]) * 2.0 ** -7)
    assert np.all(np.abs(l[nz]) <= np.abs(x[nz]) * 2.0 ** -15)


def test_six_partial_products_reach_fp32_accuracy_and_fewer_do_not():
    rng = np.random.default_rng(1)
    w, x = sample(rng, 200000), sample(rng, 200000)
    wh, wm, wl = (t.astype(np.float64) for t in triple(w))
    xh, xm, xl = (t.astype(np.float64) for t in triple(x))
    exact = w.astype(np.float64) * x.astype(np.float64)
    six = wh * xh + wh * xm + wm * xh + wh * xl + wm * xm + wl * xh
    assert np.all(np.abs(six - exact) <= np.abs(exact) * 2.0 ** -21)            # bound: 3 dropped terms of <= 2^-23 + margin
    assert np.abs(six - exact).max() / np.abs(exact).max() < 2.0 ** -22
    three = wh * xh + wh * xm + wm * xh                                          # what a 16-bit split would give
    assert (np.abs(three - exact) / np.abs(exact)).max() > 2.0 ** -17           # visibly worse: the test can tell
    # unit edge values: the adjacency entry is a small integer, exact in one bf16, and three products are exact
    a = rng.integers(1, 257, 200000).astype(np.float32)
    assert np.array_equal(upper_half(a), a)
    assert np.array_equal(a.astype(np.float64) * (xh + xm + xl), a.astype(np.float64) * x.astype(np.float64))
