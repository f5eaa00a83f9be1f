"""The arithmetic behind the bf16 matrix-instruction kernels, checked on the CPU in numpy fp32.

An fp32 value is cut by truncation into three bf16 pieces that add up to it exactly; of the nine
piece products of a * b the six with weight >= 2^-16 are kept.  These tests pin what the kernels'
comments claim about that scheme: exactness of the cut, the size and the sign of the dropped
terms.  (The kernels themselves are compared with the oracle in the GPU tests.)
"""
import numpy as np


def cut3(x):
    x = np.asarray(x, np.float32)
    p1 = (x.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    r1 = (x - p1).astype(np.float32)
    p2 = (r1.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    r2 = (r1 - p2).astype(np.float32)
    p3 = (r2.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    return p1, p2, p3


def six_products(a, b):
    a1, a2, a3 = (p.astype(np.float64) for p in cut3(a))
    b1, b2, b3 = (p.astype(np.float64) for p in cut3(b))
    return a3 * b1 + a1 * b3 + a2 * b2 + a2 * b1 + a1 * b2 + a1 * b1


def samples():
    rng = np.random.default_rng(3)
    x = rng.standard_normal(200000).astype(np.float32) * np.float32(10.0) ** rng.integers(-6, 6, 200000).astype(np.float32)
    # adversarial mantissas: all ones, and the worst case of the dropped terms; magnitudes from 1e-30
    # to 3e38 (the cut is exact while the low pieces stay normal numbers, i.e. above about 2^-110)
    worst = np.float32(1.0 + 2.0 ** -7 - 2.0 ** -23)
    special = np.array([1.0, -1.0, worst, -worst, np.float32(2.0) - np.float32(2.0 ** -23), 3.0e38, 1.0e-30, 0.0],
                       np.float32)
    return np.concatenate([x, special])


def test_three_bf16_pieces_add_up_to_the_value_exactly():
    x = samples()
    p1, p2, p3 = cut3(x)
    for p in (p1, p2, p3):                                   # every piece is a bf16 number
        assert np.all((p.view(np.uint32) & np.uint32(0xFFFF)) == 0)
    assert np.array_equal(p1.astype(np.float64) + p2.astype(np.float64) + p3.astype(np.float64), x.astype(np.float64))


def test_dropped_terms_are_small_and_one_sided():
    x = samples()
    y = np.roll(x, 7)
    exact = x.astype(np.float64) * y.astype(np.float64)
    got = six_products(x, y)
    ok = exact != 0
    rel = (exact[ok] - got[ok]) / np.abs(exact[ok]) * np.sign(exact[ok])      # > 0: magnitude lost
    assert rel.max() <= 2.0 ** -20
    assert rel.min() >= 0.0                                  # truncation: never larger in magnitude
    worst = np.float32(1.0 + 2.0 ** -7 - 2.0 ** -23)
    lost = 1.0 - six_products(worst, worst) / (float(worst) ** 2)
    assert 4.0e-7 < lost < 2.0 ** -20                        # about 2^-21, the case named in the kernel's header
    assert 1e-8 < rel.mean() < 1e-7                          # a small bias that does not average out
