"""The arithmetic the fp32-from-bf16 matrix products rely on, checked in numpy on the CPU: an fp32 value is the
exact sum of three bf16 pieces (bf16(x), bf16(x - hi), rest), and the six largest piece products reproduce the
product to within an fp32 rounding error.  (The GPU kernels are checked against the oracle in the gpu tests; this
file pins the identity and the error bound stated in the library's header.)"""
import numpy as np


def bf16_rne(x):
    """Round fp32 to the nearest bf16 (ties to even), returned as fp32."""
    b = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32)


def cut(x):
    x = np.asarray(x, dtype=np.float32)
    hi = bf16_rne(x)
    r = (x - hi).astype(np.float32)
    mid = bf16_rne(r)
    lo = (r - mid).astype(np.float32)
    return hi, mid, lo


def samples(seed, n=200000):
    rng = np.random.default_rng(seed)
    mant = rng.uniform(1.0, 2.0, n)
    expo = rng.integers(-60, 20, n)
    sign = rng.choice([-1.0, 1.0], n)
    x = (sign * mant * np.exp2(expo)).astype(np.float32)
    x[:16] = np.float32([0, 1, -1, 0.5, 1.0 + 2**-23, 1.0 - 2**-24, 3.0, 255.0, 256.0, 257.0, 1.00390625, 1.99999988,
                         2**-100, -2**-100, 65535.0, 0.1])
    return x


def test_three_pieces_sum_to_the_value_exactly():
    x = samples(1)
    hi, mid, lo = cut(x)
    assert np.array_equal(hi.astype(np.float64) + mid.astype(np.float64) + lo.astype(np.float64), x.astype(np.float64))
    # the rest fits a bf16 exactly: packing its upper 16 bits loses nothing
    assert np.array_equal(lo.view(np.uint32) & 0xFFFF, np.zeros_like(lo, dtype=np.uint32))
    ax = np.abs(x.astype(np.float64))
    assert np.all(np.abs(mid) <= 2.0**-8 * ax) and np.all(np.abs(lo) <= 2.0**-16 * ax)


def test_six_piece_products_are_within_an_fp32_rounding_error():
    x, y = samples(2), samples(3)
    xh, xm, xl = (p.astype(np.float64) for p in cut(x))
    yh, ym, yl = (p.astype(np.float64) for p in cut(y))
    six = xh * yh + xh * ym + xm * yh + xm * ym + xh * yl + xl * yh
    exact = x.astype(np.float64) * y.astype(np.float64)
    bound = 2.0**-23 * np.abs(exact)
    assert np.all(np.abs(six - exact) <= bound * 1.001)
    # the dropped products have either sign: no systematic shrinkage of positive data
    pos = (x > 0) & (y > 0)
    rel = (six[pos] - exact[pos]) / exact[pos]
    assert abs(rel.mean()) < 0.05 * np.abs(rel).mean() + 1e-12


def test_dot_product_matches_fp32_accuracy():
    """A 2048-term dot product of non-negative data (the shape of one projection output): six-piece products summed in
    fp32 are as close to the fp64 value as a plain fp32 dot product."""
    rng = np.random.default_rng(4)
    a = rng.random((64, 2048)).astype(np.float32)
    b = rng.random((64, 2048)).astype(np.float32)
    exact = (a.astype(np.float64) * b.astype(np.float64)).sum(axis=1)
    ah, am, al = cut(a)
    bh, bm, bl = cut(b)
    acc = np.zeros(64, dtype=np.float32)
    for k0 in range(0, 2048, 16):  # one matrix instruction sums 16 products into the fp32 accumulator
        s = slice(k0, k0 + 16)
        for p, q in ((al, bh), (ah, bl), (am, bm), (am, bh), (ah, bm), (ah, bh)):
            acc = (acc + (p[:, s].astype(np.float64) * q[:, s].astype(np.float64)).sum(axis=1).astype(np.float32)).astype(np.float32)
    plain = np.zeros(64, dtype=np.float32)
    for k0 in range(0, 2048, 16):
        s = slice(k0, k0 + 16)
        plain = (plain + (a[:, s].astype(np.float64) * b[:, s].astype(np.float64)).sum(axis=1).astype(np.float32)).astype(np.float32)
    e_split = np.abs(acc - exact) / exact
    e_plain = np.abs(plain - exact) / exact
    assert e_split.max() < 4e-6 and e_split.mean() < 3 * e_plain.mean() + 1e-7
