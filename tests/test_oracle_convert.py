"""binary16 conversions of the CPU checker, pinned against numpy's float16."""
import numpy as np


def test_half_to_double_all_patterns(orc):
    bits = np.arange(65536, dtype=np.uint16)
    got = orc.half_to_double(bits)
    ref = bits.view(np.float16).astype(np.float64)
    both_nan = np.isnan(got) & np.isnan(ref)
    assert np.array_equal(got[~both_nan], ref[~both_nan])
    assert np.array_equal(np.signbit(got[~both_nan]), np.signbit(ref[~both_nan]))


def test_float_to_half_rne_random_and_edges(orc):
    rng = np.random.default_rng(1)
    x = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * np.float32(100),
        rng.uniform(-1e-4, 1e-4, 100000).astype(np.float32),          # subnormal range
        rng.integers(0, 2**32, 400000, dtype=np.uint64).astype(np.uint32).view(np.float32),
        np.array([0.0, -0.0, 65504, 65519.99, 65520, 1e9, -1e9, 2**-24, 2**-25, np.nextafter(np.float32(2**-25), np.float32(1)),
                  2**-14, np.inf, -np.inf], np.float32),
    ])
    x = x[~np.isnan(x)]
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    got = orc.float_to_half_bits(x)
    assert np.array_equal(got, ref)


def test_float_to_half_exact_ties(orc):
    # midpoints between adjacent halves must go to the even neighbour
    h = np.arange(0x0000, 0x7bff, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = ((lo + hi) / 2).astype(np.float32)         # exactly representable in binary32
    assert np.array_equal(mid.astype(np.float64), (lo + hi) / 2)
    got = orc.float_to_half_bits(mid)
    even = np.where(h % 2 == 0, h, h + 1).astype(np.uint16)
    assert np.array_equal(got, even)
