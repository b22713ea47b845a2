"""Pins the oracle's fp16 conversions to numpy's IEEE binary16 (an independent implementation)."""
import numpy as np


def test_h2d_all_patterns(ref):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([ref.h2d(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_d2h_matches_numpy_rne(ref):
    rng = np.random.default_rng(1)
    with np.errstate(over="ignore"):
        xs = np.concatenate([
            rng.standard_normal(20000) * 10.0 ** rng.integers(-9, 5, 20000),
            rng.standard_normal(2000).astype(np.float32).astype(np.float64),
            np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 70000.0, -65520.0, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
                      3 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11,
                      1.0 + 2.0 ** -11 + 2.0 ** -30, 2047.5, 2048.5, np.inf, -np.inf]),
        ])
        # every midpoint between adjacent fp16 values (ties) and its neighbours
        h = np.arange(0, 0x7bff, 7, dtype=np.uint16)
        a = h.view(np.float16).astype(np.float64)
        b = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
        mid = (a + b) / 2
        xs = np.concatenate([xs, mid, np.nextafter(mid, 0), np.nextafter(mid, np.inf), -mid])
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([ref.d2h(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)
