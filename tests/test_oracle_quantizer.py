"""Pins of the oracle's group quantizer (paper Sec. 3.2.2) against what the mathematics fixes."""
import numpy as np
import pytest

BITS = [1, 2, 3, 4]


def f16(x):
    return np.asarray(x, dtype=np.float64).astype(np.float16)


def qmax_i(bits):
    q = np.full(32, 2 ** bits - 1)
    if bits == 3:
        q[[10, 21]] = 3  # the 11th element of each block of 11 (q_max case equation)
    return q


def run(ref, x16, bits):
    codes, s, z = ref.quantize_group(x16.view(np.uint16), bits)
    deq = ref.dequant_group(codes, bits, s, z)
    return codes.astype(int), np.uint16(s).view(np.float16).astype(np.float64), np.uint16(z).view(np.float16).astype(np.float64), deq


def groups(seed, n):
    rng = np.random.default_rng(seed)
    for i in range(n):
        kind = i % 6
        if kind == 0:
            x = rng.standard_normal(32)
        elif kind == 1:
            x = rng.standard_normal(32) * 10 + 3
        elif kind == 2:
            x = rng.uniform(-1e-3, 1e-3, 32)
        elif kind == 3:
            x = rng.standard_normal(32) * 2000
        elif kind == 4:
            x = rng.choice([-2.5, 0.0, 1.0, 7.0], 32)
        else:
            x = rng.uniform(-6e-5, 6e-5, 32)  # fp16 subnormal territory
        yield f16(x)


@pytest.mark.parametrize("bits", BITS)
def test_nearest_level_and_round_trip_bound(ref, bits):
    """Codes equal a brute-force nearest-level search in binary64 (ties aside) and the round trip
    obeys |x - x~| <= s_i/2 (Sec. 3.2.2 steps 2-4)."""
    qm = qmax_i(bits)
    for x16 in groups(10 + bits, 600):
        codes, s, z, deq = run(ref, x16, bits)
        x = x16.astype(np.float64)
        assert z == x.min()
        assert np.all(codes >= 0) and np.all(codes <= qm)
        if s == 0:
            assert np.all(codes == 0) and np.all(deq == z)
            continue
        step = np.where(qm == 2 ** bits - 1, s, s * 7.0 / 3.0)
        # stored scale is the fp16 rounding of range / qmax
        assert abs(s - (x.max() - x.min()) / (2 ** bits - 1)) <= 2.0 ** -11 * s * 1.01 + 2.0 ** -25
        levels = np.arange(0, 16)[None, :] * step[:, None] + z          # [32, 16]
        levels = np.where(np.arange(16)[None, :] <= qm[:, None], levels, np.inf)
        best = np.abs(x[:, None] - levels).min(1)
        mine = np.abs(x - (codes * step + z))
        assert np.all(mine <= best + 1e-6 * step + 1e-12), (x, codes)
        assert np.all(np.abs(x - deq) <= step / 2 * (1 + 2.0 ** -20) + 1e-12)
        # dequant is q*s + min on the stored quantities
        assert np.all(np.abs(deq - (codes * step + z)) <= 2.0 ** -21 * (np.abs(codes * step) + abs(z)))
        assert codes[np.argmin(x)] == 0


@pytest.mark.parametrize("bits", BITS)
def test_closed_forms(ref, bits):
    q = 2 ** bits - 1
    # constant group: zero range -> scale 0, codes 0, exact reconstruction
    codes, s, z, deq = run(ref, f16(np.full(32, 1.25)), bits)
    assert s == 0 and z == 1.25 and not codes.any() and np.all(deq == 1.25)
    # two-valued group: {0, qmax_i}
    x = np.where(np.arange(32) % 2 == 0, -3.0, 5.0)
    codes, s, z, deq = run(ref, f16(x), bits)
    assert np.array_equal(codes, np.where(np.arange(32) % 2 == 0, 0, qmax_i(bits)))
    # exactly representable ladder min + k*s with s = 0.5: codes == k, exact round trip
    k = np.arange(32) % (q + 1)
    if bits == 3:
        k[[10, 21]] = [0, q]  # 2-bit elements: put them on levels they can represent (0 and range)
    codes, s, z, deq = run(ref, f16(-1.0 + 0.5 * k), bits)
    assert s == 0.5 and z == -1.0
    want = k.copy()
    if bits == 3:
        want[[10, 21]] = [0, 3]
    assert np.array_equal(codes, want)
    assert np.allclose(deq, -1.0 + 0.5 * k, rtol=1e-7)
    # negative zero minimum is stored as +0
    x = np.zeros(32)
    x[0] = -0.0
    x[1] = 3.0
    _, s_b, z_b = ref.quantize_group(f16(x).view(np.uint16), bits)
    assert z_b == 0
    # a zero-range group stores scale +0 and codes 0 whatever the signs and order of its zeros
    for first in (0.0, -0.0):
        x = np.where(np.arange(32) % 3 == 0, -0.0, 0.0)
        x[0] = first
        codes, s_b, z_b = ref.quantize_group(f16(x).view(np.uint16), bits)
        assert s_b == 0 and z_b == 0 and not codes.any()


@pytest.mark.parametrize("bits", BITS)
def test_monotone_and_extremes(ref, bits):
    qm = qmax_i(bits)
    for x16 in groups(77, 200):
        codes, s, z, _ = run(ref, x16, bits)
        if s == 0:
            continue
        x = x16.astype(np.float64)
        full = qm == 2 ** bits - 1
        order = np.argsort(x[full], kind="stable")
        assert np.all(np.diff(codes[full][order]) >= 0)
        # the maximum maps to q_max_i of its position, the minimum to 0
        assert codes[np.argmax(x)] == qm[np.argmax(x)]
        assert codes[np.argmin(x)] == 0


def test_three_bit_block_of_eleven(ref):
    """3-bit: elements 10 and 21 carry 2-bit codes whose step is range/3 (q_max = 3 for i = 10)."""
    x = f16(np.linspace(0.0, 7.0, 32))
    x[10] = 7.0
    x[21] = 7.0 * 2 / 3
    codes, s, z, deq = run(ref, x, 3)
    assert s == 1.0 and codes[10] == 3 and codes[21] == 2
    assert np.isclose(deq[10], 7.0) and np.isclose(deq[21], 14.0 / 3.0, rtol=1e-6)
    assert codes.max() == 7


def test_half_even_ties(ref):
    """x - min exactly halfway between levels rounds to the even code (reading: rint)."""
    k = np.arange(32) % 4
    x = 0.0 + 1.0 * k
    x[5] = 0.5   # tie between 0 and 1 -> 0
    x[6] = 1.5   # tie between 1 and 2 -> 2
    x[7] = 2.5   # tie between 2 and 3 -> 2
    codes, s, z, _ = run(ref, f16(x), 2)
    assert s == 1.0 and (codes[5], codes[6], codes[7]) == (0, 2, 2)


def test_extreme_range(ref):
    for bits in BITS:
        # the step (max - min) / q_max is stored as fp16: with one bit it is the range itself, which has to
        # stay below the fp16 maximum (precondition of the 1-bit setting)
        top = 65504.0 if bits > 1 else 32000.0
        x = np.zeros(32)
        x[0] = -top
        x[1] = top
        codes, s, z, deq = run(ref, f16(x), bits)
        assert np.isfinite(s) and codes[0] == 0 and codes[1] == 2 ** bits - 1
        step = np.where(qmax_i(bits) == 2 ** bits - 1, s, s * 7 / 3)
        assert np.all(np.abs(deq - x) <= step / 2 * 1.001)


def test_one_bit_range_beyond_fp16_is_stored_as_largest_fp16(ref):
    """With one bit the step is the range itself (Sec. 3.2.2 step 1 with q_max = 1), and fp16 inputs can span up to
    2 * 65504: such a step is stored as 65504, the codes are taken against the stored step (every element at or
    above min + 65504/2 gets code 1), and everything stays finite; the lower half keeps its exact level."""
    for lo, hi in ((-65504.0, 65504.0), (-40000.0, 30000.0), (-1.0, 65504.0), (0.0, 65504.0)):
        x = np.linspace(lo, hi, 32)
        codes, s, z, deq = run(ref, f16(x), 1)
        xr = f16(x).astype(np.float64)
        rng = xr.max() - xr.min()
        assert s == min(float(np.float16(min(rng, 65504.0))), 65504.0) and z == xr.min()
        assert np.all(np.isfinite(deq))
        t = (xr - xr.min()) / s
        want = np.clip(np.rint(t.astype(np.float32)), 0, 1)
        assert np.array_equal(codes, want.astype(int))
        assert codes[0] == 0 and codes[-1] == 1
        assert np.all(deq[codes == 0] == xr.min()) and np.all(deq[codes == 1] == xr.min() + s)
    # 2-4 bits: the largest possible range over q_max is always an fp16 number (no saturation to test)
    assert 2 * 65504.0 / 3 < 65504.0
