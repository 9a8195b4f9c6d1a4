"""Pins for the oracle's binary16 casts: the IEEE 754 boundary cases written out by hand,
round trip over every binary16 code, monotonicity, and numpy's own float16 conversion (an
independent library routine) on every binary32 pattern of the exponents that matter plus a
strided sweep of all 2^32 patterns."""
import numpy as np
import pytest

import oracle


def f32(bits):
    return np.array([bits], dtype=np.uint32).view(np.float32)[0]


BOUNDARY = [
    # (float32 value, expected binary16 code, why)
    (np.float32(65504.0), 0x7BFF, "largest finite half"),
    (np.nextafter(np.float32(65520.0), np.float32(0)), 0x7BFF, "just below the overflow tie"),
    (np.float32(65520.0), 0x7C00, "tie between 65504 and 2^16 goes to even = inf"),
    (np.float32(1e9), 0x7C00, "overflow"),
    (np.float32(np.inf), 0x7C00, "+inf"),
    (np.float32(-np.inf), 0xFC00, "-inf"),
    (np.float32(2.0 ** -14), 0x0400, "smallest normal"),
    (np.float32(2.0 ** -14 * (1 - 2.0 ** -11)), 0x0400, "tie 0x3FF.8 -> even 0x400"),
    (np.float32(2.0 ** -14 * (1 - 2.0 ** -10)), 0x03FF, "largest subnormal"),
    (np.float32(2.0 ** -24), 0x0001, "smallest subnormal"),
    (np.float32(2.0 ** -25), 0x0000, "tie between 0 and 2^-24 goes to even = 0"),
    (np.nextafter(np.float32(2.0 ** -25), np.float32(1)), 0x0001, "just above that tie"),
    (np.float32(3 * 2.0 ** -25), 0x0002, "tie 1.5 -> even 2"),
    (np.float32(5 * 2.0 ** -25), 0x0002, "tie 2.5 -> even 2"),
    (np.float32(2.0 ** -26), 0x0000, "below half the smallest subnormal"),
    (np.float32(1e-45), 0x0000, "float32 subnormal"),
    (np.float32(1 + 2.0 ** -11), 0x3C00, "tie -> even (down)"),
    (np.float32(1 + 3 * 2.0 ** -11), 0x3C02, "tie -> even (up)"),
    (np.float32(1 + 2.0 ** -11 + 2.0 ** -23), 0x3C01, "just above a tie"),
    (np.float32(2 - 2.0 ** -11), 0x4000, "rounding carries into the exponent"),
    (np.float32(-0.0), 0x8000, "sign of zero kept"),
    (np.float32(0.0), 0x0000, "+0"),
    (np.float32(-1.0), 0xBC00, "-1"),
    (np.float32(0.1), 0x2E66, "0.1 = 0x3DCCCCCD -> 0x2E66"),
]


@pytest.mark.parametrize("x,code,why", BOUNDARY)
def test_boundary_table(x, code, why):
    assert int(oracle.f32_to_f16_bits(np.array([x]))[0]) == code, why
    assert int(oracle.f32_to_f16_bits(np.array([-x]))[0]) == code ^ 0x8000, why


def test_nan_maps_to_a_nan_with_the_sign_kept():
    for bits in (0x7FC00000, 0xFFC00000, 0x7F800001, 0xFFFFFFFF):
        h = int(oracle.f32_to_f16_bits(np.array([f32(bits)]))[0])
        assert (h & 0x7C00) == 0x7C00 and (h & 0x03FF) != 0 and (h >> 15) == (bits >> 31)


def test_widen_every_code_against_numpy():
    codes = np.arange(65536, dtype=np.uint16)
    got = oracle.f16_bits_to_f32(codes)
    want = codes.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_round_trip_every_non_nan_code():
    codes = np.arange(65536, dtype=np.uint16)
    codes = codes[((codes & 0x7C00) != 0x7C00) | ((codes & 0x03FF) == 0)]
    assert codes.size == 63490
    assert np.array_equal(oracle.f32_to_f16_bits(oracle.f16_bits_to_f32(codes)), codes)


def test_monotone_on_sorted_floats():
    rng = np.random.default_rng(0)
    x = np.sort(np.concatenate([
        rng.normal(scale=4.87e-3, size=200000), rng.normal(scale=1e-6, size=200000),
        rng.uniform(-70000, 70000, size=100000)]).astype(np.float32))
    h = oracle.f16_bits_to_f32(oracle.f32_to_f16_bits(x))
    assert (h[1:] >= h[:-1]).all()
    # and the rounding error is at most half a unit in the last place of the result
    fin = np.isfinite(h) & (np.abs(x) >= 2.0 ** -14)
    assert (np.abs(h[fin].astype(np.float64) - x[fin]) <= np.abs(x[fin]) * 2.0 ** -11).all()
    sub = np.abs(x) < 2.0 ** -14
    assert (np.abs(h[sub].astype(np.float64) - x[sub]) <= 2.0 ** -25).all()


def _check_range_against_numpy(first, n):
    pat = (np.arange(n, dtype=np.uint64) + first).astype(np.uint32)
    got = oracle.cast_pattern_range(first, n)
    with np.errstate(over="ignore"):
        want = pat.view(np.float32).astype(np.float16).view(np.uint16)
    nan = (pat & 0x7FFFFFFF) > 0x7F800000
    assert np.array_equal(got[~nan], want[~nan]), hex(first)
    assert ((got[nan] & 0x7C00) == 0x7C00).all() and ((got[nan] & 0x3FF) != 0).all()
    assert np.array_equal(got[nan] >> 15, (pat[nan] >> 31).astype(np.uint16))


def test_every_pattern_of_the_exponents_that_round():
    # Biased float32 exponents 100..143 hold everything from below 2^-26 up to beyond
    # 65520: every pattern of those binades, both signs, against numpy's float16 cast.
    for sign in (0, 0x80000000):
        for e in range(100, 144):
            _check_range_against_numpy(sign | (e << 23), 1 << 23)


def test_strided_sweep_of_all_patterns():
    # Every 251st pattern (a prime stride, so all low-bit combinations occur) of all 2^32.
    pat = np.arange(0, 1 << 32, 251, dtype=np.uint64).astype(np.uint32)
    got = oracle.f32_to_f16_bits(pat.view(np.float32))
    with np.errstate(over="ignore"):
        want = pat.view(np.float32).astype(np.float16).view(np.uint16)
    nan = (pat & 0x7FFFFFFF) > 0x7F800000
    assert np.array_equal(got[~nan], want[~nan])
    assert ((got[nan] & 0x7C00) == 0x7C00).all() and ((got[nan] & 0x3FF) != 0).all()


def test_found_inf_brute_force():
    # One special value at each position of small arrays; 65504 and subnormals do not count.
    specials16 = {0x7C00: 1, 0xFC00: 1, 0x7E00: 1, 0xFE01: 1, 0x7C01: 1,
                  0x7BFF: 0, 0xFBFF: 0, 0x0001: 0, 0x8000: 0}
    for n in (1, 2, 63, 64, 65, 200):
        base = np.random.default_rng(n).normal(scale=60, size=n).astype(np.float16).view(np.uint16)
        assert oracle.found_inf(base) == 0
        for pos in sorted({0, n // 2, n - 1}):
            for code, want in specials16.items():
                g = base.copy()
                g[pos] = code
                assert oracle.found_inf(g) == want, (n, pos, hex(code))
    specials32 = {np.inf: 1, -np.inf: 1, np.nan: 1, 3.4e38: 0, 1e-45: 0, -0.0: 0}
    for n in (1, 5, 129):
        base = np.random.default_rng(n).normal(size=n).astype(np.float32)
        assert oracle.found_inf(base) == 0
        for pos in sorted({0, n // 2, n - 1}):
            for val, want in specials32.items():
                g = base.copy()
                g[pos] = val
                assert oracle.found_inf(g) == want
                assert want == int(not np.isfinite(g).all())
