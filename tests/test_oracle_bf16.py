"""Pins for the oracle's bfloat16 rounding and for the reduced-precision average: hand-written
boundary cases, PyTorch's own bfloat16 conversion (an independent library routine) on every
pattern of several binades and a strided sweep of all 2^32, round trip of every code; the mean
re-rounding by hand values and by its error bound."""
import numpy as np
import pytest
import torch

import oracle


def bits(x):
    return int(np.array([x], dtype=np.float32).view(np.uint32)[0])


BOUNDARY = [
    (1.0, 0x3F80), (-1.0, 0xBF80), (0.0, 0x0000), (-0.0, 0x8000),
    (1 + 2.0 ** -8, 0x3F80),               # tie -> even (down)
    (1 + 3 * 2.0 ** -8, 0x3F82),           # tie -> even (up)
    (1 + 2.0 ** -8 + 2.0 ** -23, 0x3F81),  # just above a tie
    (2 - 2.0 ** -8, 0x4000),               # rounding carries into the exponent
    (3.3895313892515355e38, 0x7F7F),       # largest finite bfloat16
    (3.3961775292304601e38, 0x7F80),       # half way to 2^128: tie -> even = infinity
    (3.4028234663852886e38, 0x7F80),       # largest float32 overflows
    (float("inf"), 0x7F80), (float("-inf"), 0xFF80),
    (2.0 ** -126, 0x0080),                 # smallest normal
    (2.0 ** -133, 0x0001),                 # smallest bfloat16 subnormal
    (2.0 ** -134, 0x0000),                 # tie between 0 and the smallest subnormal -> 0
    (3 * 2.0 ** -134, 0x0002),             # tie 1.5 -> 2
    (1e-45, 0x0000),
    (0.1, 0x3DCD),                         # 0x3DCCCCCD rounds up
]


@pytest.mark.parametrize("x,code", BOUNDARY)
def test_boundary_table(x, code):
    assert int(oracle.f32_to_bf16_bits(np.array([x], dtype=np.float32))[0]) == code


def test_nan_stays_nan_with_sign():
    for b in (0x7FC00000, 0xFFC00000, 0x7F800001, 0xFF80FFFF, 0x7FFFFFFF):
        x = np.array([b], dtype=np.uint32).view(np.float32)
        h = int(oracle.f32_to_bf16_bits(x)[0])
        assert (h & 0x7F80) == 0x7F80 and (h & 0x7F) != 0 and (h >> 15) == (b >> 31)


def _against_torch(pat):
    x = torch.from_numpy(pat.view(np.float32).copy())
    want = x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.f32_to_bf16_bits(pat.view(np.float32))
    nan = (pat & 0x7FFFFFFF) > 0x7F800000
    assert np.array_equal(got[~nan], want[~nan])
    assert ((got[nan] & 0x7F80) == 0x7F80).all() and ((got[nan] & 0x7F) != 0).all()


def test_against_library_conversion():
    # every pattern of the binades around 1, the subnormal range and the overflow edge
    for e in (0, 1, 126, 127, 128, 254):
        for sign in (0, 0x80000000):
            _against_torch((np.arange(1 << 23, dtype=np.uint64) + (sign | (e << 23))).astype(np.uint32))
    # every 97th pattern of all 2^32
    _against_torch(np.arange(0, 1 << 32, 97, dtype=np.uint64).astype(np.uint32))


def test_round_trip_every_non_nan_code():
    codes = np.arange(65536, dtype=np.uint16)
    codes = codes[((codes & 0x7F80) != 0x7F80) | ((codes & 0x7F) == 0)]
    wide = (codes.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(oracle.bf16_bits_to_f32(codes[:512]).view(np.uint32), wide[:512].view(np.uint32))
    assert np.array_equal(oracle.f32_to_bf16_bits(wide), codes)


def test_outer_step_bf16_rounds_each_worker():
    # delta = 1 + 2^-8 is a bfloat16 tie (-> 1.0) but exact in binary16
    th0 = np.zeros(1, dtype=np.float32)
    theta = -np.array([[1 + 2.0 ** -8], [1 + 2.0 ** -8]], dtype=np.float32)
    for pg, want in ((oracle.PG_F32, 1 + 2.0 ** -8), (oracle.PG_F16, 1 + 2.0 ** -8),
                     (oracle.PG_BF16, 1.0)):
        mean = oracle.outer_step(th0.copy(), np.zeros(1, dtype=np.float32), theta.copy(), 1.0, 0.0, pg)
        assert mean[0] == np.float32(want), pg


def test_mean_rerounding_by_hand():
    # binary16: deltas 1 and 1 + 2^-10 are exact; their mean 1 + 2^-11 is a tie -> 1.0
    th0 = np.zeros(2, dtype=np.float32)
    theta = -np.array([[1.0, 3e-5], [1 + 2.0 ** -10, 1e-5]], dtype=np.float32)
    keep = oracle.outer_step(th0.copy(), np.zeros(2, dtype=np.float32), theta.copy(), 1.0, 0.0,
                             oracle.PG_F16, round_mean=False)
    rnd = oracle.outer_step(th0.copy(), np.zeros(2, dtype=np.float32), theta.copy(), 1.0, 0.0,
                            oracle.PG_F16, round_mean=True)
    assert keep[0] == np.float32(1 + 2.0 ** -11) and rnd[0] == np.float32(1.0)
    # the re-rounded mean is itself a binary16 value, and the update used it
    h = oracle.f32_to_f16_bits(rnd)
    assert np.array_equal(oracle.f16_bits_to_f32(h), rnd)
    # FP32 pseudo-gradients ignore the switch
    a = oracle.outer_step(th0.copy(), np.zeros(2, dtype=np.float32), theta.copy(), 1.0, 0.0,
                          oracle.PG_F32, round_mean=True)
    b = oracle.outer_step(th0.copy(), np.zeros(2, dtype=np.float32), theta.copy(), 1.0, 0.0,
                          oracle.PG_F32, round_mean=False)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("pg,eps,tiny", [(1, 2.0 ** -11, 2.0 ** -25), (2, 2.0 ** -8, 0.0)])
def test_reduced_precision_mean_stays_within_its_rounding_bound(pg, eps, tiny):
    # "no noticeable impact": each rounding moves a value by at most eps relative (plus half the
    # subnormal spacing), so the reduced-precision mean is within that of the FP32 mean.
    rng = np.random.default_rng(3)
    k, n = 8, 20000
    th0 = rng.normal(scale=0.02, size=n).astype(np.float32)
    theta = (th0 - rng.normal(scale=4.87e-3, size=(k, n))).astype(np.float32)
    ref = oracle.outer_step(th0.copy(), np.zeros(n, dtype=np.float32), theta.copy(), 0.7, 0.9, 0)
    dmax = np.abs(th0[None, :].astype(np.float64) - theta).max(axis=0)
    for rm in (False, True):
        got = oracle.outer_step(th0.copy(), np.zeros(n, dtype=np.float32), theta.copy(), 0.7, 0.9,
                                pg, round_mean=rm)
        bound = (2 if rm else 1) * (eps * dmax + tiny) + 1e-9
        assert (np.abs(got.astype(np.float64) - ref) <= bound).all()
