"""Pins for the oracle's delivery variants of the one-shot reduction (sum instead of mean, fp32
result from bf16 inputs) and for the learning-rate factors of paper section 6.2."""
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest

F32, BF16 = 0, 1


def _rand(oracle, rng, n, count, dtype):
    bufs = [np.ascontiguousarray(rng.normal(0, 1e-3, count).astype(np.float32)) for _ in range(n)]
    if dtype == BF16:
        bufs = [oracle.f32_to_bf16(b) for b in bufs]
    return bufs


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_defaults_are_the_plain_functions(oracle, dtype):
    rng = np.random.default_rng(30)
    n, count = 5, 48
    bufs = _rand(oracle, rng, n, count, dtype)
    for live in range(1, 1 << n):
        got = oracle.reduce_masked_ex(bufs, live, dtype)
        assert np.array_equal(got.view(np.uint8), oracle.reduce_masked(bufs, live, dtype).view(np.uint8))
        got = oracle.reduce_masked_ex(bufs, live, dtype, sum_only=True)
        want = oracle.reduce_masked(bufs, live, dtype, sum_only=True)
        assert np.array_equal(got.view(np.uint8), want.view(np.uint8))
        for zmask in (live & 0b00101, live & 0b11000):
            for contributors_only in (False, True):
                if contributors_only and zmask == live:
                    continue
                got = oracle.reduce_masked_ex(bufs, live, dtype, zero_mask=zmask,
                                              contributors_only=contributors_only)
                want = oracle.reduce_masked_zero(bufs, live, zmask, dtype, contributors_only)
                assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), (live, zmask)


def test_sum_is_the_hand_written_left_to_right_sum(oracle):
    rng = np.random.default_rng(31)
    bufs = _rand(oracle, rng, 4, 200, F32)
    s = ((bufs[0] + bufs[1]) + bufs[2]) + bufs[3]          # numpy float32 adds are IEEE single adds
    got = oracle.reduce_masked_ex(bufs, 0b1111, F32, sum_only=True)
    assert np.array_equal(got.view(np.uint32), s.view(np.uint32))
    mean = oracle.reduce_masked_ex(bufs, 0b1111, F32)
    assert np.array_equal(mean.view(np.uint32), (s * np.float32(0.25)).view(np.uint32))
    s3 = (bufs[0] + bufs[2]) + bufs[3]
    mean3 = oracle.reduce_masked_ex(bufs, 0b1101, F32)
    assert np.array_equal(mean3.view(np.uint32), (s3 * (np.float32(1) / np.float32(3))).view(np.uint32))
    # with a zero participant the divisor policy does not touch the sum
    a = oracle.reduce_masked_ex(bufs, 0b1111, F32, zero_mask=0b0010, sum_only=True)
    b = oracle.reduce_masked_ex(bufs, 0b1111, F32, zero_mask=0b0010, sum_only=True, contributors_only=True)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(a.view(np.uint32), (((bufs[0] + np.float32(0)) + bufs[2]) + bufs[3]).view(np.uint32))


def test_f32_result_from_bf16_inputs(oracle):
    rng = np.random.default_rng(32)
    n, count = 6, 300
    bufs = _rand(oracle, rng, n, count, BF16)
    wide = [oracle.bf16_to_f32(b) for b in bufs]
    for live in (0b111111, 0b101101, 0b000100):
        for sum_only in (False, True):
            got = oracle.reduce_masked_ex(bufs, live, BF16, out_dtype=F32, sum_only=sum_only)
            assert got.dtype == np.float32
            # widening is exact, so this is the fp32 reduction of the widened inputs ...
            want = oracle.reduce_masked(wide, live, F32, sum_only=sum_only)
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
            # ... and the bf16 result is its one rounding
            narrow = oracle.reduce_masked_ex(bufs, live, BF16, sum_only=sum_only)
            assert np.array_equal(oracle.f32_to_bf16(got), narrow)


def test_f32_sum_of_identical_bf16_inputs_is_exact(oracle):
    x = oracle.f32_to_bf16(np.linspace(-3, 3, 257, dtype=np.float32))
    for n in (2, 3, 5, 8, 16):
        got = oracle.reduce_masked_ex([x] * n, (1 << n) - 1, BF16, out_dtype=F32, sum_only=True)
        assert np.array_equal(got, oracle.bf16_to_f32(x) * np.float32(n))   # n*x needs <= 13 bits


def test_sum_with_zero_participants_equals_contributors_plus_zero_once(oracle):
    # x_1 + ... with +0.0 terms anywhere == (sum of the contributors) + 0.0, also for -0.0 inputs
    rng = np.random.default_rng(33)
    n, count = 5, 32
    bufs = _rand(oracle, rng, n, count, F32)
    for b in bufs:
        b[:4] = np.float32(-0.0)
    bufs[2][4:8] = np.float32(-0.0)
    for live in range(1, 1 << n):
        for zmask in range(1, 1 << n):
            if zmask & ~live or zmask == live:
                continue
            got = oracle.reduce_masked_ex(bufs, live, F32, zero_mask=zmask, sum_only=True)
            want = oracle.reduce_masked(bufs, live & ~zmask, F32, sum_only=True) + np.float32(0.0)
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (live, zmask)


def test_lr_factors_closed_forms(oracle):
    lin, root = oracle.lr_factors(8, 0xFF)
    assert lin == np.float32(1) and root == np.float32(1)
    lin, root = oracle.lr_factors(16, 0x000F)
    assert lin == np.float32(0.25) and root == np.float32(0.5)
    lin, root = oracle.lr_factors(16, 0x01FF)
    assert lin == np.float32(0.5625) and root == np.float32(0.75)
    # a zero-gradient participant is not healthy: 8 live of 16, 4 of them catching up
    lin, root = oracle.lr_factors(16, 0x00FF, 0x000F)
    assert lin == np.float32(0.25) and root == np.float32(0.5)
    lin, root = oracle.lr_factors(4, 0b0011, 0b0011)
    assert lin == 0 and root == 0
    with pytest.raises(oracle.OracleError):
        oracle.lr_factors(4, 0b0011, 0b0100)


def _round_f32(x: Decimal) -> np.float32:
    """Correctly rounded (nearest-even) binary32 of a positive Decimal below 2."""
    if x == 0:
        return np.float32(0)
    e = 0
    while x < 1:
        x *= 2
        e -= 1
    scaled = x * (1 << 23)                    # in [2^23, 2^24)
    lo = int(scaled)
    frac = scaled - lo
    if frac > Decimal("0.5") or (frac == Decimal("0.5") and lo & 1):
        lo += 1
    return np.float32(Fraction(lo, 1 << 23) * Fraction(2) ** e)


def test_lr_factors_are_correctly_rounded_for_every_count(oracle):
    getcontext().prec = 60
    for n in range(1, 65):
        for h in range(1, n + 1):
            lin, root = oracle.lr_factors(n, (1 << h) - 1)
            ratio = Decimal(h) / Decimal(n)
            assert lin == _round_f32(ratio), (h, n)
            assert root == _round_f32(ratio.sqrt()), (h, n)
