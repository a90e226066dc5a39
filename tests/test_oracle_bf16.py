"""Pins for the oracle's bf16 <-> fp32 conversion.

bf16 is the upper 16 bits of IEEE-754 binary32; narrowing rounds to nearest,
ties to even.  The pins are torch's own converter (an independent library
routine), the round trip over every bf16 pattern, and hand-picked ties.
"""
import numpy as np
import torch


def _torch_narrow(f32_bits: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(f32_bits.view(np.int32).copy()).view(torch.float32)
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _is_nan_bf16(h):
    return (h & 0x7FFF) > 0x7F80


def test_round_trip_all_bf16_patterns(oracle):
    h = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    f = oracle.bf16_to_f32(h)
    # widening is a pure bit placement: check against torch's widening
    t = torch.from_numpy(h.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32)
    assert np.array_equal(f.view(np.uint32), t.numpy().view(np.uint32))
    back = oracle.f32_to_bf16(f)
    nan = _is_nan_bf16(h)
    assert np.array_equal(back[~nan], h[~nan])
    assert np.all(_is_nan_bf16(back[nan]))
    assert np.array_equal(back[nan] & 0x8000, h[nan] & 0x8000)  # sign kept


def test_ties_and_overflow_by_hand(oracle):
    cases = {
        0x3F808000: 0x3F80,  # exactly half way, kept mantissa even -> stays
        0x3F818000: 0x3F82,  # exactly half way, kept mantissa odd -> up
        0x3F808001: 0x3F81,  # just above half way -> up
        0x3F807FFF: 0x3F80,  # just below half way -> down
        0x7F7FFFFF: 0x7F80,  # largest finite fp32 -> +inf
        0xFF7FFFFF: 0xFF80,  # -> -inf
        0x7F7F7FFF: 0x7F7F,  # below half way of the last bf16 binade -> largest finite bf16
        0x7F800000: 0x7F80,  # inf stays inf
        0x00000000: 0x0000,
        0x80000000: 0x8000,  # -0 keeps its sign
        0x00008000: 0x0000,  # denormal tie -> even (zero)
        0x00008001: 0x0001,  # denormal just above tie -> smallest bf16 denormal
        0x00018000: 0x0002,  # denormal tie, odd -> up
        0x007FFFFF: 0x0080,  # largest fp32 denormal -> smallest bf16 normal
    }
    for bits, want in cases.items():
        assert oracle.lib().oracle_f32_bits_to_bf16(bits) == want, hex(bits)
    # a signalling NaN becomes a quiet NaN of the same sign
    got = oracle.lib().oracle_f32_bits_to_bf16(0xFF800001)
    assert (got & 0x7FFF) > 0x7F80 and (got & 0x8000) and (got & 0x0040)


def test_narrowing_matches_torch_on_2_pow_27_patterns(oracle):
    # every 32nd pattern plus offsets that land on ties and their neighbours
    base = np.arange(0, 1 << 32, 1 << 10, dtype=np.uint64)  # 2^22 upper parts
    for low in (0, 1, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x1234, 0x3FF):
        for shift in (0, 0x10000):
            bits = ((base + shift + low) & 0xFFFFFFFF).astype(np.uint32)
            got = oracle.f32_to_bf16(bits.view(np.float32))
            want = _torch_narrow(bits)
            nan = (bits & 0x7FFFFFFF) > 0x7F800000
            assert np.array_equal(got[~nan], want[~nan])
            assert np.all(_is_nan_bf16(got[nan]))
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 1 << 32, size=1 << 24, dtype=np.uint64).astype(np.uint32)
    got = oracle.f32_to_bf16(bits.view(np.float32))
    want = _torch_narrow(bits)
    nan = (bits & 0x7FFFFFFF) > 0x7F800000
    assert np.array_equal(got[~nan], want[~nan])


def test_scale_is_one_fp32_division(oracle):
    assert oracle.scale(1) == np.float32(1.0)
    for N in (2, 4, 8, 16, 32, 64):
        assert oracle.scale(N) == np.float32(1.0 / N)  # exact powers of two
    for N in range(1, 65):
        assert oracle.scale(N) == np.float32(1.0) / np.float32(N)
    assert oracle.scale(7).view(np.uint32) == 0x3E124925  # fl32(1/7), by hand: 0.142857149...
