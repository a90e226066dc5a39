"""Pins for the oracle's zero-gradient participants (paper section 4.3: a replica that is catching
up takes part in the gradient exchange and sends a zero gradient)."""
import numpy as np
import pytest

F32, BF16 = 0, 1


def _rand(oracle, rng, n, count, dtype):
    bufs = [np.ascontiguousarray(rng.normal(0, 1e-3, count).astype(np.float32)) for _ in range(n)]
    if dtype == BF16:
        bufs = [oracle.f32_to_bf16(b) for b in bufs]
    return bufs


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_equals_real_zero_buffers_for_every_mask_pair(oracle, dtype):
    # the definition: a zero participant behaves exactly like a live replica whose buffer is +0.0
    rng = np.random.default_rng(20)
    n, count = 5, 64
    bufs = _rand(oracle, rng, n, count, dtype)
    bufs[1][:4] = 0 if dtype == BF16 else np.float32(-0.0)     # -0 + +0 = +0 must come out the same
    if dtype == BF16:
        bufs[1][:4] = 0x8000
    zero = np.zeros(count, dtype=bufs[0].dtype)
    nan = np.full(count, 0x7FC0 if dtype == BF16 else np.float32(np.nan), dtype=bufs[0].dtype)
    for live in range(1, 1 << n):
        for zmask in range(0, 1 << n):
            if zmask & ~live:
                continue
            with_zeros = [zero if (zmask >> r) & 1 else b for r, b in enumerate(bufs)]
            want = oracle.reduce_masked(with_zeros, live, dtype)
            poisoned = [nan if (zmask >> r) & 1 else b for r, b in enumerate(bufs)]   # never read
            got = oracle.reduce_masked_zero(poisoned, live, zmask, dtype)
            assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), (live, zmask)
            ring = oracle.ring_closed_form_zero(poisoned, live, zmask, count, 4, dtype)
            ring_want = oracle.ring_closed_form(with_zeros, live, count, 4, dtype)
            assert np.array_equal(ring.view(np.uint8), ring_want.view(np.uint8)), (live, zmask)


def test_divisor_policies(oracle):
    rng = np.random.default_rng(21)
    bufs = _rand(oracle, rng, 4, 100, F32)
    live, zmask = 0b1111, 0b0100
    participants = oracle.reduce_masked_zero(bufs, live, zmask, F32)
    contributors = oracle.reduce_masked_zero(bufs, live, zmask, F32, contributors_only=True)
    # sum over the three contributors, in index order, by hand
    s = (bufs[0] + bufs[1]) + np.float32(0.0)
    s = s + bufs[3]
    assert np.array_equal(participants, s * (np.float32(1.0) / np.float32(4.0)))
    assert np.array_equal(contributors, s * (np.float32(1.0) / np.float32(3.0)))
    # contributors-only equals the plain reduce over the contributors wherever no -0 is involved
    plain = oracle.reduce_masked(bufs, live & ~zmask, F32)
    assert np.array_equal(contributors, plain)
    with pytest.raises(oracle.OracleError):
        oracle.reduce_masked_zero(bufs, 0b0011, 0b0100, F32)           # zero replica not live
    with pytest.raises(oracle.OracleError):
        oracle.reduce_masked_zero(bufs, 0b0110, 0b0110, F32, contributors_only=True)   # nobody contributes
    allzero = oracle.reduce_masked_zero(bufs, 0b0110, 0b0110, F32)
    assert np.array_equal(allzero.view(np.uint32), np.zeros(100, dtype=np.uint32))
