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


def test_ring_divisor_contributors_only_by_hand(oracle):
    # Four replicas, replica 2 catching up (section 4.3), 16 elements in chunks of 4: portion k is
    # elements [4k, 4k+4) and absorbs ring positions k, k+1, k+2, k+3 (mod 4) in that order (section
    # 4.2, "Ring algorithm").  The divisor counts the three contributors.  Every sum is written out.
    f = np.float32
    x = [np.array([1e8, 1.0, -1e8, 3.0, 0.1, 0.2, 0.3, 0.4, 5.0, -7.0, 1e-3, 2e-3, 9.0, 0.7, -0.7, 1e-8], dtype=f),
         np.array([1.0, -1e8, 2.0, 1e8, 1.5, 2.5, 3.5, 4.5, 1e7, 1.0, -1e7, 0.5, 0.25, 1e-3, 3.0, 1.0], dtype=f),
         np.full(16, np.nan, dtype=f),                                  # zero participant: never read
         np.array([-1e8, 1e8, 1.0, 1.0, 7.0, 8.0, 9.0, 10.0, 1.0, 1e7, 1.0, -1e7, 1e-3, 0.125, 2.0, -1.0], dtype=f)]
    z = f(0.0)
    third = f(1.0) / f(3.0)
    quarter = f(1.0) / f(4.0)
    want3 = np.empty(16, dtype=f)
    want4 = np.empty(16, dtype=f)
    order = {0: (0, 1, 2, 3), 1: (1, 2, 3, 0), 2: (2, 3, 0, 1), 3: (3, 0, 1, 2)}
    for k in range(4):
        for i in range(4 * k, 4 * k + 4):
            a = None
            for r in order[k]:
                v = z if r == 2 else x[r][i]
                a = v if a is None else f(a + v)
            want3[i] = f(a * third)
            want4[i] = f(a * quarter)
    got3 = oracle.ring_closed_form_zero(x, 0b1111, 0b0100, 16, 4, F32, contributors_only=True)
    got4 = oracle.ring_closed_form_zero(x, 0b1111, 0b0100, 16, 4, F32)
    assert np.array_equal(got3.view(np.uint32), want3.view(np.uint32))
    assert np.array_equal(got4.view(np.uint32), want4.view(np.uint32))
    # the two policies really differ here (a test that cannot tell them apart pins nothing)
    assert not np.array_equal(got3, got4)
    # the rotated order is observable: portion 0 sums (1e8 + 1) + 0 - 1e8, portion 1 starts elsewhere
    assert got3[0] == f(f(f(f(1e8) + f(1.0)) + z) + f(-1e8)) * third


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_ring_divisor_contributors_only_every_mask_pair(oracle, dtype):
    # For every (live, zero) pair of five replicas: the ring's fp32 sum over real +0.0 buffers (the
    # pinned closed form in its sum mode, on the widened values), times fl(1/(N - Z)), rounded once.
    rng = np.random.default_rng(22)
    n, count, chunk = 5, 60, 4
    bufs = _rand(oracle, rng, n, count, dtype)
    wide = [oracle.bf16_to_f32(b) if dtype == BF16 else b for b in bufs]
    zero32 = np.zeros(count, dtype=np.float32)
    nan = np.full(count, 0x7FC0 if dtype == BF16 else np.float32(np.nan), dtype=bufs[0].dtype)
    seen_diff = 0
    for live in range(1, 1 << n):
        N = bin(live).count("1")
        for zmask in range(0, 1 << n):
            if zmask & ~live:
                continue
            Z = bin(zmask).count("1")
            poisoned = [nan if (zmask >> r) & 1 else b for r, b in enumerate(bufs)]
            if N - Z == 0:
                with pytest.raises(oracle.OracleError):
                    oracle.ring_closed_form_zero(poisoned, live, zmask, count, chunk, dtype, contributors_only=True)
                continue
            got = oracle.ring_closed_form_zero(poisoned, live, zmask, count, chunk, dtype, contributors_only=True)
            with_zeros = [zero32 if (zmask >> r) & 1 else b for r, b in enumerate(wide)]
            s = oracle.ring_closed_form(with_zeros, live, count, chunk, F32, sum_only=True)
            want = s if N == 1 else s * (np.float32(1.0) / np.float32(N - Z))
            if dtype == BF16:
                want = oracle.f32_to_bf16(np.ascontiguousarray(want))
            assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), (live, zmask)
            if Z and N > 1:
                other = oracle.ring_closed_form_zero(poisoned, live, zmask, count, chunk, dtype)
                seen_diff += int(not np.array_equal(other.view(np.uint8), got.view(np.uint8)))
    assert seen_diff > 50
