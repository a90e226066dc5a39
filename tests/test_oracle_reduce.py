"""Pins for the oracle's one-shot masked reduction.

What is pinned: the sum over the live replicas (paper section 4.1: the replicas'
same-rank GPUs compute the sum of their gradients) with this build's readings:
mean by one multiplication with fl32(1/N), fp32 accumulation in ascending
replica order starting from the first live value, one final rounding.
"""
import itertools

import numpy as np
import pytest

F32, BF16 = 0, 1


def _rand_f32(rng, n, count, sigma=1e-3):
    return [np.ascontiguousarray(rng.normal(0, sigma, count).astype(np.float32)) for _ in range(n)]


def _as_bf16(oracle, bufs):
    return [oracle.f32_to_bf16(b) for b in bufs]


def _brute_force(bufs_f32, mask, scale32):
    """Separately written reference: python loop over numpy.float32 scalars, index order."""
    live = [r for r in range(len(bufs_f32)) if (mask >> r) & 1]
    out = np.empty(bufs_f32[0].size, dtype=np.float32)
    with np.errstate(all="ignore"):
        for i in range(out.size):
            a = np.float32(bufs_f32[live[0]][i])
            for r in live[1:]:
                a = np.float32(a + np.float32(bufs_f32[r][i]))
            out[i] = np.float32(a * scale32)
    return out


def _same_bits_or_both_nan(a, b):
    a = np.asarray(a)
    b = np.asarray(b)
    if a.dtype == np.float32:
        nan = np.isnan(a) & np.isnan(b)
        return np.array_equal(a.view(np.uint32)[~nan], b.view(np.uint32)[~nan]) and \
            np.array_equal(np.isnan(a), np.isnan(b))
    na = (a & 0x7FFF) > 0x7F80
    nb = (b & 0x7FFF) > 0x7F80
    return np.array_equal(na, nb) and np.array_equal(a[~na], b[~na])


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_single_live_replica_is_identity(oracle, dtype):
    rng = np.random.default_rng(0)
    bufs = _rand_f32(rng, 5, 1000)
    bufs[2][:6] = np.array([0.0, -0.0, 1e-45, -1e-40, np.inf, 3.0e38], dtype=np.float32)
    if dtype == BF16:
        bufs = _as_bf16(oracle, bufs)
    for r in range(5):
        out = oracle.reduce_masked(bufs, 1 << r, dtype)
        assert np.array_equal(out.view(np.uint8), bufs[r].view(np.uint8))


def test_identical_inputs_mean_equals_input(oracle):
    rng = np.random.default_rng(1)
    x = rng.normal(0, 1e-3, 4096).astype(np.float32)
    xb = oracle.f32_to_bf16(x)                 # bf16 values
    xf = oracle.bf16_to_f32(xb)                # the same values held in fp32
    for n in range(1, 17):
        mask = (1 << n) - 1
        # k*x for k <= 16 is exact in fp32 when x has 8 significant bits, and the final
        # rounding to bf16 absorbs the two roundings of scale and product
        out = oracle.reduce_masked([xb.copy() for _ in range(n)], mask, BF16)
        assert np.array_equal(out, xb), n
    for n in (1, 2, 4, 8, 16):                 # power-of-two N: exact also with fp32 output
        out = oracle.reduce_masked([xf.copy() for _ in range(n)], (1 << n) - 1, F32)
        assert np.array_equal(out.view(np.uint32), xf.view(np.uint32)), n
    for n in (3, 5, 6, 7, 11, 13):             # general N with fp32 output: within 2 roundings
        out = oracle.reduce_masked([xf.copy() for _ in range(n)], (1 << n) - 1, F32)
        assert np.all(np.abs(out.astype(np.float64) - xf) <= 2.0 ** -23 * np.abs(xf)), n
    # N = 2 is exact for arbitrary fp32 (x + x and the halving are exact)
    out = oracle.reduce_masked([x.copy(), x.copy()], 0b11, F32)
    assert np.array_equal(out.view(np.uint32), x.view(np.uint32))


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_dropping_replica_equals_reduction_over_the_rest(oracle, dtype):
    rng = np.random.default_rng(2)
    n, count = 8, 3001
    bufs = _rand_f32(rng, n, count)
    if dtype == BF16:
        bufs = _as_bf16(oracle, bufs)
    for k in range(n):
        mask = ((1 << n) - 1) & ~(1 << k)
        poisoned = [b.copy() for b in bufs]
        poisoned[k][:] = np.float32(np.nan) if dtype == F32 else 0x7FC0
        got = oracle.reduce_masked(poisoned, mask, dtype)
        rest = [b for r, b in enumerate(bufs) if r != k]
        want = oracle.reduce_masked(rest, (1 << (n - 1)) - 1, dtype)
        assert np.array_equal(got.view(np.uint8), want.view(np.uint8))
        # a dead replica may have no buffer at all
        got2 = oracle.reduce_masked([None if r == k else b for r, b in enumerate(bufs)], mask, dtype)
        assert np.array_equal(got2.view(np.uint8), want.view(np.uint8))


def test_linearity(oracle):
    rng = np.random.default_rng(3)
    n, count = 7, 5000
    x = _rand_f32(rng, n, count)
    y = _rand_f32(rng, n, count)
    mask = 0b1011101
    base = oracle.reduce_masked(x, mask, F32)
    for e in (-20, -3, 1, 10, 40):
        s = np.float32(2.0 ** e)
        got = oracle.reduce_masked([b * s for b in x], mask, F32)
        assert np.array_equal(got.view(np.uint32), (base * s).view(np.uint32)), e
    # additive linearity holds within the summation error bound
    rx = oracle.reduce_masked(x, mask, F32).astype(np.float64)
    ry = oracle.reduce_masked(y, mask, F32).astype(np.float64)
    rxy = oracle.reduce_masked([a + b for a, b in zip(x, y)], mask, F32).astype(np.float64)
    mag = sum(np.abs(a.astype(np.float64)) + np.abs(b.astype(np.float64))
              for r, (a, b) in enumerate(zip(x, y)) if (mask >> r) & 1) / 5
    assert np.all(np.abs(rxy - (rx + ry)) <= 4e-6 * mag)


SPECIALS = np.array([0.0, -0.0, 1e-45, -1e-45, 1.1754942e-38, 1.0, 1.0 + 2 ** -23, 2 ** -24,
                     -2 ** -24, 3.0e38, -3.0e38, 1e30, -1e30, 1e-30, np.inf, np.nan],
                    dtype=np.float32)


def test_brute_force_on_16_element_inputs_every_mask(oracle):
    rng = np.random.default_rng(4)
    for n in range(1, 7):
        bufs = [SPECIALS[rng.permutation(16)].copy() for _ in range(n)]
        # a second family: neighbours 2^-24 apart and large/small cancellation
        bufs2 = [np.float32(1.0) + rng.integers(-8, 8, 16).astype(np.float32) * np.float32(2 ** -24)
                 for _ in range(n)]
        for k in range(n):
            bufs2[k][::3] *= np.float32(-1e8 if k % 2 else 1e8)
        for fam in (bufs, bufs2):
            for mask in range(1, 1 << n):
                N = bin(mask).count("1")
                want = _brute_force(fam, mask, np.float32(1.0) / np.float32(N))
                got = oracle.reduce_masked(fam, mask, F32)
                assert _same_bits_or_both_nan(got, want), (n, mask)
                # bf16 storage: same inputs rounded to bf16 first, output rounded once
                hb = _as_bf16(oracle, fam)
                wf = _brute_force([oracle.bf16_to_f32(h) for h in hb], mask,
                                  np.float32(1.0) / np.float32(N))
                gotb = oracle.reduce_masked(hb, mask, BF16)
                assert _same_bits_or_both_nan(gotb, oracle.f32_to_bf16(wf)), (n, mask)
                # the paper's literal sum (no averaging)
                ws = _brute_force(fam, mask, np.float32(1.0))
                gs = oracle.reduce_masked(fam, mask, F32, sum_only=True)
                assert _same_bits_or_both_nan(gs, ws), (n, mask)


def test_order_is_ascending_and_starts_from_first_value(oracle):
    # (1e8 + 1) - 1e8 = 0 in fp32 but (1e8 - 1e8) + 1 = 1: the order is observable
    a = np.array([1e8], dtype=np.float32)
    b = np.array([1.0], dtype=np.float32)
    c = np.array([-1e8], dtype=np.float32)
    assert oracle.reduce_masked([a, b, c], 0b111, F32, sum_only=True)[0] == 0.0
    assert oracle.reduce_masked([a, c, b], 0b111, F32, sum_only=True)[0] == 1.0
    assert oracle.reduce_masked([b, a, c], 0b111, F32, sum_only=True)[0] == 0.0
    # starting from the first value (not from +0) keeps a lone -0
    z = np.array([-0.0], dtype=np.float32)
    out = oracle.reduce_masked([z], 1, F32)
    assert out.view(np.uint32)[0] == 0x80000000
    out = oracle.reduce_masked([z, z.copy()], 3, F32)
    assert out.view(np.uint32)[0] == 0x80000000


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_within_bound_of_fp64_and_of_numpy(oracle, dtype):
    rng = np.random.default_rng(5)
    for n, mask in ((4, 0b1111), (8, 0b11110111), (16, 0xFFFF), (16, 0xFDFF)):
        bufs = _rand_f32(rng, n, 20000)
        if dtype == BF16:
            bufs = _as_bf16(oracle, bufs)
        N = bin(mask).count("1")
        got = oracle.reduce_masked(bufs, mask, dtype)
        ref, mag = oracle.reduce_f64(bufs, mask, dtype)
        # independent textbook value: numpy's own fp64 sum over the live replicas
        vals = [oracle.bf16_to_f32(b) if dtype == BF16 else b for b in bufs]
        npref = np.sum(np.stack([vals[r].astype(np.float64) for r in range(n) if (mask >> r) & 1]),
                       axis=0) / N
        assert np.allclose(ref, npref, rtol=1e-14, atol=0)
        if dtype == F32:
            assert np.all(np.abs(got.astype(np.float64) - npref) <= 1e-6 * mag)
        else:
            # one bf16 ulp of the exact mean
            g = oracle.bf16_to_f32(got).astype(np.float64)
            ulp = np.maximum(np.abs(npref), 2.0 ** -126) * 2.0 ** -7
            assert np.all(np.abs(g - npref) <= ulp)


def test_zero_gradient_participant_does_not_change_the_sum(oracle):
    # a replica that is catching up contributes an all-zero gradient (paper section 4.3):
    # the fp32 sum is bit-identical to the sum with that replica masked out
    rng = np.random.default_rng(6)
    n, count = 6, 4000
    bufs = _rand_f32(rng, n, count)
    for k in range(n):
        with_zero = [b.copy() for b in bufs]
        with_zero[k][:] = 0.0
        a = oracle.reduce_masked(with_zero, (1 << n) - 1, F32, sum_only=True)
        b = oracle.reduce_masked(bufs, ((1 << n) - 1) & ~(1 << k), F32, sum_only=True)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_bad_masks_are_rejected(oracle):
    x = [np.zeros(4, dtype=np.float32) for _ in range(3)]
    with pytest.raises(oracle.OracleError):
        oracle.reduce_masked(x, 0, F32)
    with pytest.raises(oracle.OracleError):
        oracle.reduce_masked(x, 0b1000, F32)
