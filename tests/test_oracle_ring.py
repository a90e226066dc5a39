"""Pins for the oracle's ring all-reduce (paper section 4.2, "Ring algorithm"
and the store rule under "Optimizations") and for its portion geometry."""
import json
import os

import numpy as np
import pytest

F32, BF16 = 0, 1
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(oracle, rng, n, count, dtype, mask=None):
    bufs = [np.ascontiguousarray(rng.standard_t(3, count).astype(np.float32) * np.float32(1e-4))
            for _ in range(n)]
    if dtype == BF16:
        bufs = [oracle.f32_to_bf16(b) for b in bufs]
    return bufs


def _poison(bufs, mask, dtype):
    out = []
    for r, b in enumerate(bufs):
        b = b.copy()
        if not (mask >> r) & 1:
            b[:] = np.float32(np.nan) if dtype == F32 else 0x7FC1
        out.append(b)
    return out


def test_hand_worked_four_replica_example(oracle):
    g = json.load(open(os.path.join(GOLDEN, "ring_n4_worked.json")))
    n, mask, chunk = g["n_replicas"], g["live_mask"], g["chunk_elems"]
    inputs = [np.array(v, dtype=np.float32) for v in g["inputs"]]
    # schedule: which portion each position receives at each step
    rs, ag = oracle.ring_schedule(n, mask)
    assert rs.tolist() == g["rs_received_portion"]
    assert ag.tolist() == g["ag_received_portion"]
    # in-flight partial sums after the non-final ReduceScatter steps; user buffers untouched
    for s, want in g["in_flight_after_rs_step"].items():
        bufs = [b.copy() for b in inputs]
        acc = oracle.ring_per_rank(bufs, mask, chunk, F32, rs_steps=int(s) + 1, ag_steps=0)
        assert acc.tolist() == want
        assert all(np.array_equal(a, b) for a, b in zip(bufs, inputs))
        assert oracle.ring_partial(inputs, mask, 4, chunk, F32, int(s) + 1).tolist() == want
    bufs = [b.copy() for b in inputs]
    oracle.ring_per_rank(bufs, mask, chunk, F32, rs_steps=3, ag_steps=0)
    assert [b.tolist() for b in bufs] == g["buffers_after_rs"]
    for t, want in g["buffers_after_ag_step"].items():
        bufs = [b.copy() for b in inputs]
        oracle.ring_per_rank(bufs, mask, chunk, F32, rs_steps=3, ag_steps=int(t) + 1)
        assert [b.tolist() for b in bufs] == want
    assert oracle.ring_closed_form(inputs, mask, 4, chunk, F32).tolist() == g["mean"]
    # portion k is finished by ring position k-1
    owners = [int(np.argmax([b[k] != i[k] for b, i in zip(
        [np.array(v, dtype=np.float32) for v in g["buffers_after_rs"]], inputs)])) for k in range(4)]
    assert owners == g["owner_replica_of_portion_after_rs"]


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_message_passing_ring_equals_closed_form_every_mask(oracle, dtype):
    rng = np.random.default_rng(10)
    for n in range(1, 7):
        for mask in range(1, 1 << n):
            N = bin(mask).count("1")
            for count, chunk in ((16 * N, 16), (16 * N + 5, 16), (37, 4), (3, 1), (50, 64)):
                orig = _poison(_rand(oracle, rng, n, count, dtype), mask, dtype)
                bufs = [b.copy() for b in orig]
                oracle.ring_per_rank(bufs, mask, chunk, dtype)
                want = oracle.ring_closed_form(orig, mask, count, chunk, dtype)
                for r in range(n):
                    if (mask >> r) & 1:
                        # all-reduce postcondition: every live replica holds the same bits
                        assert np.array_equal(bufs[r], want), (n, mask, count, chunk, r)
                    else:
                        # a dead replica is never written (and was never read: no NaN leaked)
                        assert np.array_equal(bufs[r].view(np.uint8), orig[r].view(np.uint8))
                assert not np.any(np.isnan(oracle.bf16_to_f32(want) if dtype == BF16 else want))


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_portion_zero_matches_one_shot_and_rest_within_bound(oracle, dtype):
    rng = np.random.default_rng(11)
    n, mask, count, chunk = 16, 0xFDFF, 15 * 64 * 7 + 13, 64
    orig = _poison(_rand(oracle, rng, n, count, dtype), mask, dtype)
    ring = oracle.ring_closed_form(orig, mask, count, chunk, dtype)
    shot = oracle.reduce_masked(orig, mask, dtype)
    sb = oracle.geometry(n, mask, count, chunk)
    assert np.array_equal(ring[:sb[1]], shot[:sb[1]])       # same order in portion 0
    ref, mag = oracle.reduce_f64(orig, mask, dtype)
    if dtype == F32:
        assert np.all(np.abs(ring.astype(np.float64) - ref) <= 1e-6 * mag)
        assert np.any(ring != shot)                          # other portions are reordered
    else:
        r = oracle.bf16_to_f32(ring).astype(np.float64)
        assert np.all(np.abs(r - ref) <= np.abs(ref) * 2.0 ** -7 + 1e-45)


def test_rotated_order_is_observable(oracle):
    # portion k sums ring[k], ring[k+1], ... with wrap-around
    a, b, c = np.float32(1e8), np.float32(1.0), np.float32(-1e8)
    bufs = [np.full(3, v, dtype=np.float32) for v in (a, b, c)]
    out = oracle.ring_closed_form(bufs, 0b111, 3, 1, F32, sum_only=True)
    # portion 0: (a+b)+c = 0 ; portion 1: (b+c)+a = 0 ; portion 2: (c+a)+b = 1
    assert out.tolist() == [0.0, 0.0, 1.0]
    live = [x.copy() for x in bufs]
    oracle.ring_per_rank(live, 0b111, 1, F32, sum_only=True)
    assert all(x.tolist() == [0.0, 0.0, 1.0] for x in live)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_store_rule_user_buffers_untouched_before_last_rs_step(oracle, dtype):
    rng = np.random.default_rng(12)
    n, mask, count, chunk = 7, 0b1101111, 600, 8
    N = 6
    orig = _poison(_rand(oracle, rng, n, count, dtype), mask, dtype)
    for s in range(0, N - 1):
        bufs = [b.copy() for b in orig]
        acc = oracle.ring_per_rank(bufs, mask, chunk, dtype, rs_steps=s, ag_steps=0)
        assert all(np.array_equal(a.view(np.uint8), b.view(np.uint8)) for a, b in zip(bufs, orig)), s
        if 1 <= s <= N - 2:
            want = oracle.ring_partial(orig, mask, count, chunk, dtype, s)
            assert np.array_equal(acc.view(np.uint32), want.view(np.uint32)), s


def test_degenerate_rings(oracle):
    rng = np.random.default_rng(13)
    x = _rand(oracle, rng, 3, 40, F32)
    # one live replica: nothing is exchanged, nothing changes
    bufs = [b.copy() for b in x]
    oracle.ring_per_rank(bufs, 0b010, 8, F32)
    assert all(np.array_equal(a, b) for a, b in zip(bufs, x))
    assert np.array_equal(oracle.ring_closed_form(x, 0b010, 40, 8, F32), x[1])
    # two live replicas: one step that is first and last; mean of two is order-free
    bufs = [b.copy() for b in x]
    oracle.ring_per_rank(bufs, 0b101, 8, F32)
    want = ((x[0] + x[2]) * np.float32(0.5)).astype(np.float32)
    assert np.array_equal(bufs[0], want) and np.array_equal(bufs[2], want)
    assert np.array_equal(bufs[1], x[1])


def test_replan_after_aborted_steps_equals_fresh_run(oracle):
    # a replica leaves before a non-final ReduceScatter step: user buffers are intact, so
    # restarting over the smaller group gives exactly the fresh result (sections 4.1, 4.2)
    rng = np.random.default_rng(14)
    n, count, chunk = 16, 16 * 15 * 4 + 3, 4
    orig = _rand(oracle, rng, n, count, BF16)
    bufs = [b.copy() for b in orig]
    oracle.ring_per_rank(bufs, 0xFFFF, chunk, BF16, rs_steps=5, ag_steps=0)
    new_mask = 0xFFFF & ~(1 << 9)
    oracle.ring_per_rank(bufs, new_mask, chunk, BF16)
    fresh = oracle.ring_closed_form(orig, new_mask, count, chunk, BF16)
    for r in range(n):
        if r == 9:
            assert np.array_equal(bufs[r], orig[r])
        else:
            assert np.array_equal(bufs[r], fresh)


def test_zero_gradient_participant_in_the_ring(oracle):
    rng = np.random.default_rng(15)
    n, count, chunk = 5, 100, 4
    x = _rand(oracle, rng, n, count, F32)
    x[2][:] = 0.0
    with_zero = oracle.ring_closed_form(x, 0b11111, count, chunk, F32, sum_only=True)
    ref, mag = oracle.reduce_f64(x, 0b11011, F32, sum_only=True)
    assert np.all(np.abs(with_zero.astype(np.float64) - ref) <= 1e-6 * mag)


def test_geometry_invariants(oracle):
    for n, mask, count, chunk in ((16, 0xFFFF, 1 << 28, 16384), (16, 0xFDFF, 1 << 28, 16384),
                                  (8, 0xF7, 1000, 16), (5, 0b10101, 17, 4), (6, 0b111111, 3, 1),
                                  (4, 0xF, 100, 1000), (64, (1 << 64) - 1, 12345, 7)):
        sb = oracle.geometry(n, mask, count, chunk)
        N = bin(mask).count("1")
        assert len(sb) == N + 1 and sb[0] == 0 and sb[-1] == count
        lens = [sb[k + 1] - sb[k] for k in range(N)]
        assert all(l >= 0 for l in lens) and sum(lens) == count
        assert all(b % chunk == 0 for b in sb[:-1] if b != count)
        assert max(lens) - min(lens) <= chunk
    assert oracle.geometry(16, 0xFFFF, 1 << 28, 16384) == [k << 24 for k in range(17)]
    sb = oracle.geometry(16, 0xFDFF, 1 << 28, 16384)
    assert sorted(set((sb[k + 1] - sb[k]) // 16384 for k in range(15))) == [1092, 1093]
    assert oracle.live_ring(8, 0b11110111) == [0, 1, 2, 4, 5, 6, 7]
