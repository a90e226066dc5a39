"""GPU: the persistent ring gated by rows of chunks (FTAR_PERSIST_CHUNKS): paper section 4.2, every
step of a partition is pipelined over the chunks of a portion.  The CPU releases row by row, in and out
of phase with the steps; results are the oracle's, bit for bit, whatever the release pattern."""
import time

import numpy as np
import pytest
import torch

from gpu_util import assert_same, code, host, rand_bufs, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2602_00277_amd import binding
    binding.lib()
    return binding


def _units(oracle, n, mask, count, chunk, part):
    """Gate units by the definition: per partition, (2N-2) steps x the largest number of chunks of a portion."""
    N = bin(mask).count("1")
    total = 0
    P = part if part else count
    for p0 in range(0, count, P):
        L = min(P, count - p0)
        sb = oracle.geometry(n, mask, L, chunk)
        rows = max(-(-(sb[k + 1] - sb[k]) // chunk) for k in range(N))
        total += (2 * N - 2) * rows
    return total


def _reference(oracle, orig, n, mask, count, chunk, part, d):
    want = np.empty_like([o for o in orig if o is not None][0])
    P = part if part else count
    for lo in range(0, count, P):
        hi = min(count, lo + P)
        sl = [None if o is None else o[lo:hi].copy() for o in orig]
        want[lo:hi] = oracle.ring_closed_form(sl, mask, hi - lo, chunk, d)
    return want


CASES = [
    # n, mask, chunk, count, partition, n_blocks
    (8, 0xFF, 8192, 8 * 8192 * 6, 0, 0),                    # every portion six whole chunks, tile == chunk (bf16)
    (8, 0b11110111, 4096, 7 * 4096 * 5 + 4096 * 3 + 100, 0, 0),  # portions of 5 and 6 chunks, a short last chunk
    (16, 0xFFFF, 2048, 16 * 2048 * 3 + 2048 * 5 + 8, 0, 7),  # small chunks (tiles clipped), few workers
    (5, 0b11111, 1000, 5 * 1000 * 4 + 333, 0, 0),            # chunk not a multiple of 8: the element-wise kernel
    (6, 0b111111, 8192, 6 * 8192 * 10 + 8192 * 2, 6 * 8192 * 4, 0),  # partitions, the last one shorter
    (2, 0b11, 4096, 2 * 4096 * 4 + 64, 0, 0),                # a ring of two: one ReduceScatter and one AllGather step
    (4, 0xF, 65536, 4 * 65536 * 2, 0, 3),                    # few workers and chunks that hold the big tile
    (12, 0xFFF, 4096, 4096 * 5, 0, 0),                       # fewer chunks than portions: empty portions
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_all_rows_released_at_once(B, oracle, dtype, case):
    n, mask, chunk, count, part, nb = CASES[case]
    say("chunk rows, all released", dtype, CASES[case])
    bufs = rand_bufs(n, count, dtype, seed=90 + case, dist="student_t3", mask=mask)
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    if part:
        plan.set_partition(part)
    units = plan.n_gate_units(B.FTAR_PERSIST_CHUNKS)
    assert units == _units(oracle, n, mask, count, chunk, part)
    assert plan.n_gate_units(0) == plan.n_slots
    acc = torch.empty(plan.acc_bytes // 4, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    for flags in (B.FTAR_PERSIST_CHUNKS, B.FTAR_PERSIST_CHUNKS | B.FTAR_PERSIST_PUBLISH | B.FTAR_PERSIST_ALIGN):
        work = [b.clone() for b in bufs]
        B.ftar_ring_persistent(plan, work, acc, ctrl, n_blocks=nb, timeout_us=5_000_000, flags=flags)
        ctrl.release(units)
        torch.cuda.synchronize()
        assert ctrl.result() == (B.FTAR_OK, units)
        want = _reference(oracle, orig, n, mask, count, chunk, part, code(dtype))
        for r in range(n):
            assert_same(host(work[r]), want if (mask >> r) & 1 else orig[r], "buf %d flags %d" % (r, flags))
    ctrl.destroy()


@pytest.mark.parametrize("case", [0, 1, 2, 4, 5, 7])
def test_cpu_releases_row_by_row_out_of_phase_with_the_steps(B, oracle, case):
    n, mask, chunk, count, part, nb = CASES[case]
    dtype = torch.bfloat16
    say("chunk rows, released in strides", CASES[case])
    bufs = rand_bufs(n, count, dtype, seed=110 + case, dist="student_t3", mask=mask)
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    if part:
        plan.set_partition(part)
    units = plan.n_gate_units(B.FTAR_PERSIST_CHUNKS)
    acc = torch.empty(plan.acc_bytes // 4, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=nb, timeout_us=5_000_000,
                           flags=B.FTAR_PERSIST_CHUNKS | B.FTAR_PERSIST_PUBLISH)
    released, stride = 0, 1
    while released < units:
        assert ctrl.progress() <= released                 # nobody runs ahead of the gate
        released = min(units, released + stride)
        stride = stride % 5 + 1                            # 1, 2, 3, 4, 5 rows at a time: not aligned with steps
        ctrl.release(released)
        t0 = time.time()
        while ctrl.progress() < released:                  # exact whenever the kernel waits
            assert time.time() - t0 < 10.0, "row %d not reported" % released
            time.sleep(0.0002)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, units)
    want = _reference(oracle, orig, n, mask, count, chunk, part, code(dtype))
    for r in range(n):
        assert_same(host(bufs[r]), want if (mask >> r) & 1 else orig[r], "buf %d" % r)
    ctrl.destroy()


def test_cancel_inside_a_step_leaves_the_inputs_intact(B, oracle):
    # rows of ReduceScatter step 1 released half way, then the cancel: the call stops there, no buffer is
    # written, the partial sums are those of the rows that ran
    n, mask, chunk, dtype = 8, 0xFF, 8192, torch.bfloat16
    count = 8 * chunk * 6
    say("chunk rows, cancel inside a step")
    bufs = rand_bufs(n, count, dtype, seed=130, dist="student_t3")
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    units = plan.n_gate_units(B.FTAR_PERSIST_CHUNKS)
    assert units == 14 * 6
    acc = torch.zeros(count, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, timeout_us=5_000_000, flags=B.FTAR_PERSIST_CHUNKS)
    ctrl.release(6 + 3)                                   # step 0 and three of the six rows of step 1
    t0 = time.time()
    while ctrl.progress() < 9 and time.time() - t0 < 10:
        time.sleep(0.0005)
    ctrl.cancel()
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_ERR_STALE_PLAN, 9)
    for r in range(n):
        assert_same(host(bufs[r]), orig[r], "buf %d untouched" % r)
    got = host(acc)
    one = oracle.ring_partial(orig, mask, count, chunk, code(dtype), 1)
    two = oracle.ring_partial(orig, mask, count, chunk, code(dtype), 2)
    sb = oracle.geometry(n, mask, count, chunk)
    for k in range(8):                                    # rows 0..2 of every portion saw step 1, rows 3..5 only step 0
        lo = sb[k]
        assert_same(got[lo:lo + 3 * chunk], two[lo:lo + 3 * chunk], "portion %d, rows that ran step 1" % k)
        assert_same(got[lo + 3 * chunk:sb[k + 1]], one[lo + 3 * chunk:sb[k + 1]], "portion %d, rows that did not" % k)
    ctrl.destroy()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_rows_reported_with_publish_can_be_read_off_the_gpu_while_the_kernel_waits(B, oracle, dtype):
    # FTAR_PERSIST_PUBLISH: a reported row has left the GPU's caches.  The kernel is held at the gate after the
    # ReduceScatter phase; a copy engine on another stream then reads the owners' portions from memory (it does
    # not look into any L2) and finds the phase's results; afterwards the AllGather phase is released.
    n, mask, chunk = 8, 0xFF, 8192
    rows = 12                                             # chunks per portion
    count = n * chunk * rows
    say("chunk rows with PUBLISH read by a copy while the kernel waits", dtype)
    bufs = rand_bufs(n, count, dtype, seed=140, dist="student_t3", mask=mask)
    orig = [host(b) for b in bufs]
    want_rs = [o.copy() for o in orig]
    oracle.ring_per_rank(want_rs, mask, chunk, code(dtype), rs_steps=n - 1, ag_steps=0)
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    flags = B.FTAR_PERSIST_CHUNKS | B.FTAR_PERSIST_PUBLISH
    units = plan.n_gate_units(flags)
    assert units == (2 * n - 2) * rows
    acc = torch.empty(plan.acc_bytes // 4, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    side = torch.cuda.Stream()
    pinned = [torch.empty(count, dtype=dtype).pin_memory() for _ in range(n)]
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, timeout_us=20_000_000, flags=flags)
    try:
        rs_units = (n - 1) * rows
        ctrl.release(rs_units)
        t0 = time.time()
        while ctrl.progress() < rs_units:
            assert time.time() - t0 < 10.0, "ReduceScatter phase not reported"
            time.sleep(0.0002)
        assert ctrl.progress() == rs_units                 # the kernel now waits for the AllGather phase
        with torch.cuda.stream(side):
            for r in range(n):
                pinned[r].copy_(bufs[r], non_blocking=True)
        side.synchronize()
        for k in range(plan.n_live):
            b, e, owner = plan.segment(k)
            got = host(pinned[owner])
            assert_same(got[b:e], want_rs[owner][b:e], "portion %d in its owner %d, read while the kernel waits" % (k, owner))
    finally:
        ctrl.release(units)
        torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, units)
    want = oracle.ring_closed_form(orig, mask, count, chunk, code(dtype))
    for r in range(n):
        assert_same(host(bufs[r]), want, "buf %d" % r)
    ctrl.destroy()
