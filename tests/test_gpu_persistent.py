"""GPU: the CPU-gated persistent ring kernel (ftar_ring_persistent): same bits as the per-step
kernels and the oracle; a wait that is never satisfied ends by timeout, a cancel ends the kernel
at the next wait; in both cases the kernel exits normally and the user buffers are intact."""
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


def _wait_progress(ctrl, at_least, limit_s=10.0):
    t0 = time.time()
    while ctrl.progress() < at_least:
        if time.time() - t0 > limit_s:
            return False
        time.sleep(0.0005)
    return True


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n,mask", [(2, 0b11), (3, 0b111), (8, 0b11110111), (16, 0xFFFF), (16, 0xFDFF)])
def test_all_steps_released_matches_oracle_and_step_kernels(B, oracle, dtype, n, mask):
    N = bin(mask).count("1")
    chunk = 1024
    count = N * chunk * 21 + 555
    say("persistent ring", dtype, n, hex(mask), count)
    bufs = rand_bufs(n, count, dtype, seed=n + 1, dist="student_t3", mask=mask)
    orig = [host(b) for b in bufs]
    ref = [b.clone() for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    B.ring_allreduce(plan, ref, acc)                      # per-step kernels
    ctrl = B.ftar_ctrl_create()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, timeout_us=5_000_000)
    ctrl.release(2 * N - 2)                               # the CPU lets every step go
    torch.cuda.synchronize()
    st, done = ctrl.result()
    assert st == B.FTAR_OK and done == 2 * N - 2
    want = oracle.ring_closed_form(orig, mask, count, chunk, code(dtype))
    for r in range(n):
        assert_same(host(bufs[r]), want if (mask >> r) & 1 else orig[r], "buf %d" % r)
        assert torch.equal(bufs[r].view(torch.uint8), ref[r].view(torch.uint8))
    ctrl.destroy()


@pytest.mark.parametrize("flags", [0, 1, 2, 3])
@pytest.mark.parametrize("n_blocks", [1, 2, 7, 64, 1024])
def test_any_cu_budget_gives_the_same_bits(B, oracle, n_blocks, flags):
    n, mask, chunk = 8, 0xFF, 512
    count = 8 * chunk * 13 + 77
    say("persistent ring blocks", n_blocks)
    bufs = rand_bufs(n, count, torch.bfloat16, seed=5, dist="student_t3")
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, torch.bfloat16)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=n_blocks, timeout_us=5_000_000, flags=flags)
    ctrl.release(14)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, 14)
    want = oracle.ring_closed_form(orig, mask, count, chunk, 1)
    for r in range(n):
        assert_same(host(bufs[r]), want, "buf %d" % r)


def test_cpu_gates_every_step(B, oracle):
    # the CPU plays the network: it releases step s+1 only after every workgroup reported step s
    n, mask, chunk = 6, 0b111111, 256
    count = 6 * chunk * 9 + 3
    say("persistent ring gated")
    bufs = rand_bufs(n, count, torch.float32, seed=8)
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, torch.float32)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, timeout_us=5_000_000, flags=B.FTAR_PERSIST_PUBLISH)
    for s in range(10):
        assert ctrl.progress() <= s
        ctrl.release(s + 1)
        assert _wait_progress(ctrl, s + 1), "step %d not reported" % s
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, 10)
    want = oracle.ring_closed_form(orig, mask, count, chunk, 0)
    for r in range(n):
        assert_same(host(bufs[r]), want, "buf %d" % r)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_unreleased_step_times_out_and_leaves_inputs_intact(B, oracle, dtype):
    # the CPU never releases ReduceScatter step 3: every workgroup's bounded wait ends by itself
    n, mask, chunk = 8, 0xFF, 512
    count = 8 * chunk * 5 + 9
    say("persistent ring timeout", dtype)
    bufs = rand_bufs(n, count, dtype, seed=9, dist="student_t3")
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, timeout_us=20_000)     # 20 ms
    ctrl.release(3)
    t0 = time.time()
    torch.cuda.synchronize()
    assert time.time() - t0 < 5.0
    st, done = ctrl.result()
    assert st == B.FTAR_ERR_STALE_PLAN and B.ftar_status_is_retryable(st) and done == 3
    for r in range(n):
        assert_same(host(bufs[r]), orig[r], "buf %d untouched" % r)
    assert_same(host(acc), oracle.ring_partial(orig, mask, count, chunk, code(dtype), 3), "in-flight partials")
    # retry: the CPU acknowledges the failure (until then anything it enqueues counts as queued behind
    # the call that timed out); then a fresh call on the same control block completes
    ctrl.cancel()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, timeout_us=5_000_000)
    ctrl.release(14)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, 14)
    want = oracle.ring_closed_form(orig, mask, count, chunk, code(dtype))
    for r in range(n):
        assert_same(host(bufs[r]), want, "buf %d after retry" % r)


def test_cancel_then_replan_over_the_survivors(B, oracle):
    # replica 9 of 16 leaves while the kernel waits for step 5: cancel, re-plan for 15, restart
    n, chunk = 16, 256
    count = 16 * 15 * chunk + 31
    say("persistent ring cancel + replan")
    bufs = rand_bufs(n, count, torch.bfloat16, seed=10, dist="student_t3")
    orig = [host(b) for b in bufs]
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    p16 = B.ftar_plan(n, 0xFFFF, count, chunk, torch.bfloat16)
    B.ftar_ring_persistent(p16, bufs, acc, ctrl, timeout_us=5_000_000)
    ctrl.release(5)
    assert _wait_progress(ctrl, 5)
    ctrl.cancel()
    torch.cuda.synchronize()
    st, done = ctrl.result()
    assert st == B.FTAR_ERR_STALE_PLAN and done == 5
    for r in range(n):
        assert_same(host(bufs[r]), orig[r], "buf %d untouched" % r)
    new_mask = 0xFFFF & ~(1 << 9)
    p15 = B.ftar_plan(n, new_mask, count, chunk, torch.bfloat16)
    B.ftar_ring_persistent(p15, bufs, acc, ctrl, timeout_us=5_000_000)
    ctrl.release(28)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, 28)
    fresh = oracle.ring_closed_form(orig, new_mask, count, chunk, 1)
    for r in range(n):
        assert_same(host(bufs[r]), orig[r] if r == 9 else fresh, "buf %d" % r)


def test_argument_errors_and_ring_of_one(B):
    plan = B.ftar_plan(4, 0b1111, 1000, 8, torch.float32)
    bufs = [torch.zeros(1000, device="cuda") for _ in range(4)]
    acc = torch.zeros(1000, device="cuda")
    ctrl = B.ftar_ctrl_create()
    say("persistent ring errors")
    with pytest.raises(B.FtarError) as e:
        B.ftar_ring_persistent(plan, bufs, acc, ctrl, timeout_us=0)
    assert e.value.status == B.FTAR_ERR_INVALID_ARG
    with pytest.raises(B.FtarError) as e:
        B.ftar_ring_persistent(plan, bufs, None, ctrl)
    assert e.value.status == B.FTAR_ERR_INVALID_ARG
    with pytest.raises(B.FtarError) as e:
        B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=5000)
    assert e.value.status == B.FTAR_ERR_INVALID_ARG
    with pytest.raises(B.FtarError) as e:
        B.ftar_ring_persistent(plan, bufs, acc, ctrl, flags=8)
    assert e.value.status == B.FTAR_ERR_INVALID_ARG
    one = B.ftar_plan(4, 0b0100, 1000, 8, torch.float32)
    B.ftar_ring_persistent(one, bufs, acc, ctrl)       # nothing to do, nothing launched
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, 0)


def _partitioned_reference(oracle, orig, n, mask, count, chunk, part, d):
    """The partitioned ring by definition: an independent ring all-reduce per partition."""
    want = np.empty_like(orig[[r for r in range(n) if (mask >> r) & 1][0]])
    for lo in range(0, count, part):
        hi = min(count, lo + part)
        sl = [None if o is None else o[lo:hi].copy() for o in orig]
        want[lo:hi] = oracle.ring_closed_form(sl, mask, hi - lo, chunk, d)
    return want


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("part", [4096, 8192 * 3, 100000, 50000 - 8])
def test_partitioned_ring_matches_a_ring_per_partition(B, oracle, dtype, part):
    n, mask, chunk = 8, 0b11110111, 512
    count = 7 * chunk * 40 + 1111
    say("persistent partitioned", dtype, part, count)
    bufs = rand_bufs(n, count, dtype, seed=part % 97, dist="student_t3", mask=mask)
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    plan.set_partition(part)
    n_parts = (count + part - 1) // part
    assert plan.n_partitions == n_parts and plan.n_slots == n_parts * 12 and plan.acc_bytes == part * 4
    # geometry of every partition against the oracle's independent rule
    for p in (0, n_parts - 1):
        lo, hi = p * part, min(count, (p + 1) * part)
        sb = oracle.geometry(n, mask, hi - lo, chunk)
        for k in range(7):
            b, e, _ = plan.partition_segment(p, k)
            assert (b, e) == (lo + sb[k], lo + sb[k + 1])
    acc = torch.full((part,), float("nan"), dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=5, timeout_us=5_000_000)
    ctrl.release(plan.n_slots)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, plan.n_slots)
    want = _partitioned_reference(oracle, orig, n, mask, count, chunk, part, code(dtype))
    for r in range(n):
        assert_same(host(bufs[r]), want if (mask >> r) & 1 else orig[r], "buf %d" % r)
    # the per-step kernels on one plan per partition over offset views give the same bits
    ref = [torch.from_numpy(o.view(np.int16 if dtype == torch.bfloat16 else np.float32).copy()).cuda().view(dtype)
           for o in orig]
    for lo in range(0, count, part):
        hi = min(count, lo + part)
        sub = B.ftar_plan(n, mask, hi - lo, chunk, dtype)
        B.ring_allreduce(sub, [x[lo:hi] for x in ref], acc)
    torch.cuda.synchronize()
    for r in range(n):
        assert torch.equal(ref[r].view(torch.uint8), bufs[r].view(torch.uint8)), r
    # the per-step calls refuse a partitioned plan
    with pytest.raises(B.FtarError) as e:
        B.ftar_reduce_step(plan, 0, bufs, torch.empty(count, dtype=torch.float32, device="cuda"))
    assert e.value.status == B.FTAR_ERR_INVALID_ARG


def test_partitioned_cancel_leaves_earlier_partitions_done_and_later_ones_untouched(B, oracle):
    n, mask, chunk, part = 4, 0xF, 256, 8192
    count = part * 5
    say("persistent partitioned cancel")
    bufs = rand_bufs(n, count, torch.float32, seed=12)
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, torch.float32)
    plan.set_partition(part)
    assert plan.n_slots == 5 * 6
    acc = torch.empty(part, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=3, timeout_us=5_000_000)
    ctrl.release(2 * 6 + 2)                  # two partitions and two ReduceScatter steps of the third
    assert _wait_progress(ctrl, 14)
    ctrl.cancel()
    torch.cuda.synchronize()
    st, done = ctrl.result()
    assert st == B.FTAR_ERR_STALE_PLAN and done == 14
    want = _partitioned_reference(oracle, orig, n, mask, count, chunk, part, 0)
    for r in range(n):
        got = host(bufs[r])
        assert_same(got[:2 * part], want[:2 * part], "finished partitions, buf %d" % r)
        assert_same(got[2 * part:], orig[r][2 * part:], "untouched partitions, buf %d" % r)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("workers", [2, 16, 255, 600])
@pytest.mark.parametrize("part,count,chunk", [(24655, 53150, 1000), (65536, 65536 * 6 + 5000, 256),
                                              (40000, 40000 * 3 + 39000, 8), (8192, 8192 * 20 + 8, 64)])
def test_shorter_last_partition_reuses_acc_only_after_everybody_is_done_with_it(B, oracle, dtype, workers, part,
                                                                                count, chunk):
    # the last partition's tiles fall elsewhere in acc than those of the partitions before it: the
    # workers hand acc over (a wait for each other) before its first slot
    n, mask = 8, 0b11010110
    say("persistent short last partition", dtype, workers, part, count, chunk)
    bufs0 = rand_bufs(n, count, dtype, seed=part % 89, dist="student_t3", mask=mask)
    orig = [host(b) for b in bufs0]
    want = _partitioned_reference(oracle, orig, n, mask, count, chunk, part, code(dtype))
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    plan.set_partition(part)
    acc = torch.empty(part, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    for rep in range(3):
        bufs = [b.clone() for b in bufs0]
        B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=workers, timeout_us=10_000_000)
        ctrl.release(plan.n_slots)
        torch.cuda.synchronize()
        assert ctrl.result() == (B.FTAR_OK, plan.n_slots)
        for r in range(n):
            assert_same(host(bufs[r]), want if (mask >> r) & 1 else orig[r], "rep %d buf %d" % (rep, r))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n_blocks,flags", [(3, 2), (16, 2), (16, 3), (300, 2)])
def test_soft_barriers_inside_long_steps_change_nothing(B, oracle, dtype, n_blocks, flags):
    # FTAR_PERSIST_ALIGN cuts a long step into runs of tiles with a bounded soft barrier between them; the tuning
    # makes the runs short (2 Mi elements) so that a step of this size has several, with a merged last one
    n, mask, chunk = 8, 0b11110111, 1024
    count = 7 * chunk * 800 + 333
    say("persistent ring, soft barriers inside steps", dtype, n_blocks, flags)
    bufs = rand_bufs(n, count, dtype, seed=61, dist="student_t3", mask=mask)
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    try:
        B.ftar_set_tuning(0, 1 << 24)
        B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=n_blocks, timeout_us=5_000_000, flags=flags)
        B.ftar_set_tuning(0, 0)
        ctrl.release(5)                                   # some steps first, the rest later
        assert _wait_progress(ctrl, 5)
        ctrl.release(12)
        torch.cuda.synchronize()
        assert ctrl.result() == (B.FTAR_OK, 12)
        want = oracle.ring_closed_form(orig, mask, count, chunk, code(dtype))
        for r in range(n):
            assert_same(host(bufs[r]), want if (mask >> r) & 1 else orig[r], "buf %d" % r)
        # a cancel while the workers wait at the gate still ends the call at once
        bufs2 = rand_bufs(n, count, dtype, seed=62, mask=mask)
        keep = [host(b) for b in bufs2]
        B.ftar_set_tuning(0, 1 << 24)
        B.ftar_ring_persistent(plan, bufs2, acc, ctrl, n_blocks=n_blocks, timeout_us=5_000_000, flags=flags)
        B.ftar_set_tuning(0, 0)
        ctrl.release(3)
        assert _wait_progress(ctrl, 3)
        ctrl.cancel()
        torch.cuda.synchronize()
        st, done = ctrl.result()
        assert st == B.FTAR_ERR_STALE_PLAN and done == 3
        for r in range(n):
            assert_same(host(bufs2[r]), keep[r], "buf %d untouched before the last ReduceScatter step" % r)
    finally:
        B.ftar_set_tuning(0, 0)
        ctrl.destroy()
