"""GPU: ftar_ring_persistent_static - the persistent ring on the library's static scratch, for callers
that cannot allocate - gives the bits of ftar_ring_persistent (and of the oracle), on two calls in a
row of which the second is smaller, and rejects what does not fit its scratch."""
import pytest
import torch

from gpu_util import assert_same, code, host, rand_bufs, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2602_00277_amd import binding
    binding.lib()
    return binding


def _both_ways(B, oracle, ctrl, n, mask, count, chunk, part, dtype, seed, n_blocks=0):
    N = bin(mask).count("1")
    say("static persistent ring", dtype, n, hex(mask), count, "partition", part, "blocks", n_blocks)
    bufs = rand_bufs(n, count, dtype, seed=seed, dist="student_t3", mask=mask)
    orig = [host(b) for b in bufs]
    ref = [b.clone() for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    if part:
        plan.set_partition(part)
    slots = plan.n_slots
    # the existing entry point, on a workspace of the caller
    acc = torch.empty(plan.acc_bytes // 4, dtype=torch.float32, device="cuda")
    B.ftar_ring_persistent(plan, ref, acc, ctrl, n_blocks=n_blocks, timeout_us=5_000_000)
    ctrl.release(slots)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, slots)
    # the entry point that allocates nothing
    B.ftar_ring_persistent_static(plan, bufs, ctrl, n_blocks=n_blocks, timeout_us=5_000_000)
    ctrl.release(slots)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, slots)
    for r in range(n):
        assert torch.equal(bufs[r].view(torch.uint8), ref[r].view(torch.uint8)), "buf %d" % r
    # and both against the oracle (partitions are rings of their own)
    P = part if part else count
    for p0 in range(0, count, P):
        L = min(P, count - p0)
        want = oracle.ring_closed_form([o[p0:p0 + L] for o in orig], mask, L, chunk, code(dtype))
        for r in range(n):
            assert_same(host(bufs[r])[p0:p0 + L], want if (mask >> r) & 1 else orig[r][p0:p0 + L],
                        "buf %d partition at %d" % (r, p0))
    plan.destroy()
    assert N >= 1


def test_static_scratch_two_calls_second_smaller(B, oracle):
    ctrl = B.ftar_ctrl_create()
    # first call: bf16, 7 of 8 live, three partitions (the last one shorter), acc = 3 * 2^17 floats
    _both_ways(B, oracle, ctrl, 8, 0b11110111, 7 * 4096 * 40 + 1234, 4096, 3 * (1 << 17), torch.bfloat16, 31)
    # second call, smaller, other type and ring size, unpartitioned: must not see the first one's leftovers
    _both_ways(B, oracle, ctrl, 5, 0b11111, 5 * 1024 * 9 + 77, 1024, 0, torch.float32, 32)
    # third: few workers (the big-tile kernel), two replicas (no partial sums at all)
    _both_ways(B, oracle, ctrl, 16, 0xFFFF, 16 * 2048 * 40, 2048, 16 * 2048 * 8, torch.bfloat16, 33, n_blocks=3)
    _both_ways(B, oracle, ctrl, 2, 0b11, 100_000, 512, 0, torch.bfloat16, 34)
    ctrl.destroy()


def test_static_scratch_limit_and_errors(B):
    ctrl = B.ftar_ctrl_create()
    limit = 4 << 20
    count = limit + 1024
    bufs = rand_bufs(3, count, torch.bfloat16, seed=35)
    before = [b.clone() for b in bufs]
    plan = B.ftar_plan(3, 0b111, count, 1024, torch.bfloat16)
    with pytest.raises(B.FtarError) as e:                      # one partition = the whole buffer: too long
        B.ftar_ring_persistent_static(plan, bufs, ctrl)
    assert e.value.status == B.FTAR_ERR_TOO_LARGE
    assert not B.ftar_status_is_retryable(B.FTAR_ERR_TOO_LARGE)
    plan.set_partition(limit + 8)
    with pytest.raises(B.FtarError) as e:
        B.ftar_ring_persistent_static(plan, bufs, ctrl)
    assert e.value.status == B.FTAR_ERR_TOO_LARGE
    torch.cuda.synchronize()
    for b, a in zip(before, bufs):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))   # nothing was enqueued
    plan.set_partition(limit)                                  # exactly the limit runs
    B.ftar_ring_persistent_static(plan, bufs, ctrl, timeout_us=5_000_000)
    ctrl.release(plan.n_slots)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, plan.n_slots)
    ref = [b.clone() for b in before]
    acc = torch.empty(limit, dtype=torch.float32, device="cuda")
    B.ftar_ring_persistent(plan, ref, acc, ctrl, timeout_us=5_000_000)
    ctrl.release(plan.n_slots)
    torch.cuda.synchronize()
    for r in range(3):
        assert torch.equal(bufs[r].view(torch.uint8), ref[r].view(torch.uint8))
    # a ring of two keeps no partial sums: no limit applies
    two = rand_bufs(2, count, torch.bfloat16, seed=36)
    plan2 = B.ftar_plan(2, 0b11, count, 1024, torch.bfloat16)
    B.ftar_ring_persistent_static(plan2, two, ctrl, timeout_us=5_000_000)
    ctrl.release(2)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, 2)
    ctrl.destroy()
