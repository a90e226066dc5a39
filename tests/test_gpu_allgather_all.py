"""GPU: the AllGather phase in one pass (every portion from its owner into all other live buffers)
leaves what the N-1 AllGather steps leave."""
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


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n,mask,count,chunk", [(2, 0b11, 5000, 64), (3, 0b111, 3 * 1024 * 9 + 5, 1024),
                                                (8, 0b11110111, 7 * 1024 * 19 + 777, 1024), (16, 0xFFFF, 16 * 4096 * 3, 4096),
                                                (16, 0xFDFF, 37, 4), (5, 0b10111, 5, 1), (20, (1 << 20) - 1 - (1 << 7), 30000, 7),
                                                (64, (1 << 64) - 1, 64 * 64 * 5 + 41, 64), (4, 0b0100, 1000, 8)])
def test_same_buffers_as_the_step_calls(B, oracle, dtype, n, mask, count, chunk):
    say("allgather_all", dtype, n, hex(mask), count, chunk)
    orig_t = rand_bufs(n, count, dtype, seed=n + 300, dist="student_t3", mask=mask)
    orig = [host(b) for b in orig_t]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    by_steps = [b.clone() for b in orig_t]
    B.ring_allreduce(plan, by_steps, acc)
    bufs = [b.clone() for b in orig_t]
    for s in range(plan.n_steps):
        B.ftar_reduce_step(plan, s, bufs, acc)
    B.ftar_allgather_all(plan, bufs)
    torch.cuda.synchronize()
    want = oracle.ring_closed_form(orig, mask, count, chunk, code(dtype))
    for r in range(n):
        if (mask >> r) & 1:
            assert torch.equal(bufs[r].view(torch.uint8), by_steps[r].view(torch.uint8)), r
        assert_same(host(bufs[r]), want if (mask >> r) & 1 else orig[r], "buf %d" % r)


def test_unaligned_buffers_and_zero_participants(B, oracle):
    n, mask, zmask, chunk = 6, 0b111011, 0b001010, 100
    count = 5 * chunk * 13 + 7
    say("allgather_all unaligned, zero participants")
    store = rand_bufs(n, count + 8, torch.bfloat16, seed=310, mask=mask)
    for r in range(n):
        if (zmask >> r) & 1:
            store[r].fill_(float("nan"))
    bufs = [s[1:1 + count] for s in store]                    # 2-byte aligned only
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, torch.bfloat16)
    B.ftar_plan_set_zero_mask(plan, zmask)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    for s in range(plan.n_steps):
        B.ftar_reduce_step(plan, s, bufs, acc)
    B.ftar_allgather_all(plan, bufs)
    torch.cuda.synchronize()
    want = oracle.ring_closed_form_zero(orig, mask, zmask, count, chunk, code(torch.bfloat16))
    for r in range(n):
        assert_same(host(bufs[r]), want if (mask >> r) & 1 else orig[r], "buf %d" % r)
    # the elements around the views are untouched
    fresh = rand_bufs(n, count + 8, torch.bfloat16, seed=310, mask=mask)
    for r in range(n):
        if (mask >> r) & 1 and not (zmask >> r) & 1:
            assert torch.equal(store[r][:1].view(torch.int16), fresh[r][:1].view(torch.int16))
            assert torch.equal(store[r][1 + count:].view(torch.int16), fresh[r][1 + count:].view(torch.int16))


def test_partitioned_plan_is_refused(B):
    plan = B.ftar_plan(4, 0b1111, 4096, 8, torch.float32)
    plan.set_partition(1024)
    bufs = [torch.zeros(4096, device="cuda") for _ in range(4)]
    with pytest.raises(B.FtarError) as e:
        B.ftar_allgather_all(plan, bufs)
    assert e.value.status == B.FTAR_ERR_INVALID_ARG


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n,mask,count,chunk", [(2, 0b11, 5000, 64), (3, 0b111, 3 * 1024 * 9 + 5, 1024),
                                                (8, 0b11110111, 7 * 1024 * 19 + 777, 1024), (16, 0xFFFF, 16 * 4096 * 3, 4096),
                                                (16, 0xFDFF, 37, 4), (20, (1 << 20) - 1 - (1 << 7), 30000, 7),
                                                (64, (1 << 64) - 1, 64 * 64 * 5 + 41, 64), (4, 0b0100, 1000, 8)])
def test_reduce_scatter_in_one_pass_is_the_state_after_the_reduce_steps(B, oracle, dtype, n, mask, count, chunk):
    say("reduce_scatter_all", dtype, n, hex(mask), count, chunk)
    orig_t = rand_bufs(n, count, dtype, seed=n + 320, dist="student_t3", mask=mask)
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    by_steps = [b.clone() for b in orig_t]
    for s in range(plan.n_steps):
        B.ftar_reduce_step(plan, s, by_steps, acc)
    bufs = [b.clone() for b in orig_t]
    B.ftar_reduce_scatter_all(plan, bufs)
    torch.cuda.synchronize()
    # the oracle's message-passing ring, stopped after its ReduceScatter phase
    want = [host(b).copy() for b in orig_t]
    oracle.ring_per_rank(want, mask, chunk, code(dtype), rs_steps=plan.n_steps, ag_steps=0)
    for r in range(n):
        assert_same(host(bufs[r]), want[r], "buf %d against the oracle" % r)
        assert_same(host(bufs[r]), host(by_steps[r]), "buf %d against the step calls" % r)
    # and the one-pass gather completes it
    B.ftar_allgather_all(plan, bufs)
    torch.cuda.synchronize()
    full = oracle.ring_closed_form([host(b) for b in orig_t], mask, count, chunk, code(dtype))
    for r in range(n):
        if (mask >> r) & 1:
            assert_same(host(bufs[r]), full, "buf %d after the gather" % r)


def test_reduce_scatter_in_one_pass_with_zero_participants_and_the_sum(B, oracle):
    n, mask, zmask, chunk = 6, 0b111011, 0b001010, 100
    count = 5 * chunk * 13 + 7
    say("reduce_scatter_all zero participants, sum")
    orig_t = rand_bufs(n, count, torch.float32, seed=330, mask=mask)
    for r in range(n):
        if (zmask >> r) & 1:
            orig_t[r].fill_(float("nan"))
    plan = B.ftar_plan(n, mask, count, chunk, torch.float32)
    B.ftar_plan_set_zero_mask(plan, zmask)
    B.ftar_plan_set_op(plan, B.FTAR_SUM)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    by_steps = [b.clone() for b in orig_t]
    for s in range(plan.n_steps):
        B.ftar_reduce_step(plan, s, by_steps, acc)
    bufs = [b.clone() for b in orig_t]
    B.ftar_reduce_scatter_all(plan, bufs)
    torch.cuda.synchronize()
    for r in range(n):
        assert_same(host(bufs[r]), host(by_steps[r]), "buf %d" % r)
    zero = np.zeros(count, dtype=np.float32)
    want = [zero.copy() if (zmask >> r) & 1 else host(b).copy() for r, b in enumerate(orig_t)]
    oracle.ring_per_rank(want, mask, chunk, code(torch.float32), rs_steps=plan.n_steps, ag_steps=0, sum_only=True)
    # portions owned by a zero participant hold the result in its buffer; its other elements are
    # whatever they were (NaN here), in the oracle's copy zeros: compare the owned portions only
    for k in range(plan.n_live):
        b, e, owner = plan.segment(k)
        assert_same(host(bufs[owner])[b:e], want[owner][b:e], "portion %d in its owner %d" % (k, owner))
