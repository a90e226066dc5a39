"""GPU parity: the per-step ring kernels (ftar_reduce_step / ftar_allgather_step) against the
CPU oracle's message-passing ring, step by step and bit-exact."""
import numpy as np
import pytest
import torch

from gpu_util import assert_same, code, host, rand_bufs, say

pytestmark = pytest.mark.gpu

DTYPES = [torch.float32, torch.bfloat16]


@pytest.fixture(scope="module")
def B():
    from paper_2602_00277_amd import binding
    binding.lib()
    return binding


def _run_and_check_every_step(B, oracle, n, mask, count, chunk, dtype, seed):
    bufs = rand_bufs(n, count, dtype, seed=seed, dist="student_t3", mask=mask)
    orig = [host(b) for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    N = plan.n_live
    assert [plan.segment(k)[0] for k in range(N)] + [count] == oracle.geometry(n, mask, count, chunk)
    acc = torch.full((count,), float("nan"), dtype=torch.float32, device="cuda")
    d = code(dtype)
    for s in range(N - 1):
        B.ftar_reduce_step(plan, s, bufs, acc)
        torch.cuda.synchronize()
        if s < N - 2:
            # in-flight partial sums; the user buffers are still untouched (store rule)
            assert_same(host(acc), oracle.ring_partial(orig, mask, count, chunk, d, s + 1), "acc after RS %d" % s)
            for r in range(n):
                assert_same(host(bufs[r]), orig[r], "buf %d after RS %d" % (r, s))
    ref = [o.copy() for o in orig]
    oracle.ring_per_rank(ref, mask, chunk, d, rs_steps=N - 1, ag_steps=0)
    for r in range(n):
        assert_same(host(bufs[r]), ref[r], "buf %d after ReduceScatter" % r)
    for t in range(N - 1):
        B.ftar_allgather_step(plan, t, bufs)
        torch.cuda.synchronize()
        ref = [o.copy() for o in orig]
        oracle.ring_per_rank(ref, mask, chunk, d, rs_steps=N - 1, ag_steps=t + 1)
        for r in range(n):
            assert_same(host(bufs[r]), ref[r], "buf %d after AG %d" % (r, t))
    final = oracle.ring_closed_form(orig, mask, count, chunk, d)
    for r in range(n):
        if (mask >> r) & 1:
            assert_same(host(bufs[r]), final, "final buf %d" % r)
        else:
            assert_same(host(bufs[r]), orig[r], "dead buf %d" % r)
    plan.destroy()


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
@pytest.mark.parametrize("n,mask", [(2, 0b11), (3, 0b111), (4, 0b1111), (5, 0b10111), (8, 0b11110111),
                                    (16, 0xFFFF), (16, 0xFDFF)])
def test_every_step_matches_message_passing_ring(B, oracle, dtype, n, mask):
    N = bin(mask).count("1")
    # portions of several 2048-vector tiles plus leftovers; last chunk short
    chunk = 1024
    count = N * chunk * 19 + 777
    say("ring steps", dtype, n, hex(mask), count, chunk)
    _run_and_check_every_step(B, oracle, n, mask, count, chunk, dtype, seed=n)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
@pytest.mark.parametrize("count,chunk", [(16 * 5, 16), (16 * 5 + 3, 16), (37, 4), (5, 1), (50, 64), (1000, 7),
                                         (3 * 4096 + 1, 4096)])
def test_small_and_unaligned_geometries(B, oracle, dtype, count, chunk):
    # odd chunk sizes force the element-wise kernels; tiny counts leave portions empty
    say("ring geometry", dtype, count, chunk)
    _run_and_check_every_step(B, oracle, 5, 0b11111, count, chunk, dtype, seed=count)
    _run_and_check_every_step(B, oracle, 4, 0b1101, count, chunk, dtype, seed=count + 1)


def test_single_live_replica_has_no_steps(B):
    plan = B.ftar_plan(4, 0b0100, 100, 8, torch.float32)
    assert plan.n_live == 1 and plan.n_steps == 0
    bufs = [torch.zeros(100, device="cuda") for _ in range(4)]
    say("ring single live")
    with pytest.raises(B.FtarError) as e:
        B.ftar_reduce_step(plan, 0, bufs, torch.zeros(100, device="cuda"))
    assert e.value.status == B.FTAR_ERR_BAD_STEP
    with pytest.raises(B.FtarError) as e:
        B.ftar_allgather_step(plan, 0, bufs)
    assert e.value.status == B.FTAR_ERR_BAD_STEP


def test_step_errors(B):
    plan = B.ftar_plan(4, 0b1111, 1000, 8, torch.float32)
    bufs = [torch.zeros(1000, device="cuda") for _ in range(4)]
    acc = torch.zeros(1000, device="cuda")
    say("ring step errors")
    for bad in (-1, 3, 100):
        with pytest.raises(B.FtarError) as e:
            B.ftar_reduce_step(plan, bad, bufs, acc)
        assert e.value.status == B.FTAR_ERR_BAD_STEP
    with pytest.raises(B.FtarError) as e:
        B.ftar_reduce_step(plan, 0, bufs, None)
    assert e.value.status == B.FTAR_ERR_INVALID_ARG
    with pytest.raises(B.FtarError) as e:
        B.ftar_reduce_step(plan, 0, [bufs[0], None, bufs[2], bufs[3]], acc)
    assert e.value.status == B.FTAR_ERR_INVALID_ARG


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
def test_replan_after_a_replica_leaves(B, oracle, dtype):
    # 16 replicas, five ReduceScatter steps run, then replica 9 leaves: the CPU re-plans for 15
    # and restarts; the result must equal a fresh 15-replica run and replica 9 stays untouched
    n, chunk = 16, 256
    count = 16 * 15 * chunk + 99
    say("ring replan", dtype, count)
    bufs = rand_bufs(n, count, dtype, seed=77, dist="student_t3")
    orig = [host(b) for b in bufs]
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    p16 = B.ftar_plan(n, 0xFFFF, count, chunk, dtype)
    for s in range(5):
        B.ftar_reduce_step(p16, s, bufs, acc)
    B.ftar_plan_destroy(p16)
    new_mask = 0xFFFF & ~(1 << 9)
    p15 = B.ftar_plan(n, new_mask, count, chunk, dtype)
    assert p15.n_live == 15
    B.ring_allreduce(p15, bufs, acc)
    torch.cuda.synchronize()
    fresh = oracle.ring_closed_form(orig, new_mask, count, chunk, code(dtype))
    for r in range(n):
        assert_same(host(bufs[r]), orig[r] if r == 9 else fresh, "buf %d" % r)


def test_portion_zero_equals_one_shot_reduce(B, oracle):
    n, mask, chunk = 8, 0xFF, 512
    count = 8 * chunk * 4
    say("ring vs one-shot")
    bufs = rand_bufs(n, count, torch.bfloat16, seed=5)
    out = torch.empty(count, dtype=torch.bfloat16, device="cuda")
    B.ftar_reduce_masked(bufs, mask, out)
    plan = B.ftar_plan(n, mask, count, chunk, torch.bfloat16)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    B.ring_allreduce(plan, bufs, acc)
    torch.cuda.synchronize()
    b, e, _ = plan.segment(0)
    assert torch.equal(bufs[0][b:e].view(torch.int16), out[b:e].view(torch.int16))
    # every live replica ends bit-identical
    for r in range(1, n):
        assert torch.equal(bufs[r].view(torch.int16), bufs[0].view(torch.int16))


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
@pytest.mark.parametrize("n,mask", [(64, (1 << 64) - 1), (64, 0xF0F0F0F0F0F0F0F1), (33, (1 << 33) - 1 - (1 << 16)),
                                    (64, 1 << 63), (64, (1 << 63) | 1)])
def test_largest_groups_on_every_ring_path(B, oracle, dtype, n, mask):
    # the mask is 64 bits wide: 64 replicas is the largest group the interface can name
    N = bin(mask).count("1")
    chunk = 64
    count = N * chunk * 5 + 41
    say("ring, largest groups", dtype, n, hex(mask), count)
    orig_t = rand_bufs(n, count, dtype, seed=64 + N, dist="student_t3", mask=mask)
    orig = [host(b) for b in orig_t]
    want = oracle.ring_closed_form(orig, mask, count, chunk, code(dtype))
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    assert plan.n_live == N and plan.n_steps == N - 1
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    for name in ("steps", "onepass", "persistent", "partitioned"):
        bufs = [b.clone() for b in orig_t]
        ref = want
        if name == "steps":
            B.ring_allreduce(plan, bufs, acc)
        elif name == "onepass":
            B.ftar_allreduce_onepass(plan, bufs)
        else:
            if name == "partitioned":
                part = N * chunk * 2
                plan.set_partition(part)
                ref = np.concatenate([oracle.ring_closed_form([None if o is None else np.ascontiguousarray(o[lo:lo + part])
                                                               for o in orig], mask, min(part, count - lo), chunk,
                                                              code(dtype)) for lo in range(0, count, part)])
            B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=9, timeout_us=10_000_000)
            ctrl.release(plan.n_slots)
            torch.cuda.synchronize()
            assert ctrl.result() == (B.FTAR_OK, plan.n_slots)
        torch.cuda.synchronize()
        for r in range(n):
            assert_same(host(bufs[r]), ref if (mask >> r) & 1 else orig[r], "%s buf %d" % (name, r))
