"""GPU: ftar_allreduce_onepass leaves exactly what the whole step schedule leaves."""
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
@pytest.mark.parametrize("n,mask", [(2, 0b11), (3, 0b111), (4, 0b1101), (8, 0b11110111), (16, 0xFFFF), (16, 0xFDFF),
                                    (20, (1 << 20) - 1 - (1 << 7))])
def test_same_bits_as_the_step_schedule_and_the_oracle(B, oracle, dtype, n, mask):
    N = bin(mask).count("1")
    chunk = 1024
    count = N * chunk * 19 + 777
    say("onepass", dtype, n, hex(mask), count)
    bufs = rand_bufs(n, count, dtype, seed=n + 3, dist="student_t3", mask=mask)
    orig = [host(b) for b in bufs]
    ref = [b.clone() for b in bufs]
    plan = B.ftar_plan(n, mask, count, chunk, dtype)
    B.ftar_allreduce_onepass(plan, bufs)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    B.ring_allreduce(plan, ref, acc)
    torch.cuda.synchronize()
    want = oracle.ring_closed_form(orig, mask, count, chunk, code(dtype))
    for r in range(n):
        assert_same(host(bufs[r]), want if (mask >> r) & 1 else orig[r], "buf %d" % r)
        assert torch.equal(bufs[r].view(torch.uint8), ref[r].view(torch.uint8)), r


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("count,chunk", [(16 * 5 + 3, 16), (37, 4), (5, 1), (50, 64), (1000, 7), (3 * 4096 + 1, 4096)])
def test_small_and_unaligned_geometries(B, oracle, dtype, count, chunk):
    say("onepass geometry", dtype, count, chunk)
    for n, mask in ((5, 0b11111), (4, 0b1101)):
        bufs = rand_bufs(n, count, dtype, seed=count, mask=mask)
        orig = [host(b) for b in bufs]
        plan = B.ftar_plan(n, mask, count, chunk, dtype)
        B.ftar_allreduce_onepass(plan, bufs)
        torch.cuda.synchronize()
        want = oracle.ring_closed_form(orig, mask, count, chunk, code(dtype))
        for r in range(n):
            assert_same(host(bufs[r]), want if (mask >> r) & 1 else orig[r], "buf %d" % r)


def test_single_live_replica_and_errors(B):
    say("onepass degenerate")
    bufs = [torch.randn(100, device="cuda") for _ in range(3)]
    keep = [b.clone() for b in bufs]
    one = B.ftar_plan(3, 0b010, 100, 8, torch.float32)
    B.ftar_allreduce_onepass(one, bufs)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(bufs, keep))
    plan = B.ftar_plan(3, 0b111, 100, 8, torch.float32)
    with pytest.raises(B.FtarError) as e:
        B.ftar_allreduce_onepass(plan, [bufs[0], None, bufs[2]])
    assert e.value.status == B.FTAR_ERR_INVALID_ARG
    plan.set_partition(48)
    with pytest.raises(B.FtarError) as e:
        B.ftar_allreduce_onepass(plan, bufs)
    assert e.value.status == B.FTAR_ERR_INVALID_ARG
