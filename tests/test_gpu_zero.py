"""GPU: zero-gradient participants (paper section 4.3): they take part, contribute +0.0, are never
read; in the ring they receive the result.  Bit-exact against the oracle."""
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


def _poison(bufs, zero_mask):
    for r, b in enumerate(bufs):
        if (zero_mask >> r) & 1:
            b.fill_(float("nan"))            # a read of a zero participant's buffer would show


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("contributors_only", [False, True])
def test_one_shot_every_zero_mask_of_five(B, oracle, dtype, contributors_only):
    n, count = 5, 4096 * 3 + 77
    live = 0b11011
    say("reduce_masked_zero", dtype, contributors_only)
    bufs = rand_bufs(n, count, dtype, seed=50, mask=live)
    bufs[0][:8] = -0.0
    for b in bufs:
        b[:4] = -0.0                         # all contributors -0.0: a zero participant turns the sum into +0.0
    out = torch.empty(count, dtype=dtype, device="cuda")
    for zmask in range(0, 1 << n):
        if zmask & ~live:
            continue
        if contributors_only and zmask == live:
            with pytest.raises(B.FtarError) as e:
                B.ftar_reduce_masked_zero(bufs, live, zmask, out, contributors_only=True)
            assert e.value.status == B.FTAR_ERR_NO_LIVE
            continue
        work = [b.clone() for b in bufs]
        _poison(work, zmask)
        B.ftar_reduce_masked_zero(work, live, zmask, out, contributors_only=contributors_only)
        torch.cuda.synchronize()
        want = oracle.reduce_masked_zero([host(b) for b in work], live, zmask, code(dtype), contributors_only)
        assert_same(host(out), want, "zero mask %s" % bin(zmask))
        # a zero participant may have no buffer at all in the one-shot call
        B.ftar_reduce_masked_zero([None if (zmask >> r) & 1 else b for r, b in enumerate(work)], live, zmask,
                                  out, contributors_only=contributors_only)
        torch.cuda.synchronize()
        assert_same(host(out), want, "NULL zero buffers, mask %s" % bin(zmask))
    with pytest.raises(B.FtarError) as e:
        B.ftar_reduce_masked_zero(bufs, live, 0b00100, out)
    assert e.value.status == B.FTAR_ERR_BAD_MASK


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("off,count", [(0, 1), (1, 1), (1, 2), (0, 1001), (1, 1001), (1, 1002), (3, 70001)])
def test_one_shot_all_zero_participants_any_alignment(B, dtype, off, count):
    say("all zero participants", dtype, off, count)
    store = torch.full((count + 8,), 7.0, dtype=dtype, device="cuda")
    out = store[off:off + count]
    B.ftar_reduce_masked_zero([None, None, None], 0b101, 0b101, out)
    torch.cuda.synchronize()
    got = host(store)
    got = got.view(np.uint32 if got.dtype == np.float32 else np.uint16)
    assert not got[off:off + count].any(), "mean of zero-gradient participants only is +0.0"
    want_other = got.dtype.type(0x40E00000 if dtype == torch.float32 else 0x40E0)
    assert (got[:off] == want_other).all() and (got[off + count:] == want_other).all(), "wrote outside out"


def test_one_shot_more_than_sixteen(B, oracle):
    n, count = 20, 5000
    live, zmask = (1 << 20) - 1, (1 << 3) | (1 << 17) | (1 << 19)
    say("reduce_masked_zero 20 replicas")
    bufs = rand_bufs(n, count, torch.float32, seed=51)
    _poison(bufs, zmask)
    out = torch.empty(count, device="cuda")
    B.ftar_reduce_masked_zero(bufs, live, zmask, out)
    torch.cuda.synchronize()
    assert_same(host(out), oracle.reduce_masked_zero([host(b) for b in bufs], live, zmask, 0))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n,live,zmask", [(2, 0b11, 0b01), (3, 0b111, 0b100), (8, 0b11110111, 0b00100001),
                                          (8, 0xFF, 0b11111110), (16, 0xFFFF, 0x8101), (20, (1 << 20) - 1, 1 << 9)])
@pytest.mark.parametrize("contributors_only", [False, True])
def test_ring_paths_with_zero_participants(B, oracle, dtype, n, live, zmask, contributors_only):
    N = bin(live).count("1")
    chunk = 512
    count = N * chunk * 11 + 333
    say("ring zero participants", dtype, n, hex(live), hex(zmask), contributors_only)
    orig_t = rand_bufs(n, count, dtype, seed=n + 7, dist="student_t3", mask=live)
    _poison(orig_t, zmask)
    orig = [host(b) for b in orig_t]
    want = oracle.ring_closed_form_zero(orig, live, zmask, count, chunk, code(dtype), contributors_only)
    plan = B.ftar_plan(n, live, count, chunk, dtype)
    B.ftar_plan_set_zero_mask(plan, zmask, contributors_only)
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    for name in ("steps", "onepass", "persistent"):
        bufs = [b.clone() for b in orig_t]
        if name == "steps":
            B.ring_allreduce(plan, bufs, acc)
        elif name == "onepass":
            B.ftar_allreduce_onepass(plan, bufs)
        else:
            B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=7, timeout_us=5_000_000)
            ctrl.release(plan.n_slots)
        torch.cuda.synchronize()
        for r in range(n):
            # zero participants receive the result too; dead replicas stay as they were
            assert_same(host(bufs[r]), want if (live >> r) & 1 else orig[r], "%s buf %d" % (name, r))


def test_plan_zero_mask_errors(B):
    plan = B.ftar_plan(4, 0b0111, 100, 8, torch.float32)
    with pytest.raises(B.FtarError) as e:
        B.ftar_plan_set_zero_mask(plan, 0b1000)
    assert e.value.status == B.FTAR_ERR_BAD_MASK
    with pytest.raises(B.FtarError) as e:
        B.ftar_plan_set_zero_mask(plan, 0b0111, True)
    assert e.value.status == B.FTAR_ERR_NO_LIVE
    B.ftar_plan_set_zero_mask(plan, 0b0010, True)
    assert abs(plan.scale - 0.5) < 1e-9
    B.ftar_plan_set_zero_mask(plan, 0, False)
    assert abs(plan.scale - 1.0 / 3.0) < 1e-7
