"""GPU: delivery variants - the sum of paper section 4.1 instead of the mean, an fp32 result from
bf16 inputs - and the learning-rate factors of section 6.2.  Bit-exact against the oracle."""
import ctypes

import numpy as np
import pytest
import torch

from gpu_util import BF16, F32, assert_same, code, host, rand_bufs, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2602_00277_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("n_live", list(range(1, 18)) + [20])
@pytest.mark.parametrize("sum_only", [False, True], ids=["mean", "sum"])
def test_f32_result_from_bf16_inputs(B, oracle, n_live, sum_only):
    n = n_live + 2                                   # replicas 1 and 3 are dead
    live = 0b1 if n_live == 1 else ((1 << n) - 1) & ~0b1010
    count = 256 * 4 * 8 * 3 + 4 * 37 + 3          # several tiles of every unroll, a vector tail, an element tail
    say("bf16 -> f32", n_live, "sum" if sum_only else "mean")
    bufs = rand_bufs(n, count, torch.bfloat16, seed=60 + n_live, dist="student_t3", mask=live)
    assert bin(live).count("1") == n_live
    out = torch.empty(count, dtype=torch.float32, device="cuda")
    B.ftar_reduce_masked_ex(bufs, live, out, op=B.FTAR_SUM if sum_only else B.FTAR_MEAN)
    torch.cuda.synchronize()
    want = oracle.reduce_masked_ex([host(b) for b in bufs], live, BF16, out_dtype=F32, sum_only=sum_only)
    assert_same(host(out), want)


@pytest.mark.parametrize("in_dtype,out_dtype", [(torch.float32, torch.float32), (torch.bfloat16, torch.bfloat16),
                                                (torch.bfloat16, torch.float32), (torch.float32, torch.bfloat16)],
                         ids=["f32", "bf16", "bf16-f32", "f32-bf16"])
def test_every_option_together(B, oracle, in_dtype, out_dtype):
    n, live, count = 6, 0b110111, 10000 + 5
    bufs = rand_bufs(n, count, in_dtype, seed=61, mask=live)
    for b in bufs:
        b[:4] = -0.0
    out = torch.empty(count, dtype=out_dtype, device="cuda")
    for zmask in (0, 0b000100, 0b110001, live):
        for contributors_only in (False, True):
            for sum_only in (False, True):
                if contributors_only and zmask == live:
                    continue
                say("reduce_masked_ex", in_dtype, out_dtype, bin(zmask), contributors_only, sum_only)
                work = [None if (zmask >> r) & 1 else b for r, b in enumerate(bufs)]
                B.ftar_reduce_masked_ex(work, live, out, zero_mask=zmask, contributors_only=contributors_only,
                                        op=B.FTAR_SUM if sum_only else B.FTAR_MEAN)
                torch.cuda.synchronize()
                want = oracle.reduce_masked_ex([host(b) for b in work], live, code(in_dtype), code(out_dtype), zmask,
                                               contributors_only, sum_only, count=count)
                assert_same(host(out), want, "zmask %s co %s sum %s" % (bin(zmask), contributors_only, sum_only))


def test_unaligned_buffers_take_the_element_path(B, oracle):
    n, live, count = 3, 0b111, 5001
    store = rand_bufs(n, count + 8, torch.bfloat16, seed=62)
    bufs = [s[1:1 + count] for s in store]        # 2-byte aligned only
    out_store = torch.empty(count + 4, dtype=torch.float32, device="cuda")
    out = out_store[1:1 + count]
    say("bf16 -> f32 unaligned")
    B.ftar_reduce_masked_ex(bufs, live, out, op=B.FTAR_SUM)
    torch.cuda.synchronize()
    want = oracle.reduce_masked_ex([host(b) for b in bufs], live, BF16, out_dtype=F32, sum_only=True)
    assert_same(host(out), want)


def test_unknown_operation_and_type_codes(B):
    bufs = rand_bufs(2, 64, torch.float32, seed=63)
    out = torch.empty(64, dtype=torch.float32, device="cuda")
    with pytest.raises(B.FtarError) as e:
        B.ftar_reduce_masked_ex(bufs, 0b11, out, op=2)
    assert e.value.status == B.FTAR_ERR_INVALID_ARG
    ptrs = (ctypes.c_void_p * 2)(bufs[0].data_ptr(), bufs[1].data_ptr())
    for in_code, out_code in ((0, 2), (3, 0), (-1, 1)):
        st = B.lib().ftar_reduce_masked_ex(ptrs, 2, 0b11, 0, 0, 64, in_code, out_code, 0, out.data_ptr(), None)
        assert st == B.FTAR_ERR_INVALID_ARG, (in_code, out_code)


@pytest.mark.parametrize("n_live", [1, 2, 3, 7, 8, 16, 17])
@pytest.mark.parametrize("sum_only", [False, True], ids=["mean", "sum"])
def test_bf16_result_from_f32_inputs(B, oracle, n_live, sum_only):
    n = n_live + 1                                   # replica 1 is dead
    live = ((1 << n) - 1) & ~0b10
    count = 256 * 4 * 4 * 3 + 4 * 19 + 2
    say("f32 -> bf16", n_live, "sum" if sum_only else "mean")
    bufs = rand_bufs(n, count, torch.float32, seed=80 + n_live, dist="student_t3", mask=live)
    assert bin(live).count("1") == n_live
    out = torch.empty(count, dtype=torch.bfloat16, device="cuda")
    B.ftar_reduce_masked_ex(bufs, live, out, op=B.FTAR_SUM if sum_only else B.FTAR_MEAN)
    torch.cuda.synchronize()
    want = oracle.reduce_masked_ex([host(b) for b in bufs], live, F32, out_dtype=BF16, sum_only=sum_only)
    assert_same(host(out), want)


def test_narrowing_of_every_fp32_pattern(B, oracle):
    # one live fp32 replica, sum, bf16 result: the kernel's whole arithmetic is x * 1.0f and the one
    # rounding to bf16, on x itself - all 2^32 patterns, NaNs, infinities and denormals included
    chunk = 1 << 26
    out = torch.empty(chunk, dtype=torch.bfloat16, device="cuda")
    say("fp32 -> bf16 narrowing, 64 chunks of 2^26 patterns")
    for i in range(0, 1 << 32, chunk):
        x = torch.arange(i, i + chunk, dtype=torch.int64, device="cuda").to(torch.int32).view(torch.float32)
        B.ftar_reduce_masked_ex([x], 0b1, out, op=B.FTAR_SUM)
        torch.cuda.synchronize()
        want = x.to(torch.bfloat16)                        # torch's converter: same rule for non-NaN
        nan = torch.isnan(x)
        assert bool((torch.isnan(out.float()) == nan).all()), "NaN positions, chunk at %#x" % i
        same = (out.view(torch.int16) == want.view(torch.int16)) | nan
        assert bool(same.all()), "chunk at %#x" % i
        idx = torch.arange(0, chunk, 251, device="cuda")   # strided sample against the oracle's converter
        got = out[idx].cpu().view(torch.int16).numpy().view(np.uint16)
        ref = oracle.f32_to_bf16(x[idx].cpu().numpy())
        both_nan = nan[idx].cpu().numpy()
        assert np.array_equal(got[~both_nan], ref[~both_nan]), "chunk at %#x (oracle sample)" % i
        # a NaN keeps its sign and upper payload and gets the quiet bit, as in the oracle
        assert np.array_equal(got[both_nan], ref[both_nan]), "chunk at %#x (NaN payloads)" % i


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n,live,zmask", [(2, 0b11, 0), (3, 0b111, 0), (8, 0b11110111, 0), (8, 0xFF, 0b00100100),
                                          (16, 0xFFFF, 0), (18, (1 << 18) - 1, 0)])
def test_ring_paths_deliver_the_sum(B, oracle, dtype, n, live, zmask):
    N = bin(live).count("1")
    chunk = 256
    count = N * chunk * 13 + 101
    say("ring sum", dtype, n, hex(live), hex(zmask))
    orig_t = rand_bufs(n, count, dtype, seed=n + 70, dist="student_t3", mask=live)
    orig = [host(b) for b in orig_t]
    zero = np.zeros(count, dtype=orig[[r for r in range(n) if (live >> r) & 1][0]].dtype)
    with_zeros = [zero if (zmask >> r) & 1 else b for r, b in enumerate(orig)]
    want = oracle.ring_closed_form(with_zeros, live, count, chunk, code(dtype), sum_only=True)
    plan = B.ftar_plan(n, live, count, chunk, dtype)
    B.ftar_plan_set_zero_mask(plan, zmask, True)     # the divisor policy must not matter for a sum
    B.ftar_plan_set_op(plan, B.FTAR_SUM)
    assert plan.scale == 1.0
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    for name in ("steps", "onepass", "persistent"):
        bufs = [b.clone() for b in orig_t]
        for r in range(n):
            if (zmask >> r) & 1:
                bufs[r].fill_(float("nan"))
        if name == "steps":
            B.ring_allreduce(plan, bufs, acc)
        elif name == "onepass":
            B.ftar_allreduce_onepass(plan, bufs)
        else:
            B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=5, timeout_us=5_000_000)
            ctrl.release(plan.n_slots)
        torch.cuda.synchronize()
        for r in range(n):
            assert_same(host(bufs[r]), want if (live >> r) & 1 else orig[r], "%s buf %d" % (name, r))
    # back to the mean with the same plan
    B.ftar_plan_set_op(plan, B.FTAR_MEAN)
    B.ftar_plan_set_zero_mask(plan, 0)
    bufs = [b.clone() for b in orig_t]
    B.ftar_allreduce_onepass(plan, bufs)
    torch.cuda.synchronize()
    first = [r for r in range(n) if (live >> r) & 1][0]
    assert_same(host(bufs[first]), oracle.ring_closed_form(orig, live, count, chunk, code(dtype)), "mean again")


def test_widening_of_every_bf16_pattern(B, oracle):
    # one live bf16 replica, sum, fp32 result: x * 1.0f of the widened value, every one of the 2^16 patterns
    x = torch.arange(0, 1 << 16, dtype=torch.int32, device="cuda").to(torch.int16).view(torch.bfloat16)
    out = torch.empty(1 << 16, dtype=torch.float32, device="cuda")
    say("bf16 -> fp32 widening, all 2^16 patterns")
    B.ftar_reduce_masked_ex([x], 0b1, out, op=B.FTAR_SUM)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint32)
    want = oracle.bf16_to_f32(np.arange(1 << 16, dtype=np.uint16)).view(np.uint32)
    nan = (want & 0x7FFFFFFF) > 0x7F800000
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal((got & 0x7FFFFFFF) > 0x7F800000, nan)
    # a NaN keeps sign and payload; a signalling one comes back quiet (x * 1.0f)
    assert np.array_equal(got[nan] | 0x00400000, want[nan] | 0x00400000)
