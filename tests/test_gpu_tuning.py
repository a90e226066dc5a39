"""GPU: results never depend on the launch shape or the cache policy, and the timing hook works."""
import ctypes

import pytest
import torch

from gpu_util import assert_same, code, host, rand_bufs, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2602_00277_amd import binding
    binding.lib()
    yield binding
    binding.ftar_set_tuning(0, 0)


TUNINGS = [(1, 0x10 | 0), (8, 0x10 | 1), (3, 0x10 | 2), (2, 0x10 | 3), (1, 0x20), (4, 0x10 | 3 | 0x20),
           (1, 2 << 8), (2, 8 << 8), (16, (8 << 8) | 0x10), (0, 0x80), (0, 0x100000), (3, 0x100000 | (9 << 12) | (1 << 16)),
           (0, 0)]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_every_tuning_gives_the_same_bits(B, oracle, dtype):
    n, mask, chunk = 8, 0b11110111, 2048
    count = 7 * chunk * 9 + 1234
    bufs0 = rand_bufs(n, count, dtype, seed=3, dist="student_t3", mask=mask)
    hb = [host(b) for b in bufs0]
    d = code(dtype)
    want_reduce = oracle.reduce_masked(hb, mask, d)
    want_ring = oracle.ring_closed_form(hb, mask, count, chunk, d)
    from paper_2602_00277_amd import workloads as W
    bucket = 4096 * 5
    masks = W.bucket_masks(n, (count + bucket - 1) // bucket, 0.8, seed=9)
    for bpc, flags in TUNINGS:
        say("tuning", dtype, bpc, hex(flags))
        B.ftar_set_tuning(bpc, flags)
        out = torch.empty(count, dtype=dtype, device="cuda")
        B.ftar_reduce_masked(bufs0, mask, out)
        outb = torch.empty(count, dtype=dtype, device="cuda")
        B.ftar_reduce_masked_bucketed(bufs0, masks, bucket, outb)
        bufs = [b.clone() for b in bufs0]
        plan = B.ftar_plan(n, mask, count, chunk, dtype)
        acc = torch.empty(count, dtype=torch.float32, device="cuda")
        B.ring_allreduce(plan, bufs, acc)
        torch.cuda.synchronize()
        assert_same(host(out), want_reduce, "reduce bpc=%d flags=%#x" % (bpc, flags))
        got_b = host(outb)
        for b, m in enumerate(masks):
            lo, hi = b * bucket, min(count, (b + 1) * bucket)
            assert_same(got_b[lo:hi], oracle.reduce_masked([h[lo:hi].copy() for h in hb], m, d),
                        "bucket %d bpc=%d flags=%#x" % (b, bpc, flags))
        for r in range(n):
            assert_same(host(bufs[r]), want_ring if (mask >> r) & 1 else hb[r],
                        "ring buf %d bpc=%d flags=%#x" % (r, bpc, flags))
    B.ftar_set_tuning(0, 0)


def test_time_next_launch_records_the_kernel(B):
    hip = None
    for line in open("/proc/self/maps"):
        if "libamdhip64" in line:
            hip = ctypes.CDLL(line.split()[-1])
            break
    assert hip is not None
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    a, b = ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipEventCreate(ctypes.byref(a)) == 0 and hip.hipEventCreate(ctypes.byref(b)) == 0
    count = 1 << 24
    bufs = rand_bufs(4, count, torch.float32, seed=1)
    out = torch.empty(count, device="cuda")
    say("time_next_launch")
    B.ftar_reduce_masked(bufs, 0xF, out)          # warm
    B.ftar_time_next_launch(a, b)
    B.ftar_reduce_masked(bufs, 0xF, out)
    B.ftar_reduce_masked(bufs, 0xF, out)          # not timed: the pair was consumed
    assert hip.hipEventSynchronize(b) == 0
    ms = ctypes.c_float()
    assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
    # 320 MiB moved: between 20 us (16 TB/s, impossible) and 5 ms
    assert 0.02 < ms.value < 5.0, ms.value
    torch.cuda.synchronize()
    hip.hipEventDestroy(a)
    hip.hipEventDestroy(b)


def test_long_reduce_goes_out_in_several_launches_with_the_same_bits_and_one_bracket(B, oracle):
    # 3 streams of 640 MiB: beyond the size up to which a one-shot reduce is a single launch
    hip = None
    for line in open("/proc/self/maps"):
        if "libamdhip64" in line:
            hip = ctypes.CDLL(line.split()[-1])
            break
    assert hip is not None
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    a, b = ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipEventCreate(ctypes.byref(a)) == 0 and hip.hipEventCreate(ctypes.byref(b)) == 0
    count = 320 * (1 << 20) + 12345
    say("long reduce in several launches", count)
    bufs = rand_bufs(3, count, torch.bfloat16, seed=9, mask=0b101)
    split, single = torch.empty(count, dtype=torch.bfloat16, device="cuda"), torch.empty(count, dtype=torch.bfloat16,
                                                                                       device="cuda")
    B.ftar_reduce_masked(bufs, 0b101, split)
    B.ftar_time_next_launch(a, b)
    B.ftar_reduce_masked(bufs, 0b101, split)
    assert hip.hipEventSynchronize(b) == 0
    ms = ctypes.c_float()
    assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
    # 1.9 GiB moved in all: a bracket around the whole series is above 0.2 ms; one launch of it
    # (about 1 GiB) at the 8 TB/s peak would already take 0.13 ms
    assert 0.2 < ms.value < 20.0, ms.value
    B.ftar_set_tuning(0, 0x40)
    B.ftar_reduce_masked(bufs, 0b101, single)
    B.ftar_set_tuning(0, 0)
    torch.cuda.synchronize()
    assert torch.equal(split.view(torch.int16), single.view(torch.int16))
    # sampled against the oracle, around every place a launch could begin and at both ends
    for lo in [0, count - 4096] + [k * 65536 * 16 - 2048 for k in range(1, 300, 23)]:
        if lo < 0 or lo + 4096 > count:
            continue
        want = oracle.reduce_masked([None if x is None else host(x[lo:lo + 4096]) for x in
                                     [bufs[0], None, bufs[2]]], 0b101, code(torch.bfloat16))
        assert_same(host(split[lo:lo + 4096]), want, "slab at %d" % lo)
    hip.hipEventDestroy(a)
    hip.hipEventDestroy(b)


@pytest.mark.parametrize("n,mask", [(4, 0xF), (6, 0b110111), (8, 0xFF), (16, 0xFFFF), (16, 0xBFFD), (17, 0x1FFFF),
                                    (20, 0xFFFFF), (33, 0x1FFFFF7FD), (64, (1 << 64) - 1)])
def test_write_windows_give_the_same_bits(B, oracle, n, mask):
    # the staged kernel (results held in LDS, written out in windows of the wall clock) against the plain
    # one and the oracle: several tiles per workgroup, a ragged tail, every pair of element types
    from paper_2602_00277_amd import workloads as W  # noqa: F401
    count = 8 * 256 * 256 * 5 + 8 * 300 + 5
    for in_dt, out_dt in ((torch.bfloat16, torch.bfloat16), (torch.float32, torch.float32),
                          (torch.bfloat16, torch.float32), (torch.float32, torch.bfloat16)):
        bufs = rand_bufs(n, count, in_dt, seed=40 + n, dist="student_t3", mask=mask)
        hb = [host(b) for b in bufs]
        want = oracle.reduce_masked_ex(hb, mask, code(in_dt), code(out_dt))
        outs = []
        # plain; windows at the default period (here: one flush at the end); short periods with a wide and
        # a narrow window, so that flushes happen inside windows, on a full stage and at the end
        for flags in (0x80, 0x100000, 0x100000 | (8 << 12) | (1 << 16), 0x100000 | (10 << 12) | (4 << 16)):
            say("write windows", n, hex(mask), in_dt, out_dt, hex(flags))
            B.ftar_set_tuning(0, flags)
            out = torch.empty(count, dtype=out_dt, device="cuda")
            B.ftar_reduce_masked_ex(bufs, mask, out)
            torch.cuda.synchronize()
            assert_same(host(out), want, "flags %#x" % flags)
            outs.append(out)
        for o in outs[1:]:
            assert torch.equal(o.view(torch.uint8), outs[0].view(torch.uint8))
    B.ftar_set_tuning(0, 0)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n", [5, 8, 20])
def test_write_windows_in_the_bucketed_reduce(B, oracle, dtype, n):
    # per-bucket masks: whole tiles are staged, bucket ends and buckets with more than 16 live replicas are
    # written directly; every flush reason (window, full stage, 32 tiles, end) with short periods
    from paper_2602_00277_amd import workloads as W
    tile = 256 * 4 * (4 if dtype == torch.float32 else 8)
    for bucket in (tile * 3 + 8 * 7, tile, tile * 40):
        count = 256 * tile * 3 + 8 * 11 + 3 if bucket != tile * 40 else tile * 40 * 7 + 5
        masks = W.bucket_masks(n, (count + bucket - 1) // bucket, 0.85, seed=n + bucket % 97)
        bufs = rand_bufs(n, count, dtype, seed=50 + n, dist="student_t3")
        hb = [host(b) for b in bufs]
        outs = []
        for flags in (0x80, 0x100000, 0x100000 | (8 << 12) | (1 << 16), 0x100000 | (10 << 12) | (4 << 16)):
            say("bucketed write windows", dtype, n, bucket, count, hex(flags))
            B.ftar_set_tuning(0, flags)
            out = torch.empty(count, dtype=dtype, device="cuda")
            B.ftar_reduce_masked_bucketed(bufs, masks, bucket, out)
            torch.cuda.synchronize()
            outs.append(out)
        got = host(outs[0])
        for b, m in enumerate(masks):
            lo, hi = b * bucket, min(count, (b + 1) * bucket)
            assert_same(got[lo:hi], oracle.reduce_masked([h[lo:hi].copy() for h in hb], m, code(dtype)), "bucket %d" % b)
        for o in outs[1:]:
            assert torch.equal(o.view(torch.uint8), outs[0].view(torch.uint8))
    B.ftar_set_tuning(0, 0)
