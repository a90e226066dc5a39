"""GPU parity at the full sizes of the five benchmark workloads, in the launch configuration
bench.py times.  Outputs are compared bit for bit with the CPU oracle on sampled slabs
(always including the first and last elements, portion / bucket boundaries and the places
where 32-bit offsets would overflow); workloads the oracle finishes in about a second are
compared on every element."""
import time

import numpy as np
import pytest
import torch

from gpu_util import assert_same, code, host, host_slab, say
from paper_2602_00277_amd import workloads as W

pytestmark = pytest.mark.gpu

SLAB = 1 << 16


@pytest.fixture(scope="module")
def B():
    from paper_2602_00277_amd import binding
    binding.lib()
    return binding


def _slab_starts(count, special, n_random, seed):
    rng = np.random.default_rng(seed)
    starts = {0, max(0, count - SLAB)}
    for s in special:
        for d in (-SLAB // 2, 0):
            starts.add(min(max(0, s + d), max(0, count - SLAB)))
    for s in rng.integers(0, max(1, count - SLAB), n_random):
        starts.add(int(s))
    return sorted(starts)


def test_cfg1_all_elements(B, oracle):
    w = W.configs()[0]
    say(w.name)
    bufs = W.draw_replicas(w, "cuda")
    out = torch.empty(w.count, dtype=w.dtype, device="cuda")
    B.ftar_reduce_masked(bufs, w.live_mask, out)
    torch.cuda.synchronize()
    hb = [host(b) for b in bufs]
    want = oracle.reduce_masked(hb, w.live_mask, code(w.dtype))
    assert_same(host(out), want, w.name)
    # against the exact mean: |got - ref| <= 1e-6 * mean(|x|) per element
    ref, mag = oracle.reduce_f64(hb, w.live_mask, code(w.dtype))
    assert np.all(np.abs(host(out).astype(np.float64) - ref) <= 1e-6 * mag)


def test_cfg2_all_elements(B, oracle):
    w = W.configs()[1]
    say(w.name)
    bufs = W.draw_replicas(w, "cuda")          # replica 3 is NaN-poisoned
    out = torch.empty(w.count, dtype=w.dtype, device="cuda")
    B.ftar_reduce_masked(bufs, w.live_mask, out)
    torch.cuda.synchronize()
    want = oracle.reduce_masked([host(b) for b in bufs], w.live_mask, code(w.dtype))
    assert_same(host(out), want, w.name)


def _ring_slabs(B, oracle, w, schedule):
    """schedule: list of (mask, n_rs_steps or None for the full ring)."""
    n, count, chunk = w.n_replicas, w.count, w.chunk_elems
    final_mask = schedule[-1][0]
    special = oracle.geometry(n, final_mask, count, chunk)[1:-1] + \
        oracle.geometry(n, schedule[0][0], count, chunk)[1:-1] + [1 << 30 // 1, (1 << 31) // w.elem_bytes]
    starts = _slab_starts(count, special, 12, seed=w.seed)
    bufs = W.draw_replicas(w, "cuda")
    orig = {s: [host_slab(b, s, s + SLAB) for b in bufs] for s in starts}
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    for mask, rs_steps in schedule:
        plan = B.ftar_plan(n, mask, count, chunk, w.dtype)
        if rs_steps is None:
            B.ring_allreduce(plan, bufs, acc)
        else:
            for s in range(rs_steps):
                B.ftar_reduce_step(plan, s, bufs, acc)
        B.ftar_plan_destroy(plan)
    torch.cuda.synchronize()
    for s in starts:
        want = oracle.ring_closed_form(orig[s], final_mask, count, chunk, code(w.dtype), begin=s, length=SLAB)
        for r in range(n):
            got = host_slab(bufs[r], s, s + SLAB)
            assert_same(got, want if (final_mask >> r) & 1 else orig[s][r], "%s slab %d replica %d" % (w.name, s, r))
    # every live replica ends bit-identical over the whole buffer (all-reduce postcondition)
    live = [r for r in range(n) if (final_mask >> r) & 1]
    for r in live[1:]:
        assert torch.equal(bufs[r].view(torch.int16), bufs[live[0]].view(torch.int16)), r


def test_cfg3a_clean_sixteen_ring(B, oracle):
    w = W.configs()[2]
    say(w.name, "clean 16-ring")
    _ring_slabs(B, oracle, w, [(0xFFFF, None)])


def test_cfg3b_replica_leaves_before_step_five(B, oracle):
    w = W.configs()[2]
    say(w.name, "5 RS steps, replica 9 leaves, re-plan for 15")
    _ring_slabs(B, oracle, w, [(0xFFFF, w.replan_before_step), (0xFFFF & ~(1 << w.replan_leaver), None)])


def test_cfg3b_through_the_persistent_kernel(B, oracle):
    # the same scenario driven the paper's way: one CPU-gated kernel; the CPU releases five steps,
    # learns that replica 9 has left, cancels, re-plans for 15 and runs the new ring to the end
    w = W.configs()[2]
    say(w.name, "persistent kernel: 5 steps, cancel, re-plan for 15")
    n, count, chunk = w.n_replicas, w.count, w.chunk_elems
    new_mask = 0xFFFF & ~(1 << w.replan_leaver)
    special = oracle.geometry(n, new_mask, count, chunk)[1:-1]
    starts = _slab_starts(count, special, 12, seed=w.seed + 100)
    bufs = W.draw_replicas(w, "cuda")
    orig = {s: [host_slab(b, s, s + SLAB) for b in bufs] for s in starts}
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    p16 = B.ftar_plan(n, 0xFFFF, count, chunk, w.dtype)
    B.ftar_ring_persistent(p16, bufs, acc, ctrl, timeout_us=5_000_000)
    ctrl.release(w.replan_before_step)
    import time
    t0 = time.time()
    while ctrl.progress() < w.replan_before_step and time.time() - t0 < 20:
        time.sleep(0.001)
    ctrl.cancel()
    torch.cuda.synchronize()
    st, done = ctrl.result()
    assert st == B.FTAR_ERR_STALE_PLAN and done == w.replan_before_step
    p15 = B.ftar_plan(n, new_mask, count, chunk, w.dtype)
    B.ftar_ring_persistent(p15, bufs, acc, ctrl, timeout_us=5_000_000, flags=B.FTAR_PERSIST_ALIGN)
    ctrl.release(28)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, 28)
    for s in starts:
        want = oracle.ring_closed_form(orig[s], new_mask, count, chunk, code(w.dtype), begin=s, length=SLAB)
        for r in range(n):
            assert_same(host_slab(bufs[r], s, s + SLAB), want if (new_mask >> r) & 1 else orig[s][r],
                        "slab %d replica %d" % (s, r))
    live = [r for r in range(n) if (new_mask >> r) & 1]
    for r in live[1:]:
        assert torch.equal(bufs[r].view(torch.int16), bufs[live[0]].view(torch.int16)), r


def _cfg3a_check(oracle, w, bufs, orig, starts, part, what, owner_only=False):
    """bufs against the oracle's closed form on the sampled slabs.  part: partition size in elements
    (a partition is a ring of its own over its own length) or 0.  owner_only: only the owner of each
    portion holds the result, everything else is as it was (the state after the ReduceScatter phase)."""
    n, count, chunk = w.n_replicas, w.count, w.chunk_elems
    mask = w.live_mask
    ring = oracle.live_ring(n, mask)
    N = len(ring)
    for s in starts:
        if part:
            p0 = (s // part) * part
            assert s + SLAB <= min(count, p0 + part), "slabs are drawn inside one partition"
            L = min(part, count - p0)
            want = oracle.ring_closed_form(orig[s], mask, L, chunk, code(w.dtype), begin=s - p0, length=SLAB)
            sb = [p0 + x for x in oracle.geometry(n, mask, L, chunk)]
        else:
            want = oracle.ring_closed_form(orig[s], mask, count, chunk, code(w.dtype), begin=s, length=SLAB)
            sb = oracle.geometry(n, mask, count, chunk)
        for r in range(n):
            got = host_slab(bufs[r], s, s + SLAB)
            if not owner_only:
                assert_same(got, want, "%s slab %d replica %d" % (what, s, r))
                continue
            exp = orig[s][r].copy()
            for k in range(N):                      # portion k belongs to ring position k-1
                if ring[(k + N - 1) % N] != r:
                    continue
                lo, hi = max(s, sb[k]), min(s + SLAB, sb[k + 1])
                if lo < hi:
                    exp[lo - s:hi - s] = want[lo - s:hi - s]
            assert_same(got, exp, "%s slab %d replica %d" % (what, s, r))


def test_cfg3a_every_other_ring_path_at_full_size(B, oracle):
    # the paths that deliver the ring's result differently, each on fresh 16 x 256 Mi inputs at full size:
    # the partitioned persistent ring (4 Mi-element partitions, 1920 slots), the one-pass all-reduce, the
    # one-pass ReduceScatter phase (owners only) completed by the one-pass AllGather phase
    w = W.configs()[2]
    n, count, chunk = w.n_replicas, w.count, w.chunk_elems
    mask = w.live_mask
    part = 4 * W.M
    sb = oracle.geometry(n, mask, count, chunk)
    psb = oracle.geometry(n, mask, part, chunk)
    special = sb[1:-1] + [1 << 30 // 1, (1 << 31) // w.elem_bytes]
    starts = set(_slab_starts(count, special, 10, seed=w.seed + 7))
    # slabs around portion boundaries INSIDE partitions (first, one in the middle, the last) and next to
    # partition boundaries; every slab lies inside one partition
    for p in (0, 17, count // part - 1):
        for b in psb[1:-1:5]:
            starts.add(p * part + max(0, b - SLAB // 2))
        starts.add(p * part)
        starts.add((p + 1) * part - SLAB)
    starts = sorted(x for x in starts if x // part == (x + SLAB - 1) // part and x + SLAB <= count)
    pristine = W.draw_replicas(w, "cuda")
    orig = {s: [host_slab(b, s, s + SLAB) for b in pristine] for s in starts}
    bufs = [torch.empty_like(b) for b in pristine]

    def fresh():
        for d, src in zip(bufs, pristine):
            d.copy_(src)

    live0 = bufs[0]
    # (a) partitioned persistent ring
    say(w.name, "persistent ring in partitions of 4 Mi elements")
    fresh()
    plan = B.ftar_plan(n, mask, count, chunk, w.dtype)
    plan.set_partition(part)
    acc = torch.empty(part, dtype=torch.float32, device="cuda")
    ctrl = B.ftar_ctrl_create()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, timeout_us=20_000_000)
    ctrl.release(plan.n_slots)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, plan.n_slots) and plan.n_slots == 64 * 30
    _cfg3a_check(oracle, w, bufs, orig, starts, part, "partitioned persistent ring")
    for r in range(1, n):
        assert torch.equal(bufs[r].view(torch.int16), live0.view(torch.int16)), r
    ctrl.destroy()
    plan.set_partition(0)
    del acc
    # (b) one-pass all-reduce
    say(w.name, "ftar_allreduce_onepass")
    fresh()
    B.ftar_allreduce_onepass(plan, bufs)
    torch.cuda.synchronize()
    _cfg3a_check(oracle, w, bufs, orig, starts, 0, "one-pass all-reduce")
    for r in range(1, n):
        assert torch.equal(bufs[r].view(torch.int16), live0.view(torch.int16)), r
    # (c) one-pass ReduceScatter phase: owners only ...
    say(w.name, "ftar_reduce_scatter_all, then ftar_allgather_all")
    fresh()
    B.ftar_reduce_scatter_all(plan, bufs)
    torch.cuda.synchronize()
    _cfg3a_check(oracle, w, bufs, orig, starts, 0, "reduce-scatter-all", owner_only=True)
    # ... completed by the one-pass AllGather phase
    B.ftar_allgather_all(plan, bufs)
    torch.cuda.synchronize()
    _cfg3a_check(oracle, w, bufs, orig, starts, 0, "reduce-scatter-all + allgather-all")
    for r in range(1, n):
        assert torch.equal(bufs[r].view(torch.int16), live0.view(torch.int16)), r
    # (d) the step kernels' ReduceScatter phase completed by the one-pass AllGather phase
    say(w.name, "15 ReduceScatter steps, then ftar_allgather_all")
    fresh()
    acc = torch.empty(count, dtype=torch.float32, device="cuda")
    for st in range(plan.n_steps):
        B.ftar_reduce_step(plan, st, bufs, acc)
    B.ftar_allgather_all(plan, bufs)
    torch.cuda.synchronize()
    _cfg3a_check(oracle, w, bufs, orig, starts, 0, "RS steps + allgather-all")
    plan.destroy()
    # (e) the persistent ring gated by rows of 8 MB chunks (the paper's chunk size: four rows per step, the
    # same portions), reported written back (PUBLISH: one workgroup per XCD writes its L2 back for all), the
    # CPU keeping two rows released beyond the progress it has seen
    say(w.name, "persistent ring, rows of 8 MB chunks, PUBLISH, released two rows ahead")
    fresh()
    big_chunk = 4 * W.M
    assert oracle.geometry(n, mask, count, big_chunk) == sb
    plan = B.ftar_plan(n, mask, count, big_chunk, w.dtype)
    flags = B.FTAR_PERSIST_CHUNKS | B.FTAR_PERSIST_PUBLISH
    units = plan.n_gate_units(flags)
    assert units == 30 * 4
    ctrl = B.ftar_ctrl_create()
    B.ftar_ring_persistent(plan, bufs, acc, ctrl, timeout_us=20_000_000, flags=flags)
    done, t0 = 0, time.time()
    ctrl.release(2)
    while done < units:
        p = ctrl.progress()
        if p > done:
            done = p
            ctrl.release(min(units, done + 2))
        assert time.time() - t0 < 30.0, "progress stuck at %d of %d" % (done, units)
    torch.cuda.synchronize()
    assert ctrl.result() == (B.FTAR_OK, units)
    _cfg3a_check(oracle, w, bufs, orig, starts, 0, "persistent ring by rows of chunks")
    for r in range(1, n):
        assert torch.equal(bufs[r].view(torch.int16), live0.view(torch.int16)), r
    ctrl.destroy()
    plan.destroy()


def test_cfg4_two_billion_elements(B, oracle):
    w = W.configs()[3]
    say(w.name)
    bufs = W.draw_replicas(w, "cuda")
    out = torch.empty(w.count, dtype=w.dtype, device="cuda")
    B.ftar_reduce_masked(bufs, w.live_mask, out)
    torch.cuda.synchronize()
    starts = _slab_starts(w.count, [1 << 30, (1 << 31) // 2, w.count // 2], 40, seed=w.seed)
    zeros = 0
    for s in starts:
        hb = [host_slab(b, s, s + SLAB) for b in bufs]
        zeros += int(sum((h & 0x7FFF == 0).sum() for h in hb))
        want = oracle.reduce_masked(hb, w.live_mask, code(w.dtype))
        assert_same(host_slab(out, s, s + SLAB), want, "%s slab %d" % (w.name, s))
    assert zeros > 0            # the workload really contains exact zeros
    # at any size: the same sum written with torch's fp32 ops in the same order, every element
    step = 1 << 27
    for lo in range(0, w.count, step):
        hi = min(w.count, lo + step)
        a = bufs[0][lo:hi].float()
        for r in range(1, w.n_replicas):
            a = a + bufs[r][lo:hi].float()
        a = (a * 0.125).to(torch.bfloat16)
        assert torch.equal(a.view(torch.int16), out[lo:hi].view(torch.int16)), lo


def test_cfg5_bucketed_dynamic_membership(B, oracle):
    w = W.configs()[4]
    say(w.name)
    edges = W.bucket_bounds(w.count, w.bucket_elems)
    n_buckets = len(edges) - 1
    assert n_buckets == 21 and edges[-1] - edges[-2] == 12 * W.M
    masks = W.bucket_masks(w.n_replicas, n_buckets, w.bucket_p_live, w.seed)
    assert any(m != 0xFF for m in masks)
    bufs = W.draw_replicas(w, "cuda")
    out = torch.empty(w.count, dtype=w.dtype, device="cuda")
    B.ftar_reduce_masked_bucketed(bufs, masks, w.bucket_elems, out)
    torch.cuda.synchronize()
    rng = np.random.default_rng(w.seed)
    for b in range(n_buckets):
        lo, hi = edges[b], edges[b + 1]
        for s in sorted({lo, hi - SLAB, int(rng.integers(lo, hi - SLAB))}):
            hb = [host_slab(x, s, s + SLAB) if (masks[b] >> r) & 1 else None for r, x in enumerate(bufs)]
            want = oracle.reduce_masked(hb, masks[b], code(w.dtype))
            assert_same(host_slab(out, s, s + SLAB), want, "%s bucket %d slab %d" % (w.name, b, s))
    # the same through the caller-side loop of one-shot calls with offset pointers
    out2 = torch.empty(w.count, dtype=w.dtype, device="cuda")
    for b in range(n_buckets):
        lo, hi = edges[b], edges[b + 1]
        B.ftar_reduce_masked([x[lo:hi] for x in bufs], masks[b], out2[lo:hi])
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), out2.view(torch.int32))


def test_more_than_two_to_the_thirty_two_elements(B, oracle):
    # element indices that do not fit 32 bits: 2 live of 3 replicas, 2^32 + 70001 bf16 elements each
    count = (1 << 32) + 70001
    say("beyond 2^32 elements", count)
    bufs = [torch.empty(count, dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4242)
    step = 1 << 28
    for b in bufs:
        for lo in range(0, count, step):
            hi = min(count, lo + step)
            b[lo:hi] = torch.randn(hi - lo, device="cuda", generator=gen).mul_(1e-3).to(torch.bfloat16)
    live = 0b101
    table = [bufs[0], None, bufs[1]]
    out = torch.empty(count, dtype=torch.bfloat16, device="cuda")
    B.ftar_reduce_masked(table, live, out)
    torch.cuda.synchronize()
    starts = _slab_starts(count, [1 << 31, 1 << 32, (1 << 32) + 65536], 12, seed=7)
    for s in starts:
        hb = [host_slab(bufs[0], s, s + SLAB), None, host_slab(bufs[1], s, s + SLAB)]
        assert_same(host_slab(out, s, s + SLAB), oracle.reduce_masked(hb, live, code(torch.bfloat16)), "slab %d" % s)
    for lo in range(0, count, step):           # every element, with torch's fp32 ops in the same order
        hi = min(count, lo + step)
        a = ((bufs[0][lo:hi].float() + bufs[1][lo:hi].float()) * 0.5).to(torch.bfloat16)
        assert torch.equal(a.view(torch.int16), out[lo:hi].view(torch.int16)), lo
    # the ring of two in one pass, in place: both buffers end with the mean (addition commutes,
    # so both portions equal the one-shot result bit for bit)
    plan = B.ftar_plan(3, live, count, 16384, torch.bfloat16)
    B.ftar_allreduce_onepass(plan, table)
    torch.cuda.synchronize()
    for b in bufs:
        for lo in range(0, count, step):
            hi = min(count, lo + step)
            assert torch.equal(b[lo:hi].view(torch.int16), out[lo:hi].view(torch.int16)), lo
