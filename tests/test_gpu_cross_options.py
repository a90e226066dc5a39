"""GPU: seeded random draws over the whole option space - element type, group size and mask,
zero-gradient participants, divisor policy, sum or mean, chunk size, ragged count, pointer
alignment, partition size, worker budget, gate unit (slots or rows of chunks), reporting and
alignment flags, release pattern - every ring path and the one-shot reduce against the
oracle, bit-exact."""
import os

import numpy as np
import pytest
import torch

from gpu_util import assert_same, code, host, rand_bufs, say

pytestmark = pytest.mark.gpu

# FTAR_SWEEP_BASE shifts every seed: a different base gives a different set of draws
BASE = int(os.environ.get("FTAR_SWEEP_BASE", "0"))


@pytest.fixture(scope="module")
def B():
    from paper_2602_00277_amd import binding
    binding.lib()
    return binding


def _draw(rng):
    n = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 11, 16, 17, 24]))
    live = int(rng.integers(1, 1 << n))
    if rng.random() < 0.4:
        live = (1 << n) - 1
    members = [r for r in range(n) if (live >> r) & 1]
    zmask = 0
    if rng.random() < 0.5:
        for r in members:
            if rng.random() < 0.3:
                zmask |= 1 << r
    contributors_only = bool(rng.random() < 0.5) and zmask != live
    sum_only = bool(rng.random() < 0.3)
    chunk = int(rng.choice([1, 3, 8, 64, 256, 1000, 4096]))
    count = int(rng.integers(1, 60000))
    if rng.random() < 0.3:
        count = len(members) * chunk * int(rng.integers(1, 6))       # exact multiple
    count = min(count, 120000)
    dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
    offset = int(rng.choice([0, 0, 0, 1, 4, 8]))                     # elements: 0 keeps 16-byte alignment
    part = 0
    if rng.random() < 0.5 and count > 16:
        part = int(rng.integers(max(1, count // 9), count))
        if rng.random() < 0.5:
            part = max(8, part // 8 * 8)
    workers = int(rng.choice([1, 3, 16, 200]))
    flags = int(rng.choice([0, 0, 1, 2, 3, 4, 5, 6, 7]))             # PUBLISH 1, ALIGN 2, CHUNKS 4
    release = str(rng.choice(["all", "all", "batches", "each"]))
    return dict(flags=flags, release=release, n=n, live=live, zmask=zmask, contributors_only=contributors_only, sum_only=sum_only,
                chunk=chunk, count=count, dtype=dtype, offset=offset, part=part, workers=workers)


def _ring_reference(oracle, orig, c, lo, hi):
    """Closed form of one ring over the element range [lo, hi) (a partition is a ring of its own)."""
    sl = [None if o is None else np.ascontiguousarray(o[lo:hi]) for o in orig]
    dt = code(c["dtype"])
    if c["sum_only"]:
        any_live = [s for r, s in enumerate(sl) if (c["live"] >> r) & 1][0]
        zero = np.zeros(hi - lo, dtype=any_live.dtype)
        sl = [zero if (c["zmask"] >> r) & 1 else s for r, s in enumerate(sl)]
        return oracle.ring_closed_form(sl, c["live"], hi - lo, c["chunk"], dt, sum_only=True)
    return oracle.ring_closed_form_zero(sl, c["live"], c["zmask"], hi - lo, c["chunk"], dt, c["contributors_only"])


def _release(ctrl, n_slots, how, rng):
    """The CPU side of the gate: everything at once, in random batches, or slot by slot waiting for
    the reported progress in between (bounded: the kernel's own timeout ends a stuck run)."""
    import time
    if how == "all" or n_slots == 0:
        ctrl.release(n_slots)
        return
    done = 0
    while done < n_slots:
        done = min(n_slots, done + (1 if how == "each" else int(rng.integers(1, 9))))
        ctrl.release(done)
        if how == "each":
            t0 = time.time()
            while ctrl.progress() < done and time.time() - t0 < 20:
                pass
            assert ctrl.progress() >= done, "progress stuck at %d of %d" % (ctrl.progress(), done)


@pytest.mark.parametrize("seed", range(120))
def test_random_option_draw(B, oracle, seed):
    rng = np.random.default_rng(1000 + BASE + seed)
    c = _draw(rng)
    say("cross options", seed, {k: (hex(v) if k in ("live", "zmask") else v) for k, v in c.items()})
    n, live, count, dtype = c["n"], c["live"], c["count"], c["dtype"]
    store = rand_bufs(n, count + 16, dtype, seed=seed, dist="student_t3" if seed % 2 else "normal", mask=live)
    for r in range(n):
        if (c["zmask"] >> r) & 1:
            store[r].fill_(float("nan"))
        elif (live >> r) & 1 and count > 4:
            store[r][c["offset"]:c["offset"] + 2] = -0.0
    views = [s[c["offset"]:c["offset"] + count] for s in store]
    orig = [host(v) for v in views]
    op = B.FTAR_SUM if c["sum_only"] else B.FTAR_MEAN

    # one-shot
    out_store = torch.empty(count + 16, dtype=dtype, device="cuda")
    out = out_store[c["offset"]:c["offset"] + count]
    B.ftar_reduce_masked_ex(views, live, out, zero_mask=c["zmask"], contributors_only=c["contributors_only"], op=op)
    torch.cuda.synchronize()
    want = oracle.reduce_masked_ex(orig, live, code(dtype), code(dtype), c["zmask"], c["contributors_only"],
                                   c["sum_only"], count=count)
    assert_same(host(out), want, "one-shot")

    # ring paths
    plan = B.ftar_plan(n, live, count, c["chunk"], dtype)
    if c["zmask"] == live and plan.n_live == 1:
        with pytest.raises(B.FtarError) as e:
            B.ftar_plan_set_zero_mask(plan, c["zmask"], c["contributors_only"])
        assert e.value.status == B.FTAR_ERR_NO_LIVE
        return
    B.ftar_plan_set_zero_mask(plan, c["zmask"], c["contributors_only"])
    B.ftar_plan_set_op(plan, op)
    want = _ring_reference(oracle, orig, c, 0, count)
    acc_store = torch.empty(count + 16, dtype=torch.float32, device="cuda")
    acc = acc_store[c["offset"]:c["offset"] + count]
    ctrl = B.ftar_ctrl_create()
    for name in ("steps", "gather_all", "scatter_all+gather_all", "onepass", "persistent", "partitioned"):
        bufs = [s.clone()[c["offset"]:c["offset"] + count] for s in store]
        ref = want
        if name == "steps":
            B.ring_allreduce(plan, bufs, acc)
        elif name == "gather_all":
            for step in range(plan.n_steps):
                B.ftar_reduce_step(plan, step, bufs, acc)
            B.ftar_allgather_all(plan, bufs)
        elif name == "scatter_all+gather_all":
            B.ftar_reduce_scatter_all(plan, bufs)
            B.ftar_allgather_all(plan, bufs)
        elif name == "onepass":
            B.ftar_allreduce_onepass(plan, bufs)
        else:
            if name == "partitioned":
                if not c["part"]:
                    continue
                plan.set_partition(c["part"])
                ref = np.concatenate([_ring_reference(oracle, orig, c, lo, min(count, lo + c["part"]))
                                      for lo in range(0, count, c["part"])])
            flags = c["flags"]
            if flags & B.FTAR_PERSIST_CHUNKS and count // c["chunk"] > 3000:
                flags &= 3                                  # rows of one or three elements by the ten thousand: slots then
            units = plan.n_gate_units(flags)
            assert units > 0 or plan.n_live < 2                 # a ring of one has no steps
            B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=c["workers"], timeout_us=10_000_000, flags=flags)
            _release(ctrl, units, c["release"], rng)
            torch.cuda.synchronize()
            assert ctrl.result() == (B.FTAR_OK, units), name
        torch.cuda.synchronize()
        for r in range(n):
            assert_same(host(bufs[r]), ref if (live >> r) & 1 else orig[r], "%s buf %d" % (name, r))
    ctrl.destroy()


@pytest.mark.parametrize("seed", range(40))
def test_random_bucketed_draw(B, oracle, seed):
    rng = np.random.default_rng(5000 + BASE + seed)
    n = int(rng.choice([1, 2, 3, 5, 8, 13, 16, 17, 30]))
    dtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
    bucket = int(rng.choice([1, 7, 8, 100, 1024, 4096, 5000, 50000]))
    n_buckets = int(rng.integers(1, 40 if bucket >= 100 else 300))
    count = (n_buckets - 1) * bucket + int(rng.integers(1, bucket + 1))
    offset = int(rng.choice([0, 0, 1, 8]))
    masks = []
    for b in range(n_buckets):
        m = int(rng.integers(0, 1 << n)) if rng.random() < 0.8 else (1 << n) - 1
        masks.append(m if m else 1 << (b % n))
    say("bucketed draw", seed, n, dtype, bucket, n_buckets, count, offset)
    store = rand_bufs(n, count + 16, dtype, seed=seed)
    views = [s[offset:offset + count] for s in store]
    out = torch.empty(count + 16, dtype=dtype, device="cuda")[offset:offset + count]
    B.ftar_reduce_masked_bucketed(views, masks, bucket, out)
    torch.cuda.synchronize()
    got, hv = host(out), [host(v) for v in views]
    for b, m in enumerate(masks):
        lo, hi = b * bucket, min(count, (b + 1) * bucket)
        want = oracle.reduce_masked([np.ascontiguousarray(h[lo:hi]) if (m >> r) & 1 else None
                                     for r, h in enumerate(hv)], m, code(dtype))
        assert_same(got[lo:hi], want, "bucket %d mask %s" % (b, hex(m)))
