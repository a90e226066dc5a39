"""GPU: seeded random draws over the whole option space - element type, group size and mask,
zero-gradient participants, divisor policy, sum or mean, chunk size, ragged count, pointer
alignment, partition size, worker budget - every ring path and the one-shot reduce against the
oracle, bit-exact."""
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
    return dict(n=n, live=live, zmask=zmask, contributors_only=contributors_only, sum_only=sum_only,
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


@pytest.mark.parametrize("seed", range(60))
def test_random_option_draw(B, oracle, seed):
    rng = np.random.default_rng(1000 + seed)
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
    for name in ("steps", "onepass", "persistent", "partitioned"):
        bufs = [s.clone()[c["offset"]:c["offset"] + count] for s in store]
        ref = want
        if name == "steps":
            B.ring_allreduce(plan, bufs, acc)
        elif name == "onepass":
            B.ftar_allreduce_onepass(plan, bufs)
        else:
            if name == "partitioned":
                if not c["part"]:
                    continue
                plan.set_partition(c["part"])
                ref = np.concatenate([_ring_reference(oracle, orig, c, lo, min(count, lo + c["part"]))
                                      for lo in range(0, count, c["part"])])
            B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=c["workers"], timeout_us=10_000_000)
            ctrl.release(plan.n_slots)
            torch.cuda.synchronize()
            assert ctrl.result() == (B.FTAR_OK, plan.n_slots), name
        torch.cuda.synchronize()
        for r in range(n):
            assert_same(host(bufs[r]), ref if (live >> r) & 1 else orig[r], "%s buf %d" % (name, r))
    ctrl.destroy()
