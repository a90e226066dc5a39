#!/usr/bin/env python3
"""Benchmark of the FTAR GPU data path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic gradients with the
shape of the largest single-GPU benchmark workload, cfg 4: one GPU's gradient shard, 8 replicas x
2,000,000,000 bf16 elements (32 GB of inputs), all live:

  plan            ftar_plan over the live set                       (CPU)
  masked reduce   ftar_reduce_masked -> out                         (36 GB per call)
  ring schedule   N-1 ftar_reduce_step + N-1 ftar_allgather_step    (14 kernels for N = 8)
  bucketed        ftar_reduce_masked_bucketed, 25 Mi-element buckets with per-bucket
                  live masks                                        (1 kernel)

`value` is the algorithmic bytes (read + written) of all those kernels divided by the wall time
of the step, inputs resident in HBM.  Every kernel launch of the timed region carries a pair of
HIP events that its own dispatch records on the stream it runs on (begin and end of the kernel);
`roofline` reports the kernel kind that takes the largest share of the step, `kernels` reports
all kinds (the first row is the masked reduce of cfg 4 itself).  Nothing of this workload fits
the 256 MB Infinity Cache, so every fraction is an HBM figure.  `ring_cfg3a` adds the four ring
kernel kinds on the third workload (16 x 256 Mi bf16, 15 + 15 steps), measured the same way after
the timed region.  `cpu_baseline` times the CPU oracle (plain single-threaded C++) on a stated
sample of the same step on the host.

The ring runs in place, so later steps reduce already reduced buffers; kernel time does not
depend on the values.  Parity is checked once, before timing, on fresh inputs, on sampled slabs
against the oracle.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak


def algorithmic_bytes(kind, n_live, elem_bytes, count):
    """Bytes the method itself must move per launch (dead replicas are never read)."""
    E = elem_bytes
    per_elem = {
        "reduce_masked": n_live * E + E,
        "rs_first": 2 * E + 4,
        "rs_mid": 4 + E + 4,
        "rs_last": 4 + E + E,
        "rs_only": 2 * E + E,
        "allgather": E + E,
    }[kind]
    return per_elem * count


class HipEvents:
    """Raw hipEvent_t pairs from the HIP runtime already loaded in this process (plumbing only)."""

    def __init__(self):
        import ctypes
        path = None
        for line in open("/proc/self/maps"):
            if "libamdhip64" in line:
                path = line.split()[-1]
                break
        if path is None:
            raise RuntimeError("HIP runtime not loaded")
        self.ct = ctypes
        self.hip = ctypes.CDLL(path)
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                 ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = self.ct.c_void_p()
        rc = self.hip.hipEventCreate(self.ct.byref(ev))
        if rc != 0:
            raise RuntimeError("hipEventCreate failed: %d" % rc)
        return ev

    def elapsed_s(self, a, b):
        ms = self.ct.c_float()
        rc = self.hip.hipEventElapsedTime(self.ct.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return ms.value * 1e-3

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)


def all_configs_report(path, B, W, torch, np):
    """The five workloads at full size: per workload the schedule's wall time (median of
    repetitions, HIP events around the whole schedule), GB/s of algorithmic bytes, % of 8 TB/s,
    parity on sampled slabs against the oracle, and the oracle's own speed on a sample."""
    sys.path.insert(0, os.path.join(ROOT, "oracle"))
    import ftar_oracle as oracle
    dev = "cuda:0"
    SLAB = 1 << 18
    rows = []
    curve = []
    share = []

    def code(dt):
        return oracle.BF16 if dt == torch.bfloat16 else oracle.F32

    def same(got, want):
        nan_g = (got & 0x7FFF) > 0x7F80 if got.dtype == np.uint16 else np.isnan(got)
        nan_w = (want & 0x7FFF) > 0x7F80 if want.dtype == np.uint16 else np.isnan(want)
        bits = np.uint16 if got.dtype == np.uint16 else np.uint32
        return bool(np.array_equal(nan_g, nan_w) and
                    np.array_equal(got.view(bits)[~nan_g], want.view(bits)[~nan_w]))

    def starts_for(count, special, seed):
        rng = np.random.default_rng(seed)
        st = {0, max(0, count - SLAB)}
        for x in special:
            st.add(min(max(0, x - SLAB // 2), max(0, count - SLAB)))
        for x in rng.integers(0, max(1, count - SLAB), 8):
            st.add(int(x))
        return sorted(st)

    def time_schedule(fn, reps):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e-3)
        ts.sort()
        return ts[len(ts) // 2], ts[0]

    def add_row(name, what, gbytes, med, mn, ok, cpu_gbs, cpu_note):
        verdict = "bit-exact" if ok else "MISMATCH"   # every row is a real comparison with the oracle on slabs
        cpu = "-" if cpu_note in ("-", "slabs") else "%.2f (%s)" % (cpu_gbs, cpu_note)
        # bytes that are served by the caches are not a fraction of the HBM peak: no percentage for those rows
        pct = "-" if "NOT an HBM fraction" in what else "%.1f" % (100 * gbytes / med / HBM_PEAK_GBS)
        rows.append("| %s | %s | %.3f | %.1f | %.0f | %s | %.0f | %s | %s |" % (
            name, what, gbytes, med * 1e6, gbytes / med, pct, gbytes / mn, verdict, cpu))
        print(rows[-1], file=sys.stderr, flush=True)

    cfgs = W.configs()
    # ---- this box's own ceilings: bare streaming kernels, dispatch-recorded times --------
    ceil_rows = []
    ev = HipEvents()
    pairs = [(ev.create(), ev.create()) for _ in range(20)]
    for mib in (128, 1024):
        words = mib * W.M // 4
        pool = [torch.randint(-2**31, 2**31 - 1, (words,), dtype=torch.int32, device=dev) for _ in range(9)]
        for n_read, n_written in ((8, 0), (1, 0), (0, 1), (0, 8), (1, 1), (2, 1), (4, 1), (7, 1), (8, 1), (4, 4)):
            if n_read + n_written > len(pool):
                continue
            rd, wr = pool[:n_read], pool[n_read:n_read + n_written]
            for _ in range(2):
                B.ftar_probe_stream(rd, wr, fill=1)
            for a, b in pairs:
                B.ftar_time_next_launch(a, b)
                B.ftar_probe_stream(rd, wr, fill=1)
            torch.cuda.synchronize()
            ts = sorted(ev.elapsed_s(a, b) for a, b in pairs)
            t = ts[len(ts) // 2]
            gbs = (n_read + n_written) * mib * W.M / 1e9 / t
            ceil_rows.append("| %d MiB | %d | %d | %.1f | %.0f | %.1f |" % (mib, n_read, n_written, t * 1e6, gbs,
                                                                        100 * gbs / HBM_PEAK_GBS))
            print(ceil_rows[-1], file=sys.stderr, flush=True)
        # the same mixes of many read streams and one written one, the writes placed in windows of the clock
        for n_read in (4, 7, 8):
            rd, wr = pool[:n_read], pool[n_read]
            period = 4096 if n_read >= 6 else 2048
            window = period // 8 if n_read >= 6 else period // 4
            for _ in range(2):
                B.ftar_probe_stream_windows(rd, wr, period, window)
            for a, b in pairs:
                B.ftar_time_next_launch(a, b)
                B.ftar_probe_stream_windows(rd, wr, period, window)
            torch.cuda.synchronize()
            ts = sorted(ev.elapsed_s(a, b) for a, b in pairs)
            t = ts[len(ts) // 2]
            gbs = (n_read + 1) * mib * W.M / 1e9 / t
            ceil_rows.append("| %d MiB | %d | 1, in write windows (%d us period, %d us window) | %.1f | %.0f | %.1f |" % (
                mib, n_read, period // 100, window // 100, t * 1e6, gbs, 100 * gbs / HBM_PEAK_GBS))
            print(ceil_rows[-1], file=sys.stderr, flush=True)
        del pool
        torch.cuda.empty_cache()
    # ---- one-shot reduces: cfg 1, 2, 4 -------------------------------------------------
    for idx in (0, 1, 3):
        w = cfgs[idx]
        bufs = W.draw_replicas(w, dev)
        out = torch.empty(w.count, dtype=w.dtype, device=dev)
        B.ftar_reduce_masked(bufs, w.live_mask, out)
        torch.cuda.synchronize()
        ok, cpu_s, cpu_elems = True, 0.0, 0
        for st in starts_for(w.count, [1 << 30], w.seed):
            hb = [None if not (w.live_mask >> r) & 1 else W.to_numpy_bits(b[st:st + SLAB])
                  for r, b in enumerate(bufs)]
            t0 = time.perf_counter()
            want = oracle.reduce_masked(hb, w.live_mask, code(w.dtype))
            cpu_s += time.perf_counter() - t0
            cpu_elems += want.size
            ok = ok and same(W.to_numpy_bits(out[st:st + SLAB]), want)
        N = bin(w.live_mask).count("1")
        gb = (N + 1) * w.elem_bytes * w.count / 1e9
        med, mn = time_schedule(lambda: B.ftar_reduce_masked(bufs, w.live_mask, out), 20)
        add_row(w.name, "ftar_reduce_masked, N=%d%s" % (N, " (20 MiB in all, cache-resident: NOT an HBM fraction)" if idx == 0 else ""),
                gb, med, mn, ok,
                (N + 1) * w.elem_bytes * cpu_elems / cpu_s / 1e9, "%d elems" % cpu_elems)
        if idx == 1:
            # the same buffers through the delivery variants of the one-shot reduce
            zmask = 1 << 5
            out32 = torch.empty(w.count, dtype=torch.float32, device=dev)
            for what, kw, o, per_elem in (
                    ("replica 5 a zero-gradient participant (never read), divisor 7", dict(zero_mask=zmask), out,
                     (N - 1 + 1) * w.elem_bytes),
                    ("sum instead of mean", dict(op=B.FTAR_SUM), out, (N + 1) * w.elem_bytes),
                    ("fp32 mean from the bf16 inputs", dict(), out32, N * w.elem_bytes + 4)):
                B.ftar_reduce_masked_ex(bufs, w.live_mask, o, **kw)
                torch.cuda.synchronize()
                ok, cpu_s, cpu_elems = True, 0.0, 0
                for st in starts_for(w.count, [], w.seed + 1):
                    hb = [None if not (w.live_mask >> r) & 1 else W.to_numpy_bits(b[st:st + SLAB])
                          for r, b in enumerate(bufs)]
                    t0 = time.perf_counter()
                    want = oracle.reduce_masked_ex(hb, w.live_mask, code(w.dtype), code(o.dtype),
                                                   kw.get("zero_mask", 0), False, kw.get("op", 0) == B.FTAR_SUM)
                    cpu_s += time.perf_counter() - t0
                    cpu_elems += want.size
                    ok = ok and same(W.to_numpy_bits(o[st:st + SLAB]), want)
                gbv = per_elem * w.count / 1e9
                med, mn = time_schedule(lambda: B.ftar_reduce_masked_ex(bufs, w.live_mask, o, **kw), 20)
                add_row(w.name, "ftar_reduce_masked_ex: " + what, gbv, med, mn, ok,
                        per_elem * cpu_elems / cpu_s / 1e9, "%d elems" % cpu_elems)
            del out32
        del bufs, out
        torch.cuda.empty_cache()
    # ---- beyond the five workloads: the paper's upper replica count (10 to 20) in the one-shot reduce ----
    n20, mask20, count20 = 20, (1 << 20) - 1 - (1 << 7) - (1 << 13), 128 * W.M
    bufs = [torch.empty(count20, dtype=torch.bfloat16, device=dev).normal_(0, 1e-3) for _ in range(n20)]
    out = torch.empty(count20, dtype=torch.bfloat16, device=dev)
    B.ftar_reduce_masked(bufs, mask20, out)
    torch.cuda.synchronize()
    ok, cpu_s, cpu_elems = True, 0.0, 0
    for st in starts_for(count20, [], 20):
        hb = [None if not (mask20 >> r) & 1 else W.to_numpy_bits(b[st:st + SLAB]) for r, b in enumerate(bufs)]
        t0 = time.perf_counter()
        want = oracle.reduce_masked(hb, mask20, code(torch.bfloat16))
        cpu_s += time.perf_counter() - t0
        cpu_elems += want.size
        ok = ok and same(W.to_numpy_bits(out[st:st + SLAB]), want)
    gb = (18 + 1) * 2 * count20 / 1e9
    med, mn = time_schedule(lambda: B.ftar_reduce_masked(bufs, mask20, out), 20)
    add_row("extra_20x128M_bf16_drop2", "ftar_reduce_masked, N=18 of 20 replicas (N(0, 1e-3); more than 16 sources: the generic kernel)",
            gb, med, mn, ok, 19 * 2 * cpu_elems / cpu_s / 1e9, "%d elems" % cpu_elems)
    del bufs, out
    torch.cuda.empty_cache()
    # ---- ring: cfg 3a (clean 16-ring) and 3b (5 steps, replica 9 leaves, re-plan) ------
    w = cfgs[2]
    E = w.elem_bytes
    for label, schedule in (("3a clean 16-ring, 15 RS + 15 AG", [(0xFFFF, None)]),
                            ("3b 5 RS steps, replica 9 leaves, 14 RS + 14 AG",
                             [(0xFFFF, w.replan_before_step), (0xFFFF & ~(1 << w.replan_leaver), None)])):
        bufs = W.draw_replicas(w, dev)
        acc = torch.empty(w.count, dtype=torch.float32, device=dev)
        final_mask = schedule[-1][0]
        special = oracle.geometry(w.n_replicas, final_mask, w.count, w.chunk_elems)[1:-1]
        starts = starts_for(w.count, special[:3] + special[-2:], w.seed)
        orig = {st: [W.to_numpy_bits(b[st:st + SLAB]) for b in bufs] for st in starts}
        plans = [(B.ftar_plan(w.n_replicas, m, w.count, w.chunk_elems, w.dtype), steps) for m, steps in schedule]

        def run():
            for plan, steps in plans:
                if steps is None:
                    B.ring_allreduce(plan, bufs, acc)
                else:
                    for s in range(steps):
                        B.ftar_reduce_step(plan, s, bufs, acc)
        run()
        torch.cuda.synchronize()
        ok, cpu_s, cpu_elems = True, 0.0, 0
        for st in starts:
            t0 = time.perf_counter()
            want = oracle.ring_closed_form(orig[st], final_mask, w.count, w.chunk_elems, code(w.dtype),
                                           begin=st, length=SLAB)
            cpu_s += time.perf_counter() - t0
            cpu_elems += SLAB
            for r in range(w.n_replicas):
                got = W.to_numpy_bits(bufs[r][st:st + SLAB])
                ok = ok and same(got, want if (final_mask >> r) & 1 else orig[st][r])
        per_elem = 0
        for m, steps in schedule:
            N = bin(m).count("1")
            full = (2 * E + 4) + (N - 3) * (8 + E) + (4 + 2 * E) + (N - 1) * 2 * E
            if steps is None:
                per_elem += full
            else:
                per_elem += (2 * E + 4) + (steps - 1) * (8 + E)
        gb = per_elem * w.count / 1e9
        med, mn = time_schedule(run, 5)
        Nf = bin(final_mask).count("1")
        add_row(w.name, label, gb, med, mn, ok, (Nf + 1) * E * cpu_elems / cpu_s / 1e9,
                "closed form, %d elems, (N+1)E bytes/elem" % cpu_elems)
        for plan, _ in plans:
            B.ftar_plan_destroy(plan)
        if len(schedule) != 1:
            del orig
        if len(schedule) == 1:
            # the other ways to the same result, each checked on fresh inputs against the oracle's closed
            # form on slabs (the buffers are restored from the saved slabs' source: a pristine copy), then timed
            PART = 4 * W.M
            pristine = W.draw_replicas(w, dev)
            pstarts = [st for st in starts if st // PART == (st + SLAB - 1) // PART]
            ring_pos = oracle.live_ring(w.n_replicas, final_mask)

            def restore():
                for d, src in zip(bufs, pristine):
                    d.copy_(src)

            def check(part=0, owner_only=False):
                """The buffers against the closed form on the slabs; part: partition size (a partition is a
                ring of its own); owner_only: the state after the ReduceScatter phase."""
                torch.cuda.synchronize()
                good = True
                Nl = len(ring_pos)
                for st in (pstarts if part else starts):
                    if part:
                        p0 = (st // part) * part
                        L = min(part, w.count - p0)
                        want = oracle.ring_closed_form(orig[st], final_mask, L, w.chunk_elems, code(w.dtype),
                                                       begin=st - p0, length=SLAB)
                    else:
                        want = oracle.ring_closed_form(orig[st], final_mask, w.count, w.chunk_elems, code(w.dtype),
                                                       begin=st, length=SLAB)
                        sb = oracle.geometry(w.n_replicas, final_mask, w.count, w.chunk_elems)
                    for r in range(w.n_replicas):
                        got = W.to_numpy_bits(bufs[r][st:st + SLAB])
                        exp = want
                        if owner_only:
                            exp = orig[st][r].copy()
                            for k in range(Nl):
                                if ring_pos[(k + Nl - 1) % Nl] == r:
                                    lo, hi = max(st, sb[k]), min(st + SLAB, sb[k + 1])
                                    if lo < hi:
                                        exp[lo - st:hi - st] = want[lo - st:hi - st]
                        good = good and same(got, exp)
                return good
            plan = B.ftar_plan(w.n_replicas, final_mask, w.count, w.chunk_elems, w.dtype)
            ctrl = B.ftar_ctrl_create()
            n_steps = 2 * plan.n_live - 2

            def persistent(nb=0, flags=0, gate=False):
                B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=nb, timeout_us=10_000_000, flags=flags)
                if not gate:
                    ctrl.release(n_steps)
                else:
                    for s in range(n_steps):
                        ctrl.release(s + 1)
                        while ctrl.progress() < s + 1:
                            pass
            for label2, fn in (("persistent kernel, all steps released at once", lambda: persistent()),
                               ("persistent kernel, PUBLISH|ALIGN, CPU releases step by step",
                                lambda: persistent(flags=3, gate=True))):
                restore()
                fn()
                good = check()
                med, mn = time_schedule(fn, 5)
                st, done = ctrl.result()
                add_row(w.name, "3a " + label2, gb, med, mn, good and st == 0 and done == n_steps, float("nan"), "slabs")
            for nb in (2, 4, 8, 16, 32, 64, 128):
                med, mn = time_schedule(lambda: persistent(nb=nb), 1 if nb < 16 else 3)
                curve.append((nb, gb / med))
            # the paper's reason for a small budget: the ring must not take the chip away from the
            # training compute.  Other work on a second stream, alone and next to the ring.
            side = torch.cuda.Stream()
            g1 = [torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16) for _ in range(2)]
            o1 = torch.empty(8192, 8192, device=dev, dtype=torch.bfloat16)
            g2 = [torch.randn(5000, 7000, device=dev, dtype=torch.bfloat16),
                  torch.randn(7000, 9000, device=dev, dtype=torch.bfloat16)]
            o2 = torch.empty(5000, 9000, device=dev, dtype=torch.bfloat16)
            ew = torch.randn(256 * W.M, device=dev)
            others = (("bf16 GEMM 8192 x 8192 x 8192 (torch.matmul)", lambda: torch.matmul(g1[0], g1[1], out=o1)),
                      ("bf16 GEMM 5000 x 7000 x 9000 (torch.matmul)", lambda: torch.matmul(g2[0], g2[1], out=o2)),
                      ("fp32 elementwise x *= c over 1 GiB", lambda: ew.mul_(1.0001)))

            def other_loop(fn, reps=40):
                with torch.cuda.stream(side):
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    fn()
                    a.record(side)
                    for _ in range(reps):
                        fn()
                    b.record(side)
                side.synchronize()
                return a.elapsed_time(b) * 1e-3 / reps
            for name, fn in others:
                alone = other_loop(fn)
                cells = []
                for nb, release in ((2, False), (2, True), (8, True)):
                    B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=nb, timeout_us=60_000_000)
                    if release:
                        ctrl.release(n_steps)
                    t = other_loop(fn)
                    still = ctrl.progress() < n_steps
                    ctrl.cancel()                  # the ring has served its purpose: end it at its next wait
                    torch.cuda.synchronize()
                    cells.append("%+.1f %%%s" % (100 * (t / alone - 1), "" if still else " (ring ended early)"))
                share.append("| %s | %.3f | %s |" % (name, alone * 1e3, " | ".join(cells)))
            del g1, o1, g2, o2, ew
            # partitions of 4 Mi elements: acc (16 MiB) and the partition's slices stay in the caches
            plan.set_partition(PART)
            n_steps = plan.n_slots
            part_acc = acc[:PART]
            restore()
            B.ftar_ring_persistent(plan, bufs, part_acc, ctrl, timeout_us=10_000_000)
            ctrl.release(n_steps)
            good = check(part=PART)
            med, mn = time_schedule(lambda: persistent(), 5)
            st, done = ctrl.result()
            add_row(w.name, "3a persistent kernel, partitions of 4 Mi elements (%d slots; the partial sums of a "
                    "partition stay in the caches: NOT an HBM fraction)" % n_steps, gb, med, mn,
                    good and st == 0 and done == n_steps, float("nan"), "slabs")
            plan.set_partition(0)
            # the ReduceScatter steps as they are, the AllGather phase in one pass
            Np = plan.n_live

            def rs_then_gather_all():
                for st_ in range(Np - 1):
                    B.ftar_reduce_step(plan, st_, bufs, acc)
                B.ftar_allgather_all(plan, bufs)
            own_gb = ((2 * E + 4) + (Np - 3) * (8 + E) + (4 + 2 * E) + Np * E) * w.count / 1e9
            restore()
            rs_then_gather_all()
            good = check()
            med, mn = time_schedule(rs_then_gather_all, 5)
            add_row(w.name, "3a 15 RS steps + ftar_allgather_all (own bytes: E + (N-1)E for the gather)", own_gb, med, mn,
                    good, float("nan"), "slabs")
            # the ReduceScatter phase in one pass (the reduce-scatter of a sharded optimizer), alone and
            # completed by the one-pass gather
            own_gb = (Np * E + E) * w.count / 1e9
            restore()
            B.ftar_reduce_scatter_all(plan, bufs)
            good = check(owner_only=True)
            med, mn = time_schedule(lambda: B.ftar_reduce_scatter_all(plan, bufs), 5)
            add_row(w.name, "3a ftar_reduce_scatter_all (own bytes: NE + E per element)", own_gb, med, mn, good,
                    float("nan"), "slabs")

            def scatter_gather():
                B.ftar_reduce_scatter_all(plan, bufs)
                B.ftar_allgather_all(plan, bufs)
            own_gb = ((Np * E + E) + Np * E) * w.count / 1e9
            restore()
            scatter_gather()
            good = check()
            med, mn = time_schedule(scatter_gather, 5)
            add_row(w.name, "3a ftar_reduce_scatter_all + ftar_allgather_all (own bytes: (2N+1)E)", own_gb, med, mn,
                    good, float("nan"), "slabs")
            # the same result in one pass: its own algorithmic bytes are 2*N*E per element
            own_gb = 2 * plan.n_live * E * w.count / 1e9
            restore()
            B.ftar_allreduce_onepass(plan, bufs)
            good = check()
            med, mn = time_schedule(lambda: B.ftar_allreduce_onepass(plan, bufs), 5)
            add_row(w.name, "3a ftar_allreduce_onepass (own bytes: 2NE per element)", own_gb, med, mn, good,
                    float("nan"), "slabs")
            ctrl.destroy()
            B.ftar_plan_destroy(plan)
            del pristine, orig
        del bufs, acc
        torch.cuda.empty_cache()
    # ---- cfg 5: per-bucket live masks ---------------------------------------------------
    w = cfgs[4]
    edges = W.bucket_bounds(w.count, w.bucket_elems)
    masks = W.bucket_masks(w.n_replicas, len(edges) - 1, w.bucket_p_live, w.seed)
    bufs = W.draw_replicas(w, dev)
    out = torch.empty(w.count, dtype=w.dtype, device=dev)
    B.ftar_reduce_masked_bucketed(bufs, masks, w.bucket_elems, out)
    torch.cuda.synchronize()
    ok, cpu_s, cpu_bytes = True, 0.0, 0
    for b in range(len(masks)):
        for st in (edges[b], edges[b + 1] - SLAB):
            hb = [W.to_numpy_bits(x[st:st + SLAB]) if (masks[b] >> r) & 1 else None for r, x in enumerate(bufs)]
            t0 = time.perf_counter()
            want = oracle.reduce_masked(hb, masks[b], code(w.dtype))
            cpu_s += time.perf_counter() - t0
            cpu_bytes += (bin(masks[b]).count("1") + 1) * w.elem_bytes * SLAB
            ok = ok and same(W.to_numpy_bits(out[st:st + SLAB]), want)
    gb = sum((edges[b + 1] - edges[b]) * w.elem_bytes * (bin(m).count("1") + 1)
             for b, m in enumerate(masks)) / 1e9
    med, mn = time_schedule(lambda: B.ftar_reduce_masked_bucketed(bufs, masks, w.bucket_elems, out), 20)
    add_row(w.name, "ftar_reduce_masked_bucketed, %d buckets, masks %s.." % (len(masks), hex(masks[0])),
            gb, med, mn, ok, cpu_bytes / cpu_s / 1e9, "%d slabs" % (2 * len(masks)))

    head = ["# The five benchmark workloads at full size on one MI355X", "",
            "Command: `python3 bench.py --all-configs %s`. Wall time of the whole call or schedule from "
            "HIP events on the launch stream (median of repetitions; min in its own column), GB/s of "
            "algorithmic bytes (read + written), parity against the CPU oracle on sampled slabs of "
            "%d elements (first, last, portion/bucket boundaries, random), and the oracle's own "
            "throughput on those slabs on one host core (%d CPUs visible)." % (path, SLAB, os.cpu_count()),
            "", "cfg 1 is 20 MiB in total: cache-resident and launch-bound, a parity case, not an HBM "
            "measurement.", "",
            "| workload | what ran | algorithmic GB | median us | GB/s | % of 8 TB/s | GB/s (best rep) | parity | oracle GB/s, 1 core (sample) |",
            "|---|---|---|---|---|---|---|---|---|"]
    tail = ["", "## Persistent ring at a small compute-unit budget (cfg 3a)", "",
            "The paper runs its reduce/copy kernel on 2 of 132 SMs because the all-reduce is bound by a "
            "~45 GB/s network. The same design point here: GB/s of algorithmic bytes against the number "
            "of worker workgroups (one per compute unit, plus the relay workgroup).", "",
            "| worker workgroups | " + " | ".join(str(nb) for nb, _ in curve) + " |",
            "|---|" + "---|" * len(curve),
            "| GB/s | " + " | ".join("%.0f" % g for _, g in curve) + " |"]
    tail += ["", "## What the memory system gives: bare streaming kernels on this GPU", "",
             "`ftar_probe_stream`: r buffers read and w buffers written by a kernel that does nothing else "
             "(16-byte lanes, non-temporal loads, non-temporal stores when more than 256 MiB are written, "
             "one workgroup per compute unit for five or more streams, random data; median of 20 launches, "
             "dispatch-recorded times).", "",
             "| stream size | read | written | us | GB/s | % of 8 TB/s |", "|---|---|---|---|---|---|"] + ceil_rows
    tail += ["", "## Other work next to the persistent ring (cfg 3a buffers)", "",
             "40 launches in a row on a second stream of the same priority: alone, next to a ring whose two "
             "worker workgroups only wait (nothing released), and next to a running ring with 2 and 8 worker "
             "workgroups. Change of the other work's time per launch; the ring is cancelled when the loop ends.", "",
             "| other work | alone, ms | 2 workers, waiting only | 2 workers, running | 8 workers, running |",
             "|---|---|---|---|---|"]
    tail += share
    with open(path, "w") as f:
        f.write("\n".join(head + rows + tail) + "\n")
    if any("MISMATCH" in r for r in rows):
        sys.exit(1)


def full_size_launches(B, W, torch):
    """Every product kernel of the full-size workloads once, one workload after the other, for a
    run under `rocprofv3 --pmc` (FETCH_SIZE or WRITE_SIZE).  Prints the algorithmic bytes that each
    group of dispatches is expected to move, in dispatch order, as one JSON line."""
    dev = "cuda:0"
    cfgs = W.configs()
    groups = []
    # a plain copy of known size first: the counters' scale factors come from it
    a = torch.empty(128 * W.M, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    b.copy_(a)
    torch.cuda.synchronize()
    for idx in (1, 3):
        w = cfgs[idx]
        bufs = W.draw_replicas(w, dev)
        out = torch.empty(w.count, dtype=w.dtype, device=dev)
        torch.cuda.synchronize()
        B.ftar_reduce_masked(bufs, w.live_mask, out)
        torch.cuda.synchronize()
        N = bin(w.live_mask).count("1")
        groups.append({"workload": w.name, "kernel": "k_reduce_masked", "read": N * w.elem_bytes * w.count,
                       "written": w.elem_bytes * w.count})
        del bufs, out
        torch.cuda.empty_cache()
    w = cfgs[2]
    E = w.elem_bytes
    bufs = W.draw_replicas(w, dev)
    acc = torch.empty(w.count, dtype=torch.float32, device=dev)
    plan = B.ftar_plan(w.n_replicas, 0xFFFF, w.count, w.chunk_elems, w.dtype)
    torch.cuda.synchronize()
    B.ring_allreduce(plan, bufs, acc)
    torch.cuda.synchronize()
    N = 16
    groups.append({"workload": w.name, "kernel": "k_ring_reduce",
                   "read": (2 * E + (N - 3) * (4 + E) + (4 + E)) * w.count,
                   "written": (4 + (N - 3) * 4 + E) * w.count})
    groups.append({"workload": w.name, "kernel": "k_ring_allgather", "read": (N - 1) * E * w.count,
                   "written": (N - 1) * E * w.count})
    B.ftar_allreduce_onepass(plan, bufs)
    torch.cuda.synchronize()
    groups.append({"workload": w.name, "kernel": "k_ring_onepass", "read": N * E * w.count,
                   "written": N * E * w.count})
    del bufs, acc
    torch.cuda.empty_cache()
    w = cfgs[4]
    edges = W.bucket_bounds(w.count, w.bucket_elems)
    masks = W.bucket_masks(w.n_replicas, len(edges) - 1, w.bucket_p_live, w.seed)
    bufs = W.draw_replicas(w, dev)
    out = torch.empty(w.count, dtype=w.dtype, device=dev)
    torch.cuda.synchronize()
    B.ftar_reduce_masked_bucketed(bufs, masks, w.bucket_elems, out)
    torch.cuda.synchronize()
    groups.append({"workload": w.name, "kernel": "k_reduce_masked",
                   "read": sum((edges[i + 1] - edges[i]) * 4 * bin(m).count("1") for i, m in enumerate(masks)),
                   "written": 4 * w.count})
    print(json.dumps({"copy_bytes": 128 * W.M, "groups": groups}), flush=True)


def diagnose_launches(B, W, torch):
    """For runs under `rocprofv3 --pmc` that look at WHY a kernel runs at the rate it does: bare
    streaming kernels over 1 GiB streams (8 read; 8 read + 1 written; 1 written; 8 written; 1 + 1)
    next to the product kernels on streams of the same size (the one-shot reduce over 8 x 512 Mi
    bf16; one clean 16-ring over 16 x 256 Mi bf16), every launch once, in this order.  Prints the
    order and the algorithmic bytes as one JSON line."""
    dev = "cuda:0"
    GiB = 1 << 30
    groups = []
    pool = [torch.randint(-2**31, 2**31 - 1, (GiB // 4,), dtype=torch.int32, device=dev) for _ in range(9)]
    torch.cuda.synchronize()
    for n_read, n_written in ((8, 0), (8, 1), (0, 1), (0, 8), (1, 1)):
        B.ftar_probe_stream(pool[:n_read], pool[n_read:n_read + n_written], fill=1)
        torch.cuda.synchronize()
        groups.append({"kernel": "k_probe_stream<%d,%d>" % (n_read, n_written), "dispatches": 1,
                       "read": n_read * GiB, "written": n_written * GiB})
    B.ftar_probe_stream_windows(pool[:8], pool[8], 4096, 512)
    torch.cuda.synchronize()
    groups.append({"kernel": "k_probe_stream_win<8>", "dispatches": 1, "read": 8 * GiB, "written": GiB})
    bufs = [p.view(torch.bfloat16) for p in pool[:8]]        # any bit pattern is a valid input
    out = pool[8].view(torch.bfloat16)
    B.ftar_set_tuning(0, 0x80)                               # the plain kernel: no write windows
    B.ftar_reduce_masked(bufs, 0xFF, out)
    torch.cuda.synchronize()
    B.ftar_set_tuning(0, 0)
    groups.append({"kernel": "k_reduce_masked<bf16,N=8> (plain)", "dispatches": "several (about 1 GiB of traffic each)",
                   "read": 8 * GiB, "written": GiB})
    B.ftar_reduce_masked(bufs, 0xFF, out)                    # the default at this size: write windows, one launch
    torch.cuda.synchronize()
    groups.append({"kernel": "k_reduce_masked_win<bf16,N=8>", "dispatches": 1, "read": 8 * GiB, "written": GiB})
    del bufs, out, pool
    torch.cuda.empty_cache()
    w = W.configs()[2]
    E = w.elem_bytes
    bufs = W.draw_replicas(w, dev)
    acc = torch.empty(w.count, dtype=torch.float32, device=dev)
    plan = B.ftar_plan(w.n_replicas, 0xFFFF, w.count, w.chunk_elems, w.dtype)
    torch.cuda.synchronize()
    B.ring_allreduce(plan, bufs, acc)
    torch.cuda.synchronize()
    N = 16
    groups.append({"kernel": "k_ring_reduce first/mid x13/last", "dispatches": 15,
                   "read": (2 * E + (N - 3) * (4 + E) + (4 + E)) * w.count,
                   "written": (4 + (N - 3) * 4 + E) * w.count})
    groups.append({"kernel": "k_ring_allgather", "dispatches": 15, "read": (N - 1) * E * w.count,
                   "written": (N - 1) * E * w.count})
    print(json.dumps({"groups": groups}), flush=True)


def cu_budget_report(path, B, W, torch):
    """The persistent ring on a small compute-unit budget (paper section 4.2, "Optimizations": few
    units, so that the training compute keeps the chip), three ways: n worker workgroups anywhere on
    the chip; the same on a stream restricted to n compute units; several workgroups on each of the
    reserved units.  And what a GEMM on a second stream loses next to each.  16 x 64 Mi bf16."""
    import ctypes
    dev = "cuda:0"
    hip = HipEvents().hip
    hip.hipExtStreamCreateWithCUMask.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint32,
                                                 ctypes.POINTER(ctypes.c_uint32)]
    hip.hipStreamDestroy.argtypes = [ctypes.c_void_p]
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    words = (n_cu + 31) // 32

    def masked_stream(cus):
        m = (ctypes.c_uint32 * words)()
        for c in cus:
            m[c // 32] |= 1 << (c % 32)
        s = ctypes.c_void_p()
        rc = hip.hipExtStreamCreateWithCUMask(ctypes.byref(s), words, m)
        if rc != 0:
            hip.hipGetLastError()          # leave no sticky error behind
            return None
        return s

    # is a stream with a compute-unit mask to be had here at all?  (all units, then a few)
    mask_note = ""
    probe = masked_stream(range(n_cu))
    if probe is None:
        mask_note = ("`hipExtStreamCreateWithCUMask` returns an error on this machine even for the mask of all "
                     "compute units: the reserved-unit columns could not be measured.")
    else:
        hip.hipStreamDestroy(probe)
        probe = masked_stream([i * 32 for i in range(n_cu // 32)])   # the same unit in every group of 32
        if probe is None:
            mask_note = ("`hipExtStreamCreateWithCUMask` accepts the mask of all compute units but no partial "
                         "one on this machine (tried: two units; one unit in every group of 32): the reserved-unit "
                         "columns could not be measured.")
        else:
            hip.hipStreamDestroy(probe)
    hip.hipGetLastError.restype = ctypes.c_int

    n, count = 16, 64 * W.M
    E = 2
    w = W.configs()[2].scaled(count)
    bufs = W.draw_replicas(w, dev)
    acc = torch.empty(count, dtype=torch.float32, device=dev)
    plan = B.ftar_plan(n, 0xFFFF, count, w.chunk_elems, w.dtype)
    ctrl = B.ftar_ctrl_create()
    n_steps = 2 * n - 2
    gb = ((2 * E + 4) + (n - 3) * (8 + E) + (4 + 2 * E) + (n - 1) * 2 * E) * count / 1e9

    def ring(stream, nb, release=True):
        B.ftar_ring_persistent(plan, bufs, acc, ctrl, n_blocks=nb, timeout_us=60_000_000, stream=stream)
        if release:
            ctrl.release(n_steps)

    def timed(stream, nb):
        ring(stream, nb)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ring(stream, nb)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    rows = []
    for k in (2, 4, 8, 16, 32):
        groups = n_cu // 32
        cus = [g * 32 + j * (32 // max(1, k // groups)) for g in range(groups) for j in range(max(1, k // groups))]
        ms = None if (mask_note or k < groups) else masked_stream(cus)   # the same units in every group of 32
        line = ["%d" % k, "%.0f" % (gb / timed(None, k))]
        B.ftar_set_tuning(0, 0x400000)                          # small tiles: several workgroups fit a unit
        line.append("%.0f" % (gb / timed(None, k)))
        for per in (1, 2, 4):
            line.append("-" if ms is None else "%.0f" % (gb / timed(ms.value, k * per)))
        B.ftar_set_tuning(0, 0)
        line.append("-" if ms is None else "%.0f" % (gb / timed(ms.value, k)))
        for per in (2, 4):                                      # more workgroups than the budget, anywhere on the chip
            B.ftar_set_tuning(0, 0x400000)
            line.append("%.0f" % (gb / timed(None, k * per)))
            B.ftar_set_tuning(0, 0)
        if mask_note:                                           # no reserved-unit columns to show
            line = [line[i] for i in (0, 1, 2, 7, 8)]
        rows.append("| " + " | ".join(line) + " |")
        print(rows[-1], file=sys.stderr, flush=True)
        torch.cuda.synchronize()
        if ms is not None:
            hip.hipStreamDestroy(ms)
    # the neighbour: a GEMM on a second stream
    side = torch.cuda.Stream()
    a = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
    b = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
    o = torch.empty(8192, 8192, device=dev, dtype=torch.bfloat16)

    def gemm_loop(reps=40):
        with torch.cuda.stream(side):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.matmul(a, b, out=o)
            e0.record(side)
            for _ in range(reps):
                torch.matmul(a, b, out=o)
            e1.record(side)
        side.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps
    alone = gemm_loop()
    share = []
    k = 8
    cus = [i * (n_cu // k) for i in range(k)]
    ms = None if mask_note else masked_stream(cus)
    cases = [("8 workers anywhere, waiting only", None, 8, 0, False),
             ("8 workers anywhere, running", None, 8, 0, True),
             ("2 workers anywhere, waiting only", None, 2, 0, False),
             ("2 workers anywhere, running", None, 2, 0, True)]
    if ms is not None:
        cases += [("8 reserved units x 1 workgroup, waiting only", ms.value, 8, 0x400000, False),
                  ("8 reserved units x 1 workgroup, running", ms.value, 8, 0x400000, True),
                  ("8 reserved units x 4 workgroups, running", ms.value, 32, 0x400000, True)]
    for label, stream, nb, flags, release in cases:
        B.ftar_set_tuning(0, flags)
        ring(stream, nb, release)
        t = gemm_loop()
        still = ctrl.progress() < n_steps
        ctrl.cancel()
        torch.cuda.synchronize()
        B.ftar_set_tuning(0, 0)
        share.append("| %s | %.3f | %+.1f %%%s |" % (label, t * 1e3, 100 * (t / alone - 1),
                                                     "" if still or not release else " (ring ended before the loop)"))
        print(share[-1], file=sys.stderr, flush=True)
    if ms is not None:
        hip.hipStreamDestroy(ms)
    ctrl.destroy()
    out = ["# The persistent ring on a compute-unit budget (one MI355X, %d compute units)" % n_cu, "",
           "Command: `python3 bench.py --cu-budget %s`. 16 x 64 Mi bf16, clean 16-ring as ONE persistent kernel, all "
           "steps released at once; GB/s of algorithmic bytes (%.1f GB per all-reduce), wall time of one call. "
           "\"Reserved units\": the ring's stream is created with `hipExtStreamCreateWithCUMask` over that many "
           "compute units, spread evenly over the chip; its workgroups can only run there. " % (path, gb) + mask_note, "",
           ("| budget n | n workgroups anywhere, big tiles (default) | anywhere, small tiles | 2n workgroups anywhere, small tiles | 4n anywhere, small tiles |"
            if mask_note else
            "| budget n | n workgroups anywhere, big tiles (default) | anywhere, small tiles | n reserved units x 1 workgroup, small tiles | x 2 | x 4 | n reserved units x 1, big tiles | 2n workgroups anywhere, small tiles | 4n anywhere, small tiles |"),
           ("|---|---|---|---|---|" if mask_note else "|---|---|---|---|---|---|---|---|---|")] + rows + [
           "", "## A GEMM next to it", "",
           "bf16 8192 x 8192 x 8192 (`torch.matmul`) 40 times on a second stream of the same priority; alone: %.3f ms." % (alone * 1e3), "",
           "| the ring | GEMM ms | change |", "|---|---|---|"] + share
    # ---- what a few workgroups can move at all ------------------------------------------------
    del bufs, acc, a, b, o
    torch.cuda.empty_cache()
    nbytes = 256 * W.M
    pool = [torch.randint(-2**31, 2**31 - 1, (nbytes // 4,), dtype=torch.int32, device=dev) for _ in range(3)]
    few = []
    for n_read in (1, 2):
        for threads, per_lane in ((256, 8), (256, 32), (1024, 8)):
            if n_read == 2 and per_lane == 32:
                continue                        # not offered: does not fit the registers
            cells = []
            for wg in (2, 8):
                def probe():
                    B.ftar_probe_stream_workgroups(pool[:n_read], pool[2], wg, threads, per_lane)
                probe()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                probe()
                e1.record()
                torch.cuda.synchronize()
                cells.append("%.1f" % ((n_read + 1) * nbytes / 1e9 / (e0.elapsed_time(e1) * 1e-3) / wg))
            few.append("| %d + 1 | %d | %d | %s |" % (n_read, threads, per_lane, " | ".join(cells)))
            print(few[-1], file=sys.stderr, flush=True)
    del pool
    torch.cuda.empty_cache()
    out += ["", "## What one workgroup can move, whatever it keeps in flight", "",
            "`ftar_probe_stream_workgroups`: the bare streaming kernel (16-byte lanes, ordinary loads and stores, streams of "
            "256 MiB) on exactly 2 and 8 workgroups. GB/s of bytes read + written PER WORKGROUP, by workgroup size and by "
            "16-byte vectors per lane and tile (loads in flight per lane). The persistent ring's worker workgroups (256 lanes, "
            "32 vectors per lane at a small budget) are to be read against these.", "",
            "| streams read + written | lanes per workgroup | vectors per lane and tile | GB/s per workgroup, 2 workgroups | 8 workgroups |",
            "|---|---|---|---|---|"] + few
    # ---- the chunk pipeline at the paper's chunk size ---------------------------------------
    S = 4 * W.M                      # 8 MB of bf16: the paper's chunk
    n, count = 16, 1024 * W.M
    bufs = [torch.empty(count, dtype=torch.bfloat16, device=dev).normal_(0, 1e-3) for _ in range(n)]
    ctrl = B.ftar_ctrl_create()
    gb2 = ((2 * E + 4) + (n - 3) * (8 + E) + (4 + 2 * E) + (n - 1) * 2 * E) * count / 1e9
    pipe = []
    for C in (1, 4, 16):
        part = S * C * n
        plan = B.ftar_plan(n, 0xFFFF, count, S, torch.bfloat16)
        plan.set_partition(part)
        acc = torch.empty(plan.acc_bytes // 4, dtype=torch.float32, device=dev)
        cells = []
        # ahead: how many rows the CPU keeps released beyond the progress it has seen (0: all at once)
        for flags, ahead in ((0, 0), (B.FTAR_PERSIST_CHUNKS, 0), (B.FTAR_PERSIST_CHUNKS | B.FTAR_PERSIST_PUBLISH, 1),
                             (B.FTAR_PERSIST_CHUNKS | B.FTAR_PERSIST_PUBLISH, 2), (B.FTAR_PERSIST_CHUNKS, 2)):
            units = plan.n_gate_units(flags)

            def run():
                B.ftar_ring_persistent(plan, bufs, acc, ctrl, timeout_us=60_000_000, flags=flags)
                if ahead == 0:
                    ctrl.release(units)
                else:
                    done = 0
                    ctrl.release(min(units, ahead))
                    while done < units:
                        p = ctrl.progress()
                        if p > done:
                            done = p
                            ctrl.release(min(units, done + ahead))
            run()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run()
            torch.cuda.synchronize()
            t = time.perf_counter() - t0
            ok = ctrl.result() == (0, units)
            cells.append("%d units, %.0f GB/s%s" % (units, gb2 / t, "" if ok else " (FAILED)"))
        pipe.append("| %d | %d Mi elements (%d partitions) | %s |" % (C, part // W.M, plan.n_partitions, " | ".join(cells)))
        print(pipe[-1], file=sys.stderr, flush=True)
        plan.destroy()
        del acc
    ctrl.destroy()
    out += ["", "## The chunk pipeline at the paper's chunk size", "",
            "16 x 1 Gi bf16 (%.0f GB per all-reduce), chunk S = 8 MB (4 Mi bf16 elements), partitions of S x C x N bytes "
            "(paper section 4.2), one persistent kernel, one workgroup per compute unit (two with partitions). Gate units: "
            "slots (a whole step of a partition), or rows of chunks (FTAR_PERSIST_CHUNKS: C rows per step). Last two columns: "
            "a CPU thread releases row u + 1 only after every workgroup has reported row u written back (PUBLISH) - the "
            "handshake fully exposed -, the same thread keeping two rows released beyond the progress it has seen, as a "
            "pipeline with chunks in flight does, and that without PUBLISH (progress then means computed, not yet written "
            "back from the L2)." % gb2, "",
            "| C | partition | gated by slots, all released | gated by rows of chunks, all released | rows released one by one by the CPU (PUBLISH) | rows released two ahead of the progress (PUBLISH) | two ahead, without PUBLISH |",
            "|---|---|---|---|---|---|---|"] + pipe
    with open(path, "w") as f:
        f.write("\n".join(out) + "\n")


def _same(np, got, want):
    nan_g = (got & 0x7FFF) > 0x7F80 if got.dtype == np.uint16 else np.isnan(got)
    nan_w = (want & 0x7FFF) > 0x7F80 if want.dtype == np.uint16 else np.isnan(want)
    bits = np.uint16 if got.dtype == np.uint16 else np.uint32
    return bool(np.array_equal(nan_g, nan_w) and
                np.array_equal(got.view(bits)[~nan_g], want.view(bits)[~nan_w]))


KERNEL_NAME = {"reduce_masked": "k_reduce_masked", "rs_first": "k_ring_reduce<kRsFirst>",
               "rs_mid": "k_ring_reduce<kRsMid>", "rs_last": "k_ring_reduce<kRsLast>",
               "rs_only": "k_ring_reduce<kRsOnly>", "allgather": "k_ring_allgather",
               "bucketed": "k_reduce_bucketed"}


def _kernel_table(kinds, dur, bytes_of, wall_s):
    rows = []
    for kind in dict.fromkeys(kinds):
        d = dur[kind]
        avg = sum(d) / len(d)
        ach = bytes_of[kind] / avg / 1e9
        rows.append({"kind": kind, "kernel": KERNEL_NAME[kind], "launches_per_step": kinds.count(kind),
                     "avg_us": round(avg * 1e6, 2), "bytes_per_launch": bytes_of[kind],
                     "achieved_GBps": round(ach, 1), "frac_of_peak": round(ach / HBM_PEAK_GBS, 4),
                     "share_of_step": round(avg * kinds.count(kind) / wall_s, 4)})
    return rows


def ring_cfg3a(B, W, torch, hip_events, reps=3):
    """The four ring kernel kinds on the third workload (16 x 256 Mi bf16, clean 16-ring): average
    dispatch-recorded duration per kind over `reps` whole schedules (one warm-up schedule first)."""
    w = W.configs()[2]
    dev = "cuda:0"
    bufs = W.draw_replicas(w, dev)
    acc = torch.empty(w.count, dtype=torch.float32, device=dev)
    plan = B.ftar_plan(w.n_replicas, w.live_mask, w.count, w.chunk_elems, w.dtype)
    N, E = plan.n_live, w.elem_bytes
    kinds = ["rs_first"] + ["rs_mid"] * (N - 3) + ["rs_last"] + ["allgather"] * (N - 1)
    bytes_of = {k: algorithmic_bytes(k, N, E, w.count) for k in set(kinds)}
    B.ring_allreduce(plan, bufs, acc)
    torch.cuda.synchronize()
    events = [[(hip_events.create(), hip_events.create()) for _ in kinds] for _ in range(reps)]
    t0 = time.perf_counter()
    for ev in events:
        for i in range(2 * (N - 1)):
            B.ftar_time_next_launch(ev[i][0], ev[i][1])
            if i < N - 1:
                B.ftar_reduce_step(plan, i, bufs, acc)
            else:
                B.ftar_allgather_step(plan, i - (N - 1), bufs)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / reps
    dur = {}
    for ev in events:
        for i, kind in enumerate(kinds):
            dur.setdefault(kind, []).append(hip_events.elapsed_s(ev[i][0], ev[i][1]))
    total = sum(bytes_of[k] for k in kinds)
    plan.destroy()
    return {"workload": w.name, "n_live": N, "count": w.count, "schedules_timed": reps,
            "ms_per_schedule": round(wall * 1e3, 3), "bytes_per_schedule": total,
            "schedule_GBps": round(total / wall / 1e9, 1),
            "kernels": _kernel_table(kinds, dur, bytes_of, wall)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true")
    ap.add_argument("--no-ring-cfg3a", action="store_true",
                    help="skip the extra measurement of the ring kernel kinds on the third workload")
    ap.add_argument("--count", type=int, default=None,
                    help="development only: elements per replica instead of cfg 4's 2,000,000,000 "
                         "(the workload name in the output then says so)")
    ap.add_argument("--all-configs", metavar="PATH", default=None,
                    help="instead of the step benchmark, run the five benchmark workloads at full "
                         "size (parity on sampled slabs, timing, oracle timing on a sample) and "
                         "write a markdown report to PATH")
    ap.add_argument("--full-size-launches", action="store_true",
                    help="launch every product kernel of the full-size workloads once (for a run under "
                         "rocprofv3 --pmc) and print the bytes each group of dispatches should move")
    ap.add_argument("--tuning", metavar="BLOCKS_PER_CU,FLAGS", default=None,
                    help="development only: ftar_set_tuning before anything runs (the output says so)")
    ap.add_argument("--cu-budget", metavar="PATH", default=None,
                    help="the persistent ring on few compute units (anywhere / on reserved units of a CU-masked "
                         "stream) and a GEMM next to it; writes a markdown report to PATH")
    ap.add_argument("--diagnose-launches", action="store_true",
                    help="bare streaming kernels and the product kernels on 1 GiB streams, each launched "
                         "once (for runs under rocprofv3 --pmc with stall and request counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (simulated replicas are separate buffers on "
              "one device; no collectives between GPUs). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_00277_amd import binding as B
    from paper_2602_00277_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()  # raises if libftar.so is not built: there is no fallback path
    torch.cuda.set_device(0)
    dev = "cuda:0"
    if args.tuning:
        bpc, flags = (int(x, 0) for x in args.tuning.split(","))
        B.ftar_set_tuning(bpc, flags)
    if args.all_configs:
        all_configs_report(args.all_configs, B, W, torch, np)
        return
    if args.full_size_launches:
        full_size_launches(B, W, torch)
        return
    if args.diagnose_launches:
        diagnose_launches(B, W, torch)
        return
    if args.cu_budget:
        cu_budget_report(args.cu_budget, B, W, torch)
        return

    w = W.configs()[3]                      # cfg 4: the largest single-GPU workload
    name = w.name + ("" if not args.tuning else "_with_tuning_" + args.tuning)
    if args.count is not None:
        w = w.scaled(args.count)
        name = "%s_scaled_to_%d_elements" % (name, args.count)
    E, count, n, mask = w.elem_bytes, w.count, w.n_replicas, w.live_mask
    bucket_elems = min(25 * W.M, count)
    n_buckets = (count + bucket_elems - 1) // bucket_elems
    bmasks = W.bucket_masks(n, n_buckets, 0.9, seed=w.seed)

    # a plain copy of known size before anything else: under `rocprofv3 --pmc` the scale factors of
    # FETCH_SIZE and WRITE_SIZE come from this first copy kernel of the run (128 MiB read and written)
    marker = torch.empty(128 * W.M, dtype=torch.uint8, device=dev)
    torch.empty_like(marker).copy_(marker)
    torch.cuda.synchronize()
    del marker

    t_setup = time.perf_counter()
    bufs = W.draw_replicas(w, dev)
    out = torch.empty(count, dtype=w.dtype, device=dev)
    out_b = torch.empty(count, dtype=w.dtype, device=dev)
    acc = torch.empty(count, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    print("bench.py: %d x %d %s drawn in %.1f s" % (n, count, "bf16" if E == 2 else "f32",
                                                    time.perf_counter() - t_setup), file=sys.stderr, flush=True)
    stream = torch.cuda.Stream()  # default priority

    plan0 = B.ftar_plan(n, mask, count, w.chunk_elems, w.dtype)
    N = plan0.n_live
    B.ftar_plan_destroy(plan0)

    # kinds in launch order within one step
    kinds = ["reduce_masked"]
    if N == 2:
        kinds += ["rs_only"]
    elif N >= 3:
        kinds += ["rs_first"] + ["rs_mid"] * (N - 3) + ["rs_last"]
    kinds += ["allgather"] * (N - 1 if N >= 2 else 0)
    kinds += ["bucketed"]
    bytes_of = {k: algorithmic_bytes(k, N, E, count) for k in set(kinds) if k != "bucketed"}
    bucket_len = [min(count, (b + 1) * bucket_elems) - b * bucket_elems for b in range(n_buckets)]
    bytes_of["bucketed"] = sum(L * E * (bin(m).count("1") + 1) for L, m in zip(bucket_len, bmasks))
    step_bytes = sum(bytes_of[k] for k in kinds)
    per_elem_step = step_bytes / count

    def step(events=None):
        """events: one (start, stop) hipEvent_t pair per kernel of the step, or None."""
        plan = B.ftar_plan(n, mask, count, w.chunk_elems, w.dtype)
        i = 0

        def arm():
            nonlocal i
            if events is not None:
                B.ftar_time_next_launch(events[i][0], events[i][1])
                i += 1
        arm()
        B.ftar_reduce_masked(bufs, mask, out, stream=stream)
        for s in range(plan.n_steps):
            arm()
            B.ftar_reduce_step(plan, s, bufs, acc, stream=stream)
        for t in range(plan.n_steps):
            arm()
            B.ftar_allgather_step(plan, t, bufs, stream=stream)
        arm()
        B.ftar_reduce_masked_bucketed(bufs, bmasks, bucket_elems, out_b, stream=stream)
        B.ftar_plan_destroy(plan)

    parity = "skipped"
    cpu_baseline = None
    if not (args.no_parity and args.no_cpu_baseline):
        sys.path.insert(0, os.path.join(ROOT, "oracle"))
        import ftar_oracle as oracle
        code = oracle.BF16 if w.dtype == torch.bfloat16 else oracle.F32
        SLAB = min(1 << 18, count)
        rng = np.random.default_rng(w.seed)
        starts = {0, count - SLAB}
        for x in [1 << 30, 1 << 31] + oracle.geometry(n, mask, count, w.chunk_elems)[1:-1] + \
                [b * bucket_elems for b in (1, 2, n_buckets // 2, n_buckets - 1)]:
            if 0 < x < count:
                starts.add(min(max(0, x - SLAB // 2), count - SLAB))
        for x in rng.integers(0, max(1, count - SLAB), 8):
            starts.add(int(x))
        starts = sorted(starts)

        if not args.no_parity:
            orig = {st: [W.to_numpy_bits(b[st:st + SLAB]) for b in bufs] for st in starts}
            step()                       # one whole step on the fresh inputs
            torch.cuda.synchronize()
            ok = True
            for st in starts:
                want_out = oracle.reduce_masked(orig[st], mask, code)
                ok = ok and _same(np, W.to_numpy_bits(out[st:st + SLAB]), want_out)
                want_ring = oracle.ring_closed_form(orig[st], mask, count, w.chunk_elems, code,
                                                    begin=st, length=SLAB)
                for r in range(n):
                    got = W.to_numpy_bits(bufs[r][st:st + SLAB])
                    ok = ok and _same(np, got, want_ring if (mask >> r) & 1 else orig[st][r])
                # the bucketed pass runs on the ring's output: every live buffer holds want_ring
                got_b = W.to_numpy_bits(out_b[st:st + SLAB])
                lo = st
                while lo < st + SLAB:
                    b = lo // bucket_elems
                    hi = min(st + SLAB, (b + 1) * bucket_elems)
                    piece = want_ring[lo - st:hi - st]
                    slabs = [piece if (bmasks[b] >> r) & 1 else None for r in range(n)]
                    ok = ok and _same(np, got_b[lo - st:hi - st], oracle.reduce_masked(slabs, bmasks[b], code))
                    lo = hi
            parity = ("bit-exact vs oracle on %d slabs of %d elements (ends, 2^30, portion and bucket "
                      "boundaries, random): masked reduce, all %d ring buffers, bucketed reduce"
                      % (len(starts), SLAB, n)) if ok else "MISMATCH"
            if not ok:
                print("bench.py: GPU step does not match the oracle", file=sys.stderr)
                sys.exit(1)
            del orig
        if not args.no_cpu_baseline:
            # the oracle's step on a bounded sample: CS slabs of CL elements, each slab put through
            # the one-shot reduce, the message-passing ring (the slab as a ring of its own: the same
            # work per element as in the full ring) and the per-bucket reduce
            CL = min(1 << 25, count)
            CS = max(1, min(8, count // CL))
            cpu_s = 0.0
            for i in range(CS):
                st = (count - CL) * i // max(1, CS - 1) if CS > 1 else 0
                slab = [W.to_numpy_bits(b[st:st + CL]) for b in bufs]
                t0 = time.perf_counter()
                oracle.reduce_masked(slab, mask, code)
                oracle.ring_per_rank(slab, mask, w.chunk_elems, code)
                lo = 0
                while lo < CL:
                    b = (st + lo) // bucket_elems
                    hi = min(CL, (b + 1) * bucket_elems - st)
                    oracle.reduce_masked([x[lo:hi] if (bmasks[b] >> r) & 1 else None for r, x in enumerate(slab)],
                                         bmasks[b], code)
                    lo = hi
                cpu_s += time.perf_counter() - t0
                del slab
            cpu_baseline = {"value": round(per_elem_step * CS * CL / cpu_s / 1e9, 3), "unit": "GB/s", "cores": 1,
                            "kind": "oracle", "seconds": round(cpu_s, 3), "host_cpus_visible": os.cpu_count(),
                            "sample": "%d slabs of %d elements per replica (%.2f %% of the workload), each put "
                                      "through the whole step: one-shot masked reduce + message-passing ring "
                                      "(the slab as a ring of its own) + per-bucket reduce; same algorithmic "
                                      "bytes per element as the GPU step" % (CS, CL, 100.0 * CS * CL / count)}

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    hip_events = HipEvents()
    events = [[(hip_events.create(), hip_events.create()) for _ in kinds] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    dur = {}
    for ev in events:
        for i, kind in enumerate(kinds):
            dur.setdefault(kind, []).append(hip_events.elapsed_s(ev[i][0], ev[i][1]))
    kernels = _kernel_table(kinds, dur, bytes_of, ms_per_step * 1e-3)
    dom = max(kernels, key=lambda k: k["share_of_step"])
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    # HBM bytes per launch from the committed rocprofv3 --pmc summary: only if it was taken on this workload
    traffic = None
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        try:
            traffic = json.load(open(traffic_file)).get(name, {}).get(dom["kind"])
        except Exception:
            traffic = None
    result = {
        "metric": "masked gradient all-reduce GB/s (read+write) and % of MI355X HBM peak",
        "value": round(value, 1), "unit": "GB/s", "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": name, "n_replicas": n, "live_mask": bin(mask), "n_live": N,
                   "count": count, "storage_dtype": "bf16" if E == 2 else "f32", "chunk_elems": w.chunk_elems,
                   "bucket_elems": bucket_elems,
                   "step": "plan + masked reduce + %d RS + %d AG step kernels + bucketed reduce"
                           % (N - 1, N - 1),
                   "bytes_per_step": step_bytes},
        "roofline": {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["achieved_GBps"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(dom["achieved_GBps"] / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "bytes_per_launch": dom["bytes_per_launch"],
                     "avg_us": dom["avg_us"]},
        "kernels": kernels,
        "cpu_baseline": cpu_baseline,
        "parity": parity,
    }
    if not args.no_ring_cfg3a and args.count is None:
        del bufs, out, out_b, acc
        torch.cuda.empty_cache()
        result["ring_cfg3a"] = ring_cfg3a(B, W, torch, hip_events)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
