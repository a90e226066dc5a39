"""GPU: host threads may call the library at the same time, each on a stream of its own (the
library keeps its per-call state per thread and holds no lock)."""
import threading

import pytest
import torch

from gpu_util import assert_same, code, host, rand_bufs, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2602_00277_amd import binding
    binding.lib()
    return binding


def test_four_host_threads_on_four_streams(B, oracle):
    n, live, chunk = 6, 0b110111, 256
    count = 5 * chunk * 37 + 11
    say("four host threads")
    jobs = []
    for t in range(4):
        dtype = torch.bfloat16 if t % 2 else torch.float32
        bufs = rand_bufs(n, count, dtype, seed=200 + t, mask=live)
        orig = [host(b) for b in bufs]
        jobs.append(dict(dtype=dtype, bufs=bufs, orig=orig, out=torch.empty(count, dtype=dtype, device="cuda"),
                         acc=torch.empty(count, dtype=torch.float32, device="cuda"), stream=torch.cuda.Stream(),
                         error=None))
    torch.cuda.synchronize()

    def work(j):
        try:
            plan = B.ftar_plan(n, live, count, chunk, j["dtype"])
            for _ in range(10):
                B.ftar_reduce_masked(j["bufs"], live, j["out"], stream=j["stream"])
            # an error on this thread must not show up on another one
            try:
                B.ftar_reduce_step(plan, 99, j["bufs"], j["acc"], stream=j["stream"])
            except B.FtarError as e:
                assert e.status == B.FTAR_ERR_BAD_STEP
            B.ring_allreduce(plan, j["bufs"], j["acc"], stream=j["stream"])
            j["stream"].synchronize()
        except Exception as e:      # surfaced by the main thread
            j["error"] = e

    threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for i, j in enumerate(jobs):
        assert j["error"] is None, (i, j["error"])
        assert_same(host(j["out"]), oracle.reduce_masked(j["orig"], live, code(j["dtype"])), "one-shot, thread %d" % i)
        want = oracle.ring_closed_form(j["orig"], live, count, chunk, code(j["dtype"]))
        for r in range(n):
            assert_same(host(j["bufs"][r]), want if (live >> r) & 1 else j["orig"][r], "ring, thread %d buf %d" % (i, r))
