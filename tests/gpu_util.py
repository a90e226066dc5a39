"""Helpers shared by the GPU parity tests: host copies as raw bits and bit-exact comparison."""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2602_00277_amd import workloads as W  # noqa: E402

F32, BF16 = 0, 1


def say(*a):
    """Name the case before the GPU step runs, flushed (a fault may take the box down)."""
    print("[case]", *a, flush=True)


def code(dtype):
    return F32 if dtype == torch.float32 else BF16


def host(t):
    return None if t is None else W.to_numpy_bits(t)


def host_slab(t, lo, hi):
    return W.to_numpy_bits(t[lo:hi])


def is_nan(a):
    if a.dtype == np.float32:
        return np.isnan(a)
    return (a & 0x7FFF) > 0x7F80


def assert_same(got, want, what=""):
    """Bit-exact, except that any NaN matches any NaN."""
    assert got.dtype == want.dtype and got.shape == want.shape, (what, got.dtype, want.dtype, got.shape, want.shape)
    ng, nw = is_nan(got), is_nan(want)
    assert np.array_equal(ng, nw), what + ": NaN positions differ"
    g = got.view(np.uint32 if got.dtype == np.float32 else np.uint16)
    w = want.view(np.uint32 if want.dtype == np.float32 else np.uint16)
    bad = (g != w) & ~ng
    if np.any(bad):
        i = int(np.argmax(bad))
        raise AssertionError("%s: %d of %d elements differ, first at %d: got %s want %s" %
                             (what, int(bad.sum()), bad.size, i, hex(int(g[i])), hex(int(w[i]))))


def rand_bufs(n, count, dtype, seed, device="cuda", dist="normal", mask=None):
    w = W.Workload("t", n, count, dtype, dist, 1e-3 if dist == "normal" else 1e-4, seed,
                   (1 << n) - 1 if mask is None else mask)
    return W.draw_replicas(w, device)
