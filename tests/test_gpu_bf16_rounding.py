"""GPU parity of the bf16 rounding inside the kernels, over (almost) every fp32 pattern.

With four live bf16 replicas the mean is 0.25 * (a + b + c + d) and 0.25 is exact, so choosing
a, b, c as the three 8-bit pieces of 4*f (and d = 0) makes the fp32 value that gets rounded equal
to f exactly: the kernel's final rounding is exercised on f itself.  Patterns whose pieces would
underflow or whose 4*f overflows are left out; the remaining ~2^32 * 0.73 patterns are compared
with the oracle's converter on a strided sample and with torch's converter on all of them."""
import numpy as np
import pytest
import torch

from gpu_util import say

pytestmark = pytest.mark.gpu


def _pieces(bits_lo, bits_hi):
    """fp32 patterns [bits_lo, bits_hi) -> f and three bf16 tensors whose exact sum is 4*f."""
    f = torch.arange(bits_lo, bits_hi, dtype=torch.int64, device="cuda").to(torch.int32).view(torch.float32)
    g = f * 4.0
    a = (g.view(torch.int32) & -65536).view(torch.float32)          # top 8 significand bits
    r1 = g - a                                                        # exact
    b = (r1.view(torch.int32) & -65536).view(torch.float32)
    c = r1 - b                                                        # exact, <= 8 bits
    ok = torch.isfinite(g) & (a + b + c == g) & (c.to(torch.bfloat16).float() == c) & \
        (b.to(torch.bfloat16).float() == b)
    ok &= f.view(torch.int32) != -2147483648      # -0: the sum (-0) + (+0) is +0, not f
    return f, a.to(torch.bfloat16), b.to(torch.bfloat16), c.to(torch.bfloat16), ok


def test_rounding_of_every_representable_sum(oracle):
    from paper_2602_00277_amd import binding as B
    B.lib()
    chunk = 1 << 26
    checked = 0
    say("bf16 rounding, 64 chunks of 2^26 patterns")
    for i in range(0, 1 << 32, chunk):
        f, a, b, c, ok = _pieces(i, i + chunk)
        d = torch.zeros_like(a)
        out = torch.empty(chunk, dtype=torch.bfloat16, device="cuda")
        B.ftar_reduce_masked([a, b, c, d], 0b1111, out)
        torch.cuda.synchronize()
        want_t = f.to(torch.bfloat16)
        same = (out.view(torch.int16) == want_t.view(torch.int16)) | ~ok
        assert bool(same.all()), "chunk at %#x" % i
        checked += int(ok.sum())
        # strided sample against the oracle's own converter
        idx = torch.arange(0, chunk, 257, device="cuda")
        fs = f[idx].cpu().numpy()
        oks = ok[idx].cpu().numpy()
        got = out[idx].cpu().view(torch.int16).numpy().view(np.uint16)
        want = oracle.f32_to_bf16(fs)
        assert np.array_equal(got[oks], want[oks]), "chunk at %#x (oracle sample)" % i
    assert checked > 0.70 * (1 << 32), checked
