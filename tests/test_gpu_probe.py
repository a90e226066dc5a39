"""GPU: the measurement-only streaming probe does what its header says (so that the ceilings it
reports are ceilings of the stated traffic)."""
import pytest
import torch

from gpu_util import say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2602_00277_amd import binding
    binding.lib()
    return binding


def _bufs(n, words, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return [torch.randint(-2**31, 2**31 - 1, (words,), dtype=torch.int32, device="cuda", generator=g) for _ in range(n)]


@pytest.mark.parametrize("n_read,n_written", [(1, 1), (2, 1), (3, 1), (4, 1), (7, 1), (8, 1), (16, 1), (4, 4), (8, 8)])
def test_written_streams_hold_the_xor_of_the_read_ones(B, n_read, n_written):
    words = 3 * 32 * 1024 // 4 * 5                      # 15 x 32 KiB
    say("probe", n_read, n_written)
    read = _bufs(n_read, words, n_read)
    keep = [r.clone() for r in read]
    written = [torch.zeros(words, dtype=torch.int32, device="cuda") for _ in range(n_written)]
    B.ftar_probe_stream(read, written)
    torch.cuda.synchronize()
    want = keep[0].clone()
    for r in keep[1:]:
        want ^= r
    for w in written:
        assert torch.equal(w, want)
    for r, k in zip(read, keep):
        assert torch.equal(r, k)


@pytest.mark.parametrize("n", [1, 2, 4, 8])
def test_write_only_and_read_only(B, n):
    words = 32 * 1024 // 4 * 7
    say("probe write-only / read-only", n)
    written = [torch.zeros(words, dtype=torch.int32, device="cuda") for _ in range(n)]
    B.ftar_probe_stream([], written, fill=0x12345678)
    torch.cuda.synchronize()
    for w in written:
        assert bool((w == 0x12345678).all())
    read = _bufs(n, words, 100 + n)
    keep = [r.clone() for r in read]
    B.ftar_probe_stream(read, [])
    torch.cuda.synchronize()
    for r, k in zip(read, keep):
        assert torch.equal(r, k)


def test_mixes_and_sizes_that_are_not_offered(B):
    a = [torch.zeros(32 * 1024 // 4, dtype=torch.int32, device="cuda") for _ in range(6)]
    with pytest.raises(B.FtarError) as e:
        B.ftar_probe_stream(a[:5], a[5:])               # 5 + 1 is not in the list
    assert e.value.status == B.FTAR_ERR_INVALID_ARG
    odd = [torch.zeros(1000, dtype=torch.int32, device="cuda") for _ in range(2)]
    with pytest.raises(B.FtarError) as e:
        B.ftar_probe_stream(odd[:1], odd[1:])           # not a multiple of 32 KiB
    assert e.value.status == B.FTAR_ERR_INVALID_ARG


@pytest.mark.parametrize("n_read", [1, 2, 4, 7, 8, 16])
@pytest.mark.parametrize("period,window", [(4096, 512), (64, 32), (256, 256)])
def test_windowed_probe_writes_the_xor_whatever_the_window(B, n_read, period, window):
    words = 32 * 1024 // 4 * 4 * 300                    # 300 x 128 KiB: several tiles per workgroup, a full stage now and then
    say("windowed probe", n_read, period, window)
    read = _bufs(n_read, words, 200 + n_read)
    keep = [r.clone() for r in read]
    written = torch.zeros(words, dtype=torch.int32, device="cuda")
    B.ftar_probe_stream_windows(read, written, period, window)
    torch.cuda.synchronize()
    want = keep[0].clone()
    for r in keep[1:]:
        want ^= r
    assert torch.equal(written, want)
    for r, k in zip(read, keep):
        assert torch.equal(r, k)
    with pytest.raises(B.FtarError):
        B.ftar_probe_stream_windows(read, written, 1000, 10)      # the period is not a power of two
    if n_read == 1:
        with pytest.raises(B.FtarError):
            B.ftar_probe_stream_windows(read + read + read, written, 4096, 512)   # 3 + 1 is not offered


@pytest.mark.parametrize("n_read", [1, 2])
@pytest.mark.parametrize("threads,per_lane", [(256, 8), (256, 32), (1024, 8)])
@pytest.mark.parametrize("n_workgroups", [1, 2, 7])
def test_few_workgroup_probe_writes_the_xor(B, n_read, threads, per_lane, n_workgroups):
    words = threads * per_lane * 4 * 19               # 19 tiles: uneven over 2 and 7 workgroups
    say("few-workgroup probe", n_read, threads, per_lane, n_workgroups)
    read = _bufs(n_read, words, 300 + n_read)
    keep = [r.clone() for r in read]
    written = torch.zeros(words, dtype=torch.int32, device="cuda")
    if n_read == 2 and per_lane == 32:                # not offered: two streams of 32 vectors do not fit the registers
        with pytest.raises(B.FtarError):
            B.ftar_probe_stream_workgroups(read, written, n_workgroups, threads, per_lane)
        return
    B.ftar_probe_stream_workgroups(read, written, n_workgroups, threads, per_lane)
    torch.cuda.synchronize()
    want = keep[0].clone()
    for r in keep[1:]:
        want ^= r
    assert torch.equal(written, want)
    with pytest.raises(B.FtarError):
        B.ftar_probe_stream_workgroups(read, written, n_workgroups, 512, 8)        # not an offered shape
    with pytest.raises(B.FtarError):
        B.ftar_probe_stream_workgroups([r[:-4] for r in read], written[:-4], n_workgroups, threads, per_lane)   # not whole tiles
