"""Seeded synthetic inputs with the shapes of the five benchmark workloads.

This module only produces INPUTS (random gradient values, live masks, sizes).
It contains none of the reduction's arithmetic and is the one module that both
the HIP-path tests and the CPU-oracle tests may import.

The paper measures its all-reduce on message sizes of 256 MB to 1 GB across 2
to 16 ranks and designs it for 200-500 MB messages and up to 16 ranks (section
4.2 "Ring algorithm", section 6.3); it says nothing about gradient values.  The
value distributions are therefore this build's: N(0, sigma=1e-3), or Student-t
with 3 degrees of freedom scaled by 1e-4 (heavy tails), optionally with a
fraction of exact zeros.  Values are drawn in fp32 with torch's counter-based
generator on the device the data lives on and then rounded to the storage
dtype; whatever bytes come out are handed unchanged to both sides of a parity
test, so differences between host and device generators cannot matter.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

M = 1 << 20

_DRAW_CHUNK = 1 << 26  # elements drawn per generator call (bounds temporary memory)


@dataclass
class Workload:
    name: str
    n_replicas: int
    count: int                 # elements per replica
    dtype: torch.dtype
    dist: str                  # "normal" | "student_t3"
    value_scale: float
    seed: int
    live_mask: int
    chunk_elems: int = 16384
    zero_frac: float = 0.0
    bucket_elems: Optional[int] = None      # bucketed membership only
    bucket_p_live: float = 0.9
    replan_before_step: Optional[int] = None  # ring only: (0-based RS step, replica that leaves)
    replan_leaver: Optional[int] = None
    notes: str = ""

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == torch.float32 else 2

    def scaled(self, count: int) -> "Workload":
        """Same workload at a smaller element count (for tests the oracle finishes quickly)."""
        w = Workload(**self.__dict__)
        w.count = count
        if w.bucket_elems is not None:
            w.bucket_elems = max(1, int(self.bucket_elems * (count / self.count)))
        return w


def configs() -> List[Workload]:
    """The five workloads, in the order the benchmark definition lists them."""
    return [
        Workload("cfg1_4x1M_f32", 4, 1_048_576, torch.float32, "normal", 1e-3, 0, 0b1111,
                 chunk_elems=16384, notes="cache-resident parity case"),
        Workload("cfg2_8x64M_bf16_drop3", 8, 64 * M, torch.bfloat16, "normal", 1e-3, 1,
                 0b11110111, notes="replica 3 dead, single bucket"),
        Workload("cfg3_ring_16x256M_bf16", 16, 256 * M, torch.bfloat16, "student_t3", 1e-4, 2,
                 0xFFFF, replan_before_step=5, replan_leaver=9,
                 notes="ring schedule; replica 9 leaves before RS step 5"),
        Workload("cfg4_8x2e9_bf16", 8, 2_000_000_000, torch.bfloat16, "student_t3", 1e-4, 3,
                 0xFF, zero_frac=1e-3, notes="one GPU's HSDP gradient shard"),
        Workload("cfg5_bucketed_8x512M_f32", 8, 512 * M, torch.float32, "normal", 1e-3, 4,
                 0xFF, bucket_elems=25 * M, notes="per-bucket live masks"),
    ]


def _generator(device, seed: int, replica: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1_000_003 + replica * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    return g


def draw_replica(w: Workload, replica: int, device, count: Optional[int] = None) -> torch.Tensor:
    """One replica's gradient buffer (1-D tensor of w.dtype on `device`)."""
    count = w.count if count is None else count
    g = _generator(device, w.seed, replica)
    out = torch.empty(count, dtype=w.dtype, device=device)
    for lo in range(0, count, _DRAW_CHUNK):
        m = min(_DRAW_CHUNK, count - lo)
        if w.dist == "normal":
            x = torch.randn(m, generator=g, device=device, dtype=torch.float32)
        elif w.dist == "student_t3":
            z = torch.randn(4, m, generator=g, device=device, dtype=torch.float32)
            x = z[0] / torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0)
            del z
        else:
            raise ValueError(w.dist)
        x.mul_(w.value_scale)
        if w.zero_frac > 0.0:
            u = torch.rand(m, generator=g, device=device, dtype=torch.float32)
            x.masked_fill_(u < w.zero_frac, 0.0)
            del u
        out[lo:lo + m] = x.to(w.dtype)
        del x
    return out


def draw_replicas(w: Workload, device, count: Optional[int] = None,
                  poison_dead: bool = True) -> List[torch.Tensor]:
    """All n_replicas buffers.  Dead replicas are filled with NaN so that any read shows."""
    count = w.count if count is None else count
    bufs = []
    for r in range(w.n_replicas):
        if not (w.live_mask >> r) & 1 and poison_dead:
            bufs.append(torch.full((count,), float("nan"), dtype=w.dtype, device=device))
        else:
            bufs.append(draw_replica(w, r, device, count))
    return bufs


def bucket_bounds(count: int, bucket_elems: int) -> List[int]:
    """Bucket boundaries [0, b, 2b, ..., count]."""
    edges = list(range(0, count, bucket_elems)) + [count]
    return edges


def bucket_masks(n_replicas: int, n_buckets: int, p_live: float, seed: int) -> List[int]:
    """Per-bucket live masks: each replica live with probability p_live, independently;
    an empty draw is replaced by the single bit (bucket index mod n_replicas)."""
    rng = np.random.default_rng(seed)
    masks = []
    for b in range(n_buckets):
        bits = rng.random(n_replicas) < p_live
        m = 0
        for r in range(n_replicas):
            if bits[r]:
                m |= 1 << r
        if m == 0:
            m = 1 << (b % n_replicas)
        masks.append(m)
    return masks


def to_numpy_bits(t: torch.Tensor) -> np.ndarray:
    """Host copy of a tensor as numpy: float32 stays float32, bf16 becomes its uint16 bit patterns."""
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    if t.dtype == torch.float32:
        return t.numpy().copy()
    raise TypeError(t.dtype)


def from_numpy_bits(a: np.ndarray, device) -> torch.Tensor:
    """Inverse of to_numpy_bits."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(device)
    if a.dtype == np.float32:
        return torch.from_numpy(a.copy()).to(device)
    raise TypeError(a.dtype)
