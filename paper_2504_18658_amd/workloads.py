"""Seeded synthetic inputs for the five workloads (shapes only, no method arithmetic).

The paper benchmarks its collectives on randomly initialised GPU tensors
(artifact appendix) at 16 MB - 1 GB messages and 32 - 2048 ranks (Section V-A);
these generators stand in for that: same shapes, seeded values.  Both the HIP
path and the CPU oracle consume the bytes produced here; nothing in this
module adds, rounds-for-the-method or permutes anything the method computes.
bf16 values are made with torch's own float32 -> bfloat16 cast.

Every generator takes `device`; a torch.Generator on that device is seeded with
the workload's seed, so a given (seed, device type) always yields the same bytes.
"""
import math
from dataclasses import dataclass, field

import torch

MB = 1 << 20


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def uniform_pm1(n, seed, device="cpu", dtype=torch.float32):
    """n values uniform in [-1, 1) drawn in fp32, cast to dtype."""
    x = torch.rand(n, generator=_gen(seed, device), device=device, dtype=torch.float32)
    x = x.mul_(2.0).sub_(1.0)
    return x if dtype == torch.float32 else x.to(dtype)


def normal(n, seed, std=1.0, device="cpu", dtype=torch.float32):
    """n values ~ N(0, std^2) drawn in fp32, cast to dtype."""
    x = torch.randn(n, generator=_gen(seed, device), device=device, dtype=torch.float32)
    if std != 1.0:
        x = x.mul_(std)
    return x if dtype == torch.float32 else x.to(dtype)


def random_bits16(n, seed, device="cpu"):
    """n random 16-bit patterns (every bf16 encoding, NaN and inf included), as bfloat16."""
    x = torch.randint(-32768, 32768, (n,), generator=_gen(seed, device), device=device,
                      dtype=torch.int16)
    return x.view(torch.bfloat16)


def small_integers(n, seed, device="cpu", dtype=torch.float32, lo=-8, hi=9):
    """Integers in [lo, hi): exact in bf16 and fp32, so every summation order agrees."""
    x = torch.randint(lo, hi, (n,), generator=_gen(seed, device), device=device, dtype=torch.int32)
    return x.to(dtype)


def bucket_sizes_bytes(seed=4, nbuckets=40, lo=16 * MB, ratio=32.0, quantum=1024):
    """Log-uniform bucket sizes in [lo, lo*ratio), rounded down to a multiple of quantum bytes."""
    u = torch.rand(nbuckets, generator=_gen(seed, "cpu"), dtype=torch.float64)
    return [int(math.floor(lo * (ratio ** float(v)) / quantum)) * quantum for v in u]


@dataclass
class Workload:
    name: str
    nodes: int
    gpus: int
    dtype: torch.dtype
    chunk: int  # elements per rank-chunk
    seed: int
    dist: str
    extra: dict = field(default_factory=dict)

    @property
    def ranks(self):
        return self.nodes * self.gpus

    @property
    def esize(self):
        return 4 if self.dtype == torch.float32 else 2


# The five workloads at full size.  `chunk` can be overridden for small parity cases.
def cfg1(chunk=131072):
    """Flat reduce-scatter local reduction: 8 ranks, fp32 chunks of 512 KB, uniform[-1,1), seed 0."""
    return Workload("cfg1_flat_reduce_p8_f32", 1, 8, torch.float32, chunk, 0, "uniform")


def cfg2(chunk=1048576):
    """Hierarchical all-gather reassembly: 4 x 8 ranks, 64 MB bf16 message, random bits, seed 1."""
    return Workload("cfg2_allgather_4x8_bf16_64MB", 4, 8, torch.bfloat16, chunk, 1, "bits")


def cfg3(chunk=1048576):
    """Two-level reduce-scatter share: 16 x 8 ranks, 256 MB bf16 message, uniform[-1,1), seed 2."""
    return Workload("cfg3_two_level_rs_16x8_bf16_256MB", 16, 8, torch.bfloat16, chunk, 2, "uniform")


def cfg4(chunk=16384, nodes=256):
    """All-reduce share at 256 x 8 ranks: 128 MB fp32, 2048 chunks of 64 KB, N(0,1), seed 3."""
    return Workload("cfg4_allreduce_256x8_f32_128MB", nodes, 8, torch.float32, chunk, 3, "normal")


def cfg5(scale=1.0, nbuckets=40):
    """ZeRO-3-shaped gradient buckets: 40 reduce-scatters over 8 x 8 ranks, bf16 ~ N(0, 1e-3), seed 4.
    scale < 1 shrinks every bucket (kept a multiple of 1024 bytes) for small parity cases."""
    sizes = bucket_sizes_bytes(4, nbuckets)
    sizes = [max(1024, int(s * scale) // 1024 * 1024) for s in sizes]
    w = Workload("cfg5_zero3_buckets_8x8_bf16", 8, 8, torch.bfloat16, 0, 4, "normal1e-3")
    w.extra["bucket_bytes"] = sizes
    return w


def draw(w, n, device="cpu", seed_offset=0):
    """n elements of workload w's value distribution and dtype."""
    seed = w.seed + 1000 * seed_offset
    if w.dist == "uniform":
        return uniform_pm1(n, seed, device, w.dtype)
    if w.dist == "normal":
        return normal(n, seed, 1.0, device, w.dtype)
    if w.dist == "normal1e-3":
        return normal(n, seed, 1e-3, device, w.dtype)
    if w.dist == "bits":
        return random_bits16(n, seed, device)
    raise ValueError(w.dist)


def two_level_input(w, device="cpu", seed_offset=0, chunk=None):
    """x[gpus][nodes][chunk]: piece g = what node-mate g sent (chunks bound for every node)."""
    c = w.chunk if chunk is None else chunk
    return draw(w, w.gpus * w.nodes * c, device, seed_offset).view(w.gpus, w.nodes, c)


def shuffled_slot_order(nslots, seed):
    """A permutation of arena slots, so that a pointer array built from it is not monotone."""
    return torch.randperm(nslots, generator=_gen(seed, "cpu")).tolist()
