"""Shared helpers for the tests: torch <-> numpy views and guarded device buffers."""
import numpy as np
import torch


def to_np(t):
    """Device/host tensor -> numpy array the oracle accepts (bf16 as uint16 bit patterns)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def same_bits(a, b):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    return a.dtype == b.dtype and a.size == b.size and a.tobytes() == b.tobytes()


def first_diff(a, b):
    a = np.ascontiguousarray(a).reshape(-1)
    b = np.ascontiguousarray(b).reshape(-1)
    av = a.view(np.uint16 if a.itemsize == 2 else np.uint32 if a.itemsize == 4 else np.uint8)
    bv = b.view(av.dtype)
    idx = np.flatnonzero(av != bv)
    if idx.size == 0:
        return "identical"
    i = int(idx[0])
    return "%d of %d differ; first at %d: got %r want %r" % (idx.size, av.size, i, a[i], b[i])


class Guarded:
    """A device buffer of `numel` elements with poisoned guard bands on both sides.

    `view` is the usable tensor (optionally shifted by `offset_elems` to break 16-byte
    alignment); check() asserts the guards were not written."""

    GUARD = 64  # elements

    def __init__(self, numel, dtype, device="cuda", offset_elems=0):
        self.dtype = dtype
        self.numel = numel
        self.lo = self.GUARD + offset_elems
        total = self.lo + numel + self.GUARD
        narrow = dtype in (torch.bfloat16, torch.float16)
        int_dt = torch.int16 if narrow else torch.int32
        self.poison = 0x7FC1 if narrow else 0x7FC12345   # a NaN in every one of the three formats
        raw = torch.full((total,), self.poison, dtype=int_dt, device=device)
        self.raw = raw
        self.view = raw.view(dtype)[self.lo:self.lo + numel]

    def check(self):
        r = self.raw.cpu()
        assert bool((r[:self.lo] == self.poison).all()), "write below the output buffer"
        assert bool((r[self.lo + self.numel:] == self.poison).all()), "write above the output buffer"
