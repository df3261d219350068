"""Buffers beyond 4 GiB: every byte offset the kernels form must be 64-bit.  At these sizes the
oracle checks sampled windows (it computes them one by one); a property that holds at any size
-- equality with torch's own element-wise IEEE arithmetic, or chunk-by-chunk byte equality --
covers every element on the GPU."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2504_18658_amd as pccl
from util import same_bits, to_np

pytestmark = pytest.mark.gpu

DEV = "cuda"
F32, BF16 = torch.float32, torch.bfloat16
G4 = 1 << 32


def _sync():
    torch.cuda.synchronize()


@pytest.fixture(autouse=True)
def _free_between_tests():
    yield
    torch.cuda.empty_cache()


def _rand(n, dtype, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    x = torch.empty(n, dtype=dtype, device=DEV)
    x.uniform_(-1.0, 1.0, generator=g)
    return x


def _windows(n, width=4096):
    """Head, the elements either side of every 4 GiB byte boundary is covered by the caller's
    choice of n; here: head, middle, tail."""
    return [0, n // 2 - width // 2, n - width]


def test_local_reduce_fp32_beyond_4gib():
    n = (1 << 30) + 4099                                   # 4 GiB + 16 KiB of fp32 per source, ragged tail
    src = _rand(2 * n, F32, 1).view(2, n)
    dst = torch.empty(n, dtype=F32, device=DEV)
    pccl.pccl_local_reduce(dst, src)
    _sync()
    assert torch.equal(dst.view(torch.int32), (src[0] + src[1]).view(torch.int32))
    for lo in _windows(n) + [(1 << 30) - 2048]:
        sl = slice(lo, lo + 4096)
        assert same_bits(to_np(dst[sl]), oracle.flat_reduce([to_np(src[0][sl]), to_np(src[1][sl])]))


def test_local_reduce_bf16_three_sources_beyond_4gib():
    n = (1 << 31) + 11                                     # 4 GiB of bf16 per source + a ragged tail
    src = _rand(3 * n, BF16, 2).view(3, n)
    dst = torch.empty(n, dtype=BF16, device=DEV)
    pccl.pccl_local_reduce(dst, src)
    _sync()
    step = 1 << 28
    for lo in range(0, n, step):                           # torch's fp32 adds and bf16 cast, piecewise
        sl = slice(lo, min(n, lo + step))
        ref = ((src[0][sl].float() + src[1][sl].float()) + src[2][sl].float()).to(BF16)
        assert torch.equal(dst[sl].view(torch.int16), ref.view(torch.int16)), lo
    for lo in _windows(n) + [(1 << 31) - 2048]:
        sl = slice(lo, lo + 4096)
        assert same_bits(to_np(dst[sl]), oracle.flat_reduce([to_np(src[k][sl]) for k in range(3)]))


def test_two_level_lds_kernel_beyond_4gib():
    n = (1 << 30) + 5
    nodes, gpus = 2, 2
    src = _rand(nodes * gpus * n, F32, 3).view(nodes * gpus, n)
    ptrs = pccl.device_pointer_array([src[k] for k in range(nodes * gpus)])
    dst = torch.empty(n, dtype=F32, device=DEV)
    os.environ["PCCL_FORCE_TWO_LEVEL_KERNEL"] = "lds"
    pccl.diag_reload_env()
    try:
        pccl.pccl_local_reduce_ptrs_two_level(dst, ptrs, nodes, gpus, n, F32)
        _sync()
    finally:
        os.environ.pop("PCCL_FORCE_TWO_LEVEL_KERNEL", None)
        pccl.diag_reload_env()
    assert torch.equal(dst.view(torch.int32), ((src[0] + src[1]) + (src[2] + src[3])).view(torch.int32))
    for lo in _windows(n) + [(1 << 30) - 2048]:
        sl = slice(lo, lo + 4096)
        want = oracle.two_level_reduce([to_np(src[k][sl]) for k in range(4)], nodes, gpus)
        assert same_bits(to_np(dst[sl]), want)


def test_accumulate_bf16_beyond_4gib():
    n = (1 << 31) + 9
    acc = _rand(n, BF16, 4)
    recv = _rand(n, BF16, 5)
    before = acc.clone()
    pccl.pccl_accumulate(acc, recv)
    _sync()
    step = 1 << 28
    for lo in range(0, n, step):
        sl = slice(lo, min(n, lo + step))
        assert torch.equal(acc[sl].view(torch.int16), (before[sl] + recv[sl]).view(torch.int16)), lo
    for lo in _windows(n) + [(1 << 31) - 2048]:
        sl = slice(lo, lo + 4096)
        assert same_bits(to_np(acc[sl]), oracle.accumulate(to_np(before[sl]), to_np(recv[sl])))


def test_pack_and_unpack_chunks_beyond_4gib():
    nodes, gpus = 2, 2
    cb = G4 + 48                                           # bytes per chunk: tiles, offsets and strides > 2^32
    g = torch.Generator(device=DEV)
    g.manual_seed(6)
    src = torch.randint(0, 256, (nodes * gpus * cb,), generator=g, device=DEV, dtype=torch.uint8)
    dst = torch.empty_like(src)
    pccl.pccl_hier_pack(dst, src, nodes, gpus)
    _sync()
    s, d = src.view(nodes, gpus, cb), dst.view(gpus, nodes, cb)
    for n in range(nodes):
        for k in range(gpus):
            assert torch.equal(d[k, n], s[n, k]), (n, k)   # the definition, chunk by chunk
    # the oracle on windows: a small message made of the same window of every chunk
    for off in (0, cb // 2, cb - 4096):                    # the last window straddles the 4 GiB offset
        mini = np.stack([to_np(s[n, k, off:off + 4096]) for n in range(nodes) for k in range(gpus)])
        want = oracle.hier_pack(mini.reshape(-1), nodes, gpus).reshape(gpus, nodes, 4096)
        got = np.stack([to_np(d[k, n, off:off + 4096]) for k in range(gpus) for n in range(nodes)])
        assert same_bits(got.reshape(gpus, nodes, 4096), want)
    back = torch.empty_like(src)
    pccl.pccl_hier_unpack(back, dst, nodes, gpus)
    _sync()
    assert torch.equal(back, src)                          # round trip = identity


def test_one_launch_share_beyond_4gib():
    """pccl_reduce_scatter_local with received chunks (both phases in one launch): 2 x 2 ranks with
    2 GiB + 16 B chunks, so pieces, partial rows and the own row's offsets pass 2^32 bytes."""
    nodes, gpus, my_node = 2, 2, 1
    c = (1 << 30) + 8                                      # bf16 elements per chunk
    x = _rand(gpus * nodes * c, BF16, 41).view(gpus, nodes, c)
    inter = _rand(nodes * c, BF16, 42).view(nodes, c)
    d_inter = pccl.device_pointer_array([inter[n] for n in range(nodes)])
    shard = torch.empty(c, dtype=BF16, device=DEV)
    partial = torch.empty(nodes * c, dtype=BF16, device=DEV)
    pccl.pccl_reduce_scatter_local(shard, partial, x, d_inter=d_inter, my_node=my_node)
    _sync()
    ref_partial = (x[0].float() + x[1].float()).to(BF16)   # two pieces: one add, one rounding
    assert torch.equal(partial.view(torch.int16), ref_partial.view(torch.int16).reshape(-1))
    ref_shard = (inter[0].float() + ref_partial[1].float()).to(BF16)
    assert torch.equal(shard.view(torch.int16), ref_shard.view(torch.int16))
    del ref_partial, ref_shard
    for lo in (0, c // 2, c - 4096):
        sl = slice(lo, lo + 4096)
        want_s, want_p = oracle.reduce_scatter_local(to_np(x[:, :, sl]), my_node=my_node,
                                                     inter=[to_np(inter[n, sl]) for n in range(nodes)])
        assert same_bits(to_np(shard[sl]), want_s)
        assert same_bits(to_np(partial.view(nodes, c)[:, sl]), want_p)


def test_one_launch_share_from_rank_order_messages_beyond_4gib():
    """pccl_reduce_scatter_local_unpacked with received chunks (both phases in one launch over the rows
    of rank-order messages): 2 x 2 ranks with 2 GiB + 16 B chunks, so rows, messages and the own row's
    offsets pass 2^32 bytes."""
    nodes, gpus, my_node, my_gpu = 2, 2, 1, 1
    c = (1 << 30) + 8                                      # bf16 elements per chunk
    msgs = _rand(gpus * nodes * gpus * c, BF16, 43).view(gpus, nodes, gpus, c)   # [message][node][gpu][chunk]
    inter = _rand(nodes * c, BF16, 44).view(nodes, c)
    d_inter = pccl.device_pointer_array([inter[n] for n in range(nodes)])
    shard = torch.empty(c, dtype=BF16, device=DEV)
    partial = torch.empty(nodes * c, dtype=BF16, device=DEV)
    pccl.pccl_reduce_scatter_local_unpacked(shard, partial, msgs=msgs.view(gpus, nodes * gpus * c), d_inter=d_inter,
                                            nodes=nodes, gpus_per_node=gpus, my_node=my_node, my_gpu=my_gpu)
    _sync()
    pieces = msgs[:, :, my_gpu, :]                          # [message][node][chunk]
    ref_partial = (pieces[0].float() + pieces[1].float()).to(BF16)
    assert torch.equal(partial.view(torch.int16), ref_partial.view(torch.int16).reshape(-1))
    ref_shard = (inter[0].float() + ref_partial[1].float()).to(BF16)
    assert torch.equal(shard.view(torch.int16), ref_shard.view(torch.int16))
    del ref_partial, ref_shard
    for lo in (0, c // 2, c - 4096):
        sl = slice(lo, lo + 4096)
        want_s, want_p = oracle.reduce_scatter_local(to_np(pieces[:, :, sl]), my_node=my_node,
                                                     inter=[to_np(inter[n, sl]) for n in range(nodes)])
        assert same_bits(to_np(shard[sl]), want_s)
        assert same_bits(to_np(partial.view(nodes, c)[:, sl]), want_p)


def test_fused_tail_chunks_beyond_4gib():
    """pccl_phase2_reassemble_local with 4 GiB + 48 B chunks: tile indices, chunk offsets and the own
    chunk's reduction all beyond 2^32 bytes."""
    nodes, gpus, my_node, my_gpu = 2, 2, 1, 0
    c = (1 << 31) + 24                                     # bf16 elements per chunk
    partial = _rand(nodes * c, BF16, 21).view(nodes, c)
    gathered = _rand(nodes * gpus * c, BF16, 22)
    out = torch.empty_like(gathered)
    pccl.pccl_phase2_reassemble_local(out, partial.view(-1), src=gathered, nodes=nodes, gpus_per_node=gpus,
                                      my_node=my_node, my_gpu=my_gpu)
    _sync()
    o, gsrc = out.view(nodes, gpus, c), gathered.view(gpus, nodes, c)
    for n in range(nodes):
        for k in range(gpus):
            if (n, k) == (my_node, my_gpu):
                want = (partial[0].float() + partial[1].float()).to(BF16)     # two terms: one add, one rounding
                step = 1 << 28
                for lo in range(0, c, step):
                    sl = slice(lo, min(c, lo + step))
                    assert torch.equal(o[n, k, sl].view(torch.int16), want[sl].view(torch.int16)), lo
                del want
            else:
                assert torch.equal(o[n, k], gsrc[k, n]), (n, k)
    for lo in (0, c // 2, c - 4096):                       # the oracle on windows of the own chunk
        sl = slice(lo, lo + 4096)
        want = oracle.rs_phase2([to_np(partial[0, sl]), to_np(partial[1, sl])])
        assert same_bits(to_np(o[my_node, my_gpu, sl]), want)


def test_ring_and_halving_one_launch_beyond_4gib():
    """Four ranks with 1 GiB + 16 B chunks: the message and the received buffers are 4 GiB and more,
    so row and chunk offsets of the one-launch replays pass 2^32 bytes."""
    p, c = 4, (1 << 29) + 8                                # bf16 elements per chunk
    msg0 = _rand(p * c, BF16, 31).view(p, c)
    recv = _rand((p - 1) * c, BF16, 32).view(p - 1, c)
    rank = 2
    msg = msg0.clone()
    pccl.pccl_ring_reduce_scatter_local(msg, recv, rank)
    _sync()
    for s_ in range(p - 1):
        ch = (rank - 2 - s_) % p
        assert torch.equal(msg[ch].view(torch.int16), (msg0[ch] + recv[s_]).view(torch.int16)), s_
    assert torch.equal(msg[(rank - 1) % p], msg0[(rank - 1) % p])             # the one chunk no step touches
    for lo in (0, c - 4096):
        sl = slice(lo, lo + 4096)
        want = oracle.ring_rs_local(to_np(msg0[:, sl]), [to_np(recv[s_, sl]) for s_ in range(p - 1)], rank)
        assert same_bits(to_np(msg[:, sl]), want)
    msg = msg0.clone()
    pccl.pccl_halving_reduce_scatter_local(msg, recv.view(-1), rank)
    _sync()
    flat = recv.view(-1)
    # rank 2 keeps chunks 2..3 at step 0 (adds the first received half), then chunk 2 (adds the last chunk)
    first = (msg0[2:4].reshape(-1) + flat[: 2 * c]).view(2, c)
    assert torch.equal(msg[3].view(torch.int16), first[1].view(torch.int16))
    assert torch.equal(msg[2].view(torch.int16), (first[0] + flat[2 * c:]).view(torch.int16))
    assert torch.equal(msg[:2], msg0[:2])
    for lo in (0, c - 4096):
        sl = slice(lo, lo + 4096)
        halves = [to_np(torch.stack([flat[lo:lo + 4096], flat[c + lo:c + lo + 4096]])), to_np(flat[2 * c + lo:2 * c + lo + 4096])]
        want = oracle.halving_rs_local(to_np(msg0[:, sl]), halves, rank)
        assert same_bits(to_np(msg[:, sl]), want)


@pytest.fixture
def tiny_grid_x(monkeypatch):
    """Lower the x extent of a launch to 4096 work-items so that small problems take the
    x/z-split path that buffers of tens of GiB take."""
    monkeypatch.setenv("PCCL_GRID_X_LIMIT", "4096")
    pccl.diag_reload_env()


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_split_grids_on_small_problems(tiny_grid_x, dtype):
    from paper_2504_18658_amd import workloads as W
    from util import Guarded
    import oracle as O
    odt = {F32: O.F32, BF16: O.BF16}[dtype]
    # streaming reduce: 8 sources, 100003 elements -> hundreds of tiles over x and z, ragged tail
    count = 100003
    host = W.normal(8 * count, 1, 1.0, "cpu", dtype).view(8, count)
    dst = Guarded(count, dtype)
    pccl.pccl_local_reduce(dst.view, host.to(DEV))
    _sync()
    assert same_bits(to_np(dst.view), O.flat_reduce([to_np(host[s]) for s in range(8)]))
    dst.check()
    # LDS two-level kernel
    nodes, gpus, cnt = 20, 4, 5000 + 3
    h2 = W.normal(nodes * gpus * cnt, 2, 1.0, "cpu", dtype).view(nodes * gpus, cnt)
    d2 = h2.to(DEV)
    out = Guarded(cnt, dtype)
    os.environ["PCCL_FORCE_TWO_LEVEL_KERNEL"] = "lds"
    pccl.diag_reload_env()
    try:
        pccl.pccl_local_reduce_ptrs_two_level(out.view, pccl.device_pointer_array([d2[k] for k in range(nodes * gpus)]),
                                              nodes, gpus, cnt, dtype)
        _sync()
    finally:
        os.environ.pop("PCCL_FORCE_TWO_LEVEL_KERNEL", None)
        pccl.diag_reload_env()
    assert same_bits(to_np(out.view), O.two_level_reduce([to_np(h2[k]) for k in range(nodes * gpus)], nodes, gpus, odt))
    out.check()
    # accumulate
    a_h, r_h = W.normal(count, 3, 1.0, "cpu", dtype), W.normal(count, 4, 1.0, "cpu", dtype)
    acc = Guarded(count, dtype)
    acc.view.copy_(a_h.to(DEV))
    pccl.pccl_accumulate(acc.view, r_h.to(DEV))
    _sync()
    assert same_bits(to_np(acc.view), O.accumulate(to_np(a_h), to_np(r_h)))
    acc.check()
    # reduce-scatter share (rows) and the batched form (three buckets, one empty)
    n, g, c = 5, 4, 3000 + 5
    x_h = W.normal(g * n * c, 5, 1.0, "cpu", dtype).view(g, n, c)
    x = x_h.to(DEV)
    ws, wp = O.reduce_scatter_local(to_np(x_h))
    s1, p1 = Guarded(c, dtype), Guarded(n * c, dtype)
    s2, p2 = Guarded(c, dtype), Guarded(n * c, dtype)
    empty = torch.empty(g, n, 0, dtype=dtype, device=DEV)
    table = pccl.BucketTable([(s1.view, p1.view, x), (torch.empty(0, dtype=dtype, device=DEV),
                                                      torch.empty(0, dtype=dtype, device=DEV), empty),
                              (s2.view, p2.view, x)])
    pccl.pccl_reduce_scatter_local_batched(table)
    _sync()
    for s_, p_ in ((s1, p1), (s2, p2)):
        assert same_bits(to_np(s_.view), ws) and same_bits(to_np(p_.view), wp.reshape(-1))
        s_.check()
        p_.check()
    P = n * g
    msgs_h = W.normal(g * P * c, 6, 1.0, "cpu", dtype).view(g, P * c)
    pccl.pccl_reduce_scatter_local_unpacked(s1.view, p1.view, msgs=msgs_h.to(DEV), nodes=n, gpus_per_node=g, my_gpu=2)
    _sync()
    ws, wp = O.reduce_scatter_local_unpacked([to_np(msgs_h[k]) for k in range(g)], n, g, 2)
    assert same_bits(to_np(s1.view), ws) and same_bits(to_np(p1.view), wp.reshape(-1))
    s1.check()
    p1.check()


def test_streaming_reduce_with_more_tiles_than_one_grid_dimension_holds():
    """8 fp32 sources of 2^31 + 3 elements (8 GiB each): one element per thread, so the launch has
    more than 2^31 work-items and spreads over x and z without any test knob."""
    n = (1 << 31) + 3
    src = torch.empty(8, n, dtype=F32, device=DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(7)
    step = 1 << 28
    for k in range(8):
        for lo in range(0, n, step):
            src[k, lo:lo + step].uniform_(-1.0, 1.0, generator=g)
    dst = torch.empty(n, dtype=F32, device=DEV)
    pccl.pccl_local_reduce(dst, src)
    _sync()
    for lo in range(0, n, step):
        sl = slice(lo, min(n, lo + step))
        ref = src[0][sl].clone()
        for k in range(1, 8):
            ref += src[k][sl]
        assert torch.equal(dst[sl].view(torch.int32), ref.view(torch.int32)), lo
    for lo in (0, (1 << 31) - 2048, n - 4096):
        sl = slice(lo, lo + 4096)
        assert same_bits(to_np(dst[sl]), oracle.flat_reduce([to_np(src[k][sl]) for k in range(8)]))
