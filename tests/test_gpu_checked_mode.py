"""PCCL_CHECK_POINTERS: with it set, a call whose ranges are not inside memory a kernel can
reach is refused on the host (PCCL_ERR_ADDRESS) instead of being launched, and valid calls
give the same bit-exact results as without it.

Every refused call here is first shown to be refused by the stand-alone range test
(pccl_check_device_range, which launches nothing), so no kernel ever sees a bad address."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2504_18658_amd as pccl
from paper_2504_18658_amd import workloads as W
from util import same_bits, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda"
F32, BF16 = torch.float32, torch.bfloat16
OK, ERR_NULL, ERR_INVALID, ERR_ADDRESS = pccl.PCCL_OK, pccl.PCCL_ERR_NULL, pccl.PCCL_ERR_INVALID, pccl.PCCL_ERR_ADDRESS
GIB = 1 << 30


def _sync():
    torch.cuda.synchronize()


def test_range_test_accepts_reachable_memory_and_refuses_the_rest():
    t = torch.zeros(1 << 20, dtype=F32, device=DEV)
    assert pccl.pccl_check_device_range(t) == OK
    assert pccl.pccl_check_device_range(t[123:]) == OK                       # inside an allocation
    assert pccl.pccl_check_device_range(t.data_ptr(), 0) == OK
    assert pccl.pccl_check_device_range(0, 0) == OK
    assert pccl.pccl_check_device_range(0, 16) == ERR_NULL
    big = torch.zeros(64 << 20, dtype=torch.uint8, device=DEV)               # a block of its own
    assert pccl.pccl_check_device_range(big) == OK
    assert pccl.pccl_check_device_range(big.data_ptr(), big.numel() + 64 * GIB) == ERR_ADDRESS
    assert pccl.pccl_check_device_range(big.data_ptr() + big.numel() - 16, 64 * GIB) == ERR_ADDRESS
    host = np.zeros(4096, dtype=np.uint8)                                    # pageable host memory
    assert pccl.pccl_check_device_range(host.ctypes.data, host.size) == ERR_ADDRESS
    assert pccl.pccl_check_device_range(0x1000, 16) == ERR_ADDRESS           # nobody's address
    # a refused query leaves no error behind for the next launch
    src = W.normal(2 * 1000, 1, 1.0, "cpu", F32).view(2, 1000)
    dst = torch.empty(1000, dtype=F32, device=DEV)
    pccl.pccl_local_reduce(dst, src.to(DEV))
    _sync()
    assert same_bits(to_np(dst), oracle.flat_reduce([to_np(src[0]), to_np(src[1])]))


def test_pinned_host_memory_is_reachable():
    pinned = torch.zeros(4096, dtype=F32).pin_memory()
    assert pccl.pccl_check_device_range(pinned.data_ptr(), pinned.numel() * 4) == OK


@pytest.mark.parametrize("level", ["1", "2"])
def test_valid_calls_are_unchanged_in_checked_mode(monkeypatch, level):
    monkeypatch.setenv("PCCL_CHECK_POINTERS", level)
    pccl.diag_reload_env()
    n, g, c = 5, 4, 3000 + 5
    P = n * g
    x_h = W.normal(g * n * c, 5, 1.0, "cpu", BF16).view(g, n, c)
    x = x_h.to(DEV)
    inter_h = W.normal(n * c, 6, 1.0, "cpu", BF16).view(n, c)
    inter = inter_h.to(DEV)
    d_inter = pccl.device_pointer_array([inter[k] for k in range(n)])
    shard, partial = torch.empty(c, dtype=BF16, device=DEV), torch.empty(n * c, dtype=BF16, device=DEV)
    pccl.pccl_reduce_scatter_local(shard, partial, x, d_inter=d_inter, my_node=2, average=True)
    _sync()
    ws, wp = oracle.reduce_scatter_local(to_np(x_h), my_node=2, inter=[to_np(inter_h[k]) for k in range(n)], average=True)
    assert same_bits(to_np(shard), ws) and same_bits(to_np(partial), wp.reshape(-1))

    msgs_h = W.normal(g * P * c, 7, 1.0, "cpu", BF16).view(g, P * c)
    msgs = msgs_h.to(DEV)
    pccl.pccl_reduce_scatter_local_unpacked(shard, partial, msgs=msgs, nodes=n, gpus_per_node=g, my_gpu=1)
    _sync()
    ws, wp = oracle.reduce_scatter_local_unpacked([to_np(msgs_h[k]) for k in range(g)], n, g, 1)
    assert same_bits(to_np(shard), ws) and same_bits(to_np(partial), wp.reshape(-1))

    msg = msgs[0]
    packed, back = torch.empty_like(msg), torch.empty_like(msg)
    pccl.pccl_hier_pack(packed, msg, n, g)
    pccl.pccl_hier_unpack(back, packed, n, g)
    slots = pccl.device_pointer_array([packed.view(P, c)[k] for k in range(P)])
    viaslots = torch.empty_like(msg)
    pccl.pccl_allgather_reassemble(viaslots, d_slots=slots, nodes=n, gpus_per_node=g)
    _sync()
    assert same_bits(to_np(packed), oracle.hier_pack(to_np(msgs_h[0]), n, g).view(np.uint16))
    assert torch.equal(back.view(torch.int16), msg.view(torch.int16))
    assert torch.equal(viaslots.view(torch.int16), msg.view(torch.int16))

    srcs_h = W.normal(P * 777, 8, 1.0, "cpu", F32).view(P, 777)
    srcs = srcs_h.to(DEV)
    ptrs = pccl.device_pointer_array([srcs[k] for k in range(P)])
    out = torch.empty(777, dtype=F32, device=DEV)
    pccl.pccl_local_reduce_ptrs(out, ptrs, 777, F32)
    _sync()
    assert same_bits(to_np(out), oracle.flat_reduce([to_np(srcs_h[k]) for k in range(P)]))
    pccl.pccl_local_reduce_ptrs_two_level(out, ptrs, n, g, 777, F32)
    _sync()
    assert same_bits(to_np(out), oracle.two_level_reduce([to_np(srcs_h[k]) for k in range(P)], n, g))

    s1, p1 = torch.empty(c, dtype=BF16, device=DEV), torch.empty(n * c, dtype=BF16, device=DEV)
    table = pccl.BucketTable([(s1, p1, x), (shard, partial, x)])
    pccl.pccl_reduce_scatter_local_batched(table)
    ptable = pccl.PermuteTable([(packed, msg), (back, msgs[1])], n, g)
    pccl.pccl_hier_pack_batched(ptable)
    _sync()
    ws, wp = oracle.reduce_scatter_local(to_np(x_h))
    assert same_bits(to_np(s1), ws) and same_bits(to_np(p1), wp.reshape(-1))
    assert same_bits(to_np(back), oracle.hier_pack(to_np(msgs_h[1]), n, g).view(np.uint16))

    s3, p3 = torch.empty(c, dtype=BF16, device=DEV), torch.empty(n * c, dtype=BF16, device=DEV)
    mtable = pccl.BucketTable([(s3, p3, msgs)], nodes=n)
    pccl.pccl_reduce_scatter_local_unpacked_batched(mtable, 1)
    _sync()
    ws, wp = oracle.reduce_scatter_local_unpacked([to_np(msgs_h[k]) for k in range(g)], n, g, 1)
    assert same_bits(to_np(s3), ws) and same_bits(to_np(p3), wp.reshape(-1))

    ring_h = W.normal(4 * c, 9, 1.0, "cpu", BF16).view(4, c)
    recv_h = W.normal(3 * c, 10, 1.0, "cpu", BF16).view(3, c)
    ring = ring_h.to(DEV)
    pccl.pccl_ring_reduce_scatter_local(ring, recv_h.to(DEV), 1)
    halv = ring_h.to(DEV)
    pccl.pccl_halving_reduce_scatter_local(halv, recv_h.to(DEV).view(-1), 1)
    acc = ring_h[0].to(DEV)
    pccl.pccl_accumulate(acc, ring_h[1].to(DEV))
    _sync()
    assert same_bits(to_np(acc), oracle.accumulate(to_np(ring_h[0]), to_np(ring_h[1])))
    want_ring = oracle.ring_rs_local(to_np(ring_h), [to_np(recv_h[k]) for k in range(3)], 1)
    assert same_bits(to_np(ring), want_ring)
    want_halv = oracle.halving_rs_local(to_np(ring_h), [to_np(recv_h[0:2]), to_np(recv_h[2:3])], 1)
    assert same_bits(to_np(halv), want_halv)


def test_a_call_with_an_unreachable_range_is_refused_not_launched(monkeypatch):
    monkeypatch.setenv("PCCL_CHECK_POINTERS", "1")
    pccl.diag_reload_env()
    L = pccl.lib()
    n = 4096
    host = np.ones(2 * n, dtype=np.float32)                      # pageable host memory as the source
    dst = torch.full((n,), 7.0, dtype=F32, device=DEV)
    assert pccl.pccl_check_device_range(host.ctypes.data, host.nbytes) == ERR_ADDRESS   # shown first
    rc = L.pccl_local_reduce(dst.data_ptr(), host.ctypes.data, n * 4, 2, n, pccl.PCCL_F32, pccl.PCCL_F32,
                             pccl.PCCL_SUM, None)
    assert rc == ERR_ADDRESS
    assert "ADDRESS" in pccl.status_string(rc)
    rc = L.pccl_accumulate(dst.data_ptr(), host.ctypes.data, n, pccl.PCCL_F32, pccl.PCCL_SUM, None)
    assert rc == ERR_ADDRESS
    rc = L.pccl_hier_pack(dst.data_ptr(), host.ctypes.data, 4, 2, n * 4 // 8, None)
    assert rc == ERR_ADDRESS
    # a source range longer than the block that holds it: two 64 MB blocks, the source in the
    # higher one so that its overrun points away from the destination
    torch.cuda.empty_cache()                                     # so that each tensor is a fresh block
    a = torch.zeros(64 << 20, dtype=torch.uint8, device=DEV)
    b = torch.zeros(64 << 20, dtype=torch.uint8, device=DEV)
    lo, hi = (a, b) if a.data_ptr() < b.data_ptr() else (b, a)
    count = (48 << 20) // 4                                      # two sources of 48 MB = 96 MB claimed
    assert pccl.pccl_check_device_range(hi.data_ptr(), 2 * count * 4) == ERR_ADDRESS            # shown first
    assert pccl.pccl_check_device_range(lo.data_ptr(), count * 4) == OK
    rc = L.pccl_local_reduce(lo.data_ptr(), hi.data_ptr(), count * 4, 2, count, pccl.PCCL_F32, pccl.PCCL_F32,
                             pccl.PCCL_SUM, None)
    assert rc == ERR_ADDRESS
    _sync()
    assert bool((dst == 7.0).all()) and bool((lo == 0).all())


def test_level_two_looks_inside_device_tables(monkeypatch):
    L = pccl.lib()
    n = 1024
    srcs = torch.ones(4, n, dtype=F32, device=DEV)
    host = np.ones(n, dtype=np.float32)
    assert pccl.pccl_check_device_range(host.ctypes.data, host.nbytes) == ERR_ADDRESS            # shown first
    good = [srcs[k].data_ptr() for k in range(4)]
    bad = torch.tensor(good[:3] + [host.ctypes.data], dtype=torch.int64, device=DEV)
    dst = torch.full((n,), 7.0, dtype=F32, device=DEV)
    monkeypatch.setenv("PCCL_CHECK_POINTERS", "2")
    pccl.diag_reload_env()
    rc = L.pccl_local_reduce_ptrs(dst.data_ptr(), bad.data_ptr(), 4, n, pccl.PCCL_F32, pccl.PCCL_F32, pccl.PCCL_SUM, None)
    assert rc == ERR_ADDRESS
    # the slot of the caller's own node is never dereferenced, so it may hold anything
    inter = pccl.device_pointer_array([srcs[0], srcs[1]])
    inter_bad_own = torch.tensor([good[0], host.ctypes.data], dtype=torch.int64, device=DEV)
    x = torch.ones(2, 2, n, dtype=F32, device=DEV)
    shard, partial = torch.empty(n, dtype=F32, device=DEV), torch.empty(2 * n, dtype=F32, device=DEV)
    rc = L.pccl_reduce_scatter_local(shard.data_ptr(), partial.data_ptr(), x.data_ptr(), 2 * n * 4, inter_bad_own.data_ptr(),
                                     2, 2, 1, n, pccl.PCCL_F32, pccl.PCCL_SUM, None)
    assert rc == OK
    _sync()
    assert bool((shard == 3.0).all())                            # srcs[0] (ones) + partial[1] (1 + 1)
    rc = L.pccl_reduce_scatter_local(shard.data_ptr(), partial.data_ptr(), x.data_ptr(), 2 * n * 4, inter_bad_own.data_ptr(),
                                     2, 2, 0, n, pccl.PCCL_F32, pccl.PCCL_SUM, None)
    assert rc == ERR_ADDRESS                                     # as node 0 the bad slot 1 would be read
    del inter
    # a descriptor table whose device copy differs from its host mirror
    s1, p1 = torch.empty(n, dtype=F32, device=DEV), torch.empty(2 * n, dtype=F32, device=DEV)
    table = pccl.BucketTable([(s1, p1, x)])
    table.device[32] ^= 1                                        # chunk_count on the device only
    _sync()
    rc = L.pccl_reduce_scatter_local_batched(table.device.data_ptr(), ctypes.addressof(table.host), 1, 2, 2,
                                             pccl.PCCL_F32, pccl.PCCL_SUM, None)
    assert rc == ERR_INVALID
    _sync()
    assert bool((dst == 7.0).all())
