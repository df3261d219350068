"""Seeded random shapes through every reduction and shuffle entry point, against the oracle bit
for bit: node and GPU counts that are not powers of two, ragged element counts, one-element
misalignment of sources and outputs, strided and pointer-array forms, sum and average.  The
draws are deterministic (the seed is the test id), so a failure names its case."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_18658_amd as pccl
from paper_2504_18658_amd import workloads as W
from util import Guarded, first_diff, same_bits, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda"
F32, BF16, F16 = torch.float32, torch.bfloat16, torch.float16
ODT = {F32: oracle.F32, BF16: oracle.BF16, F16: oracle.F16}


def _out(n, dtype, offset=0):
    g = Guarded(n, dtype if dtype != F16 else BF16, offset_elems=offset)
    return g, (g.view.view(dtype) if dtype == F16 else g.view)


def _shifted(host, off):
    """The host tensor on the device at a one-element misalignment `off` (0 or 1)."""
    raw = torch.empty(host.numel() + 8, dtype=host.dtype, device=DEV)
    view = raw[off:off + host.numel()]
    view.copy_(host.reshape(-1))
    return view.view(host.shape)


@pytest.mark.parametrize("seed", range(60))
def test_random_two_level_share(seed):
    rng = np.random.default_rng(1000 + seed)
    nodes, gpus = int(rng.integers(1, 41)), int(rng.integers(1, 13))
    c = int(rng.choice([1, 2, 63, 64, 65, 127, 129, 500, 1023, 2050, 4097]))
    dtype = [F32, BF16, F16][int(rng.integers(0, 3))]
    average = bool(rng.integers(0, 2))
    my_node, my_gpu = int(rng.integers(0, nodes)), int(rng.integers(0, gpus))
    use_inter, off = bool(rng.integers(0, 2)), int(rng.integers(0, 2))
    case = dict(nodes=nodes, gpus=gpus, c=c, dtype=dtype, average=average, my_node=my_node, my_gpu=my_gpu,
                inter=use_inter, off=off)
    print("case", case, flush=True)
    P = nodes * gpus
    msgs_h = W.normal(gpus * P * c, 3 * seed + 1, 1.0, "cpu", dtype).view(gpus, P * c)
    inter_h = W.normal(nodes * c, 3 * seed + 2, 1.0, "cpu", dtype).view(nodes, c)
    inter = _shifted(inter_h, off)
    d_inter = pccl.device_pointer_array([inter[k] for k in range(nodes)]) if use_inter else None
    want_inter = [to_np(inter_h[k]) for k in range(nodes)] if use_inter else None

    # from pre-shuffled pieces: piece g2 = chunks (n, my_gpu) of node-mate g2's message, n = 0..nodes-1
    x_h = msgs_h.view(gpus, nodes, gpus, c)[:, :, my_gpu, :].contiguous()
    shard, sv = _out(c, dtype, off)
    partial, pv = _out(nodes * c, dtype)
    pccl.pccl_reduce_scatter_local(sv, pv, _shifted(x_h, 0), d_inter=d_inter, my_node=my_node, average=average)
    torch.cuda.synchronize()
    ws, wp = oracle.reduce_scatter_local(to_np(x_h), my_node=my_node, inter=want_inter, average=average)
    assert same_bits(to_np(sv), ws), (case, first_diff(to_np(sv), ws))
    assert same_bits(to_np(pv), wp.reshape(-1)), case
    shard.check()
    partial.check()

    # straight from the rank-order messages: the same numbers by definition
    shard2, sv2 = _out(c, dtype)
    partial2, pv2 = _out(nodes * c, dtype, off)
    pccl.pccl_reduce_scatter_local_unpacked(sv2, pv2, msgs=msgs_h.to(DEV), d_inter=d_inter, nodes=nodes, gpus_per_node=gpus,
                                            my_node=my_node, my_gpu=my_gpu, average=average)
    torch.cuda.synchronize()
    assert same_bits(to_np(sv2), ws) and same_bits(to_np(pv2), wp.reshape(-1)), case
    shard2.check()
    partial2.check()

    # all P sources through the pointer-array two-level sum (node-major), and flat over one node's worth
    srcs_h = msgs_h.view(gpus, P, c)[0]                                  # P chunks standing for P ranks
    srcs = _shifted(srcs_h, off)
    ptrs = pccl.device_pointer_array([srcs[k] for k in range(P)])
    out, ov = _out(c, dtype)
    pccl.pccl_local_reduce_ptrs_two_level(ov, ptrs, nodes, gpus, c, dtype, average=average)
    torch.cuda.synchronize()
    want = oracle.two_level_reduce([to_np(srcs_h[k]) for k in range(P)], nodes, gpus, ODT[dtype], average=average)
    assert same_bits(to_np(ov), want), (case, first_diff(to_np(ov), want))
    pccl.pccl_local_reduce_ptrs(ov, ptrs, c, dtype, average=average)
    torch.cuda.synchronize()
    want = oracle.flat_reduce([to_np(srcs_h[k]) for k in range(P)], ODT[dtype], average=average)
    assert same_bits(to_np(ov), want), (case, first_diff(to_np(ov), want))
    out.check()


@pytest.mark.parametrize("seed", range(40))
def test_random_shuffles(seed):
    rng = np.random.default_rng(2000 + seed)
    nodes, gpus = int(rng.integers(1, 70)), int(rng.integers(1, 13))
    cb = int(rng.choice([0, 1, 2, 15, 16, 17, 1000, 1024, 1025, 4096 + 48, 70000, 65536, 300000]))
    src_off, dst_off = int(rng.integers(0, 3)) * 7, int(rng.integers(0, 3)) * 9
    case = dict(nodes=nodes, gpus=gpus, cb=cb, src_off=src_off, dst_off=dst_off)
    print("case", case, flush=True)
    P = nodes * gpus
    gen = torch.Generator()
    gen.manual_seed(seed)
    host = torch.randint(0, 256, (P * cb,), generator=gen, dtype=torch.uint8)
    raw = torch.empty(P * cb + 64, dtype=torch.uint8, device=DEV)
    src = raw[src_off:src_off + P * cb].copy_(host)
    outs = [Guarded((P * cb + dst_off) // 4 + 8, F32) for _ in range(3)]
    packed, back, via = (o.view.view(torch.uint8)[dst_off:dst_off + P * cb] for o in outs)
    pccl.pccl_hier_pack(packed, src, nodes, gpus)
    pccl.pccl_hier_unpack(back, packed, nodes, gpus)
    if cb:
        slots = pccl.device_pointer_array([packed[k * cb:(k + 1) * cb] for k in range(P)])
        pccl.pccl_allgather_reassemble(via, d_slots=slots, nodes=nodes, gpus_per_node=gpus)
    torch.cuda.synchronize()
    assert same_bits(to_np(packed), oracle.hier_pack(host.numpy(), nodes, gpus)), case
    assert torch.equal(back, src), case
    if cb:
        assert torch.equal(via, src), case
    for o in outs:
        o.check()
