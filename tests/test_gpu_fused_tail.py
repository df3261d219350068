"""pccl_phase2_reassemble_local -- the inter-node phase of the reduce-scatter share and the
all-gather shuffle in one launch, the rank's own shard landing straight at its rank-order
place -- against the oracle's composition of the two definitions (bit equality), through
every tile body behind it: unrolled streaming (1, 2, 4, 8, 16 nodes), batched streaming
(3, 5, 13 nodes) and the LDS-staged slice (more than 16 nodes)."""
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


def _draw(n, dtype, seed):
    return W.normal(n, seed, 1.0, "cpu", dtype)


def _host(t):
    return to_np(t) if t.dtype != F16 else t.cpu().numpy()


def _case(nodes, gpus, chunk, dtype, my_node, my_gpu, use_inter, use_slots, seed, dst_off=0, average=False):
    """Run one call; return (got, want) rank-order buffers as numpy arrays."""
    P = nodes * gpus
    partial_h = _draw(nodes * chunk, dtype, seed).view(nodes, chunk)
    inter_h = _draw(nodes * chunk, dtype, seed + 1).view(nodes, chunk)
    gathered_h = _draw(P * chunk, dtype, seed + 2).view(P, chunk)              # hierarchical slot order
    partial, gathered = partial_h.to(DEV), gathered_h.to(DEV)
    d_inter = None
    if use_inter:
        inter = inter_h.to(DEV)
        d_inter = pccl.device_pointer_array([inter[j] for j in range(nodes)])
    d_slots, keep = None, None
    if use_slots:
        # every slot in its own place (shuffled order inside one arena); the rank's own slot points nowhere useful
        arena = torch.empty(P + 3, chunk + 8, dtype=dtype, device=DEV)
        order = W.shuffled_slot_order(P, seed)
        keep = [arena[order[k] + 1, :chunk] for k in range(P)]
        for k in range(P):
            keep[k].copy_(gathered[k])
        own = my_gpu * nodes + my_node
        ptrs = [t.data_ptr() for t in keep]
        ptrs[own] = 0                                                         # never read: NULL is fine
        d_slots = torch.tensor(ptrs, dtype=torch.int64).to(DEV)
    dst = Guarded(P * chunk, dtype, offset_elems=dst_off) if dtype != F16 else None   # guard bands: fp32 / bf16
    out = dst.view if dst is not None else torch.empty(P * chunk, dtype=dtype, device=DEV)
    print("fused tail", nodes, gpus, chunk, dtype, my_node, my_gpu, use_inter, use_slots, dst_off, flush=True)
    pccl.pccl_phase2_reassemble_local(out, partial, d_inter=d_inter, src=None if use_slots else gathered.view(-1),
                                      d_slots=d_slots, nodes=nodes, gpus_per_node=gpus, my_node=my_node,
                                      my_gpu=my_gpu, average=average)
    torch.cuda.synchronize()
    if dst is not None:
        dst.check()
    rows = [_host(partial_h[n]) if (not use_inter or n == my_node) else _host(inter_h[n]) for n in range(nodes)]
    slots = [_host(gathered_h[k]) for k in range(P)]
    slots[my_gpu * nodes + my_node] = None
    want = oracle.phase2_reassemble(rows, slots, nodes, gpus, my_node, my_gpu, divisor=P if average else 0)
    return _host(out), want


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
@pytest.mark.parametrize("nodes", [1, 2, 3, 4, 5, 8, 13, 16, 17, 40])
@pytest.mark.parametrize("chunk", [1, 7, 1000, 4096 * 3 + 5])
def test_tail_matches_oracle(dtype, nodes, chunk):
    gpus = 1 + (nodes + chunk) % 4
    my_node, my_gpu = nodes // 2, gpus - 1
    use_inter, use_slots = bool((nodes + chunk) & 1), bool(chunk & 2)
    got, want = _case(nodes, gpus, chunk, dtype, my_node, my_gpu, use_inter, use_slots, seed=nodes * 1000 + chunk)
    assert same_bits(got, want), first_diff(got, want)


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("dst_off", [1, 3])
@pytest.mark.parametrize("nodes", [4, 16, 24])
def test_tail_unaligned_destination_and_odd_chunks(dtype, dst_off, nodes):
    got, want = _case(nodes, 3, 2049, dtype, 1, 2, True, True, seed=50 + nodes, dst_off=dst_off)
    assert same_bits(got, want), first_diff(got, want)
    got, want = _case(nodes, 2, 515, dtype, nodes - 1, 0, False, False, seed=60 + nodes, dst_off=dst_off)
    assert same_bits(got, want), first_diff(got, want)


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
@pytest.mark.parametrize("nodes", [2, 16, 32])
def test_tail_average_divides_the_own_shard_only(dtype, nodes):
    got, want = _case(nodes, 4, 777, dtype, 1, 3, True, False, seed=70 + nodes, average=True)
    assert same_bits(got, want), first_diff(got, want)


def test_tail_every_rank_position():
    """The own chunk lands at rank-order place my_node*M + my_gpu for every (my_node, my_gpu)."""
    nodes, gpus, chunk = 3, 4, 130
    for n in range(nodes):
        for g in range(gpus):
            got, want = _case(nodes, gpus, chunk, BF16, n, g, True, True, seed=200 + n * gpus + g)
            assert same_bits(got, want), (n, g, first_diff(got, want))


def test_phase1_only_then_tail_equals_the_three_call_path():
    """shard=None runs phase 1 only; finishing with the fused tail gives the bits of
    pccl_reduce_scatter_local followed by pccl_allgather_reassemble with the shard in its slot."""
    w = W.cfg3(chunk=3000 + 8)
    w.nodes = 8
    my_node, my_gpu = 5, 2
    x = W.two_level_input(w, DEV, seed_offset=3)
    inter = W.draw(w, w.nodes * w.chunk, DEV, seed_offset=4).view(w.nodes, w.chunk)
    d_inter = pccl.device_pointer_array([inter[j] for j in range(w.nodes)])
    gathered = W.draw(w, w.ranks * w.chunk, DEV, seed_offset=5)
    # three calls
    partial = torch.empty(w.nodes * w.chunk, dtype=w.dtype, device=DEV)
    shard = torch.empty(w.chunk, dtype=w.dtype, device=DEV)
    pccl.pccl_reduce_scatter_local(shard, partial, x, d_inter=d_inter, my_node=my_node)
    g2 = gathered.clone().view(w.gpus, w.nodes, w.chunk)
    g2[my_gpu, my_node].copy_(shard)
    ref = torch.empty_like(gathered)
    pccl.pccl_allgather_reassemble(ref, src=g2.view(-1), nodes=w.nodes, gpus_per_node=w.gpus)
    # two calls
    partial2 = torch.full_like(partial, 9.0)
    pccl.pccl_reduce_scatter_local(None, partial2, x, d_inter=d_inter, my_node=my_node)
    out = torch.empty_like(gathered)
    pccl.pccl_phase2_reassemble_local(out, partial2, d_inter=d_inter, src=gathered, nodes=w.nodes,
                                      gpus_per_node=w.gpus, my_node=my_node, my_gpu=my_gpu)
    torch.cuda.synchronize()
    assert same_bits(to_np(partial2), to_np(partial))
    assert same_bits(to_np(out), to_np(ref)), first_diff(to_np(out), to_np(ref))
    # the same from rank-order messages
    msgs = W.draw(w, w.gpus * w.ranks * w.chunk, DEV, seed_offset=6).view(w.gpus, w.ranks * w.chunk)
    pa = torch.empty_like(partial)
    pb = torch.empty_like(partial)
    sh = torch.empty_like(shard)
    pccl.pccl_reduce_scatter_local_unpacked(sh, pa, msgs=msgs, nodes=w.nodes, gpus_per_node=w.gpus, my_node=my_node,
                                            my_gpu=my_gpu)
    pccl.pccl_reduce_scatter_local_unpacked(None, pb, msgs=msgs, nodes=w.nodes, gpus_per_node=w.gpus, my_node=my_node,
                                            my_gpu=my_gpu)
    torch.cuda.synchronize()
    assert same_bits(to_np(pa), to_np(pb))


def test_cfg3_size_tail_full():
    """16 x 8 ranks, 2 MB bf16 chunks: 15 received chunks through d_inter, 256 MB of gathered shards."""
    w = W.cfg3()
    my_node, my_gpu = 5, 3
    partial = W.draw(w, w.nodes * w.chunk, DEV, seed_offset=31).view(w.nodes, w.chunk)
    inter = W.draw(w, w.nodes * w.chunk, DEV, seed_offset=32).view(w.nodes, w.chunk)
    d_inter = pccl.device_pointer_array([inter[j] for j in range(w.nodes)])
    gathered = W.draw(w, w.ranks * w.chunk, DEV, seed_offset=33)
    out = Guarded(w.ranks * w.chunk, w.dtype)
    pccl.pccl_phase2_reassemble_local(out.view, partial.view(-1), d_inter=d_inter, src=gathered, nodes=w.nodes,
                                      gpus_per_node=w.gpus, my_node=my_node, my_gpu=my_gpu)
    torch.cuda.synchronize()
    out.check()
    rows = [to_np(partial[n]) if n == my_node else to_np(inter[n]) for n in range(w.nodes)]
    slots = [to_np(gathered.view(w.ranks, w.chunk)[k]) for k in range(w.ranks)]
    slots[my_gpu * w.nodes + my_node] = None
    want = oracle.phase2_reassemble(rows, slots, w.nodes, w.gpus, my_node, my_gpu, nthreads=16)
    got = to_np(out.view)
    assert same_bits(got, want), first_diff(got, want)


def test_cfg4_size_tail_full():
    """256 x 8 ranks, 64 KB fp32 chunks: 256 node partials through a pointer array, 2048 gathered
    shards in shuffled arena slots through d_slots."""
    w = W.cfg4()
    my_node, my_gpu = 200, 6
    partial = W.draw(w, w.nodes * w.chunk, DEV, seed_offset=41).view(w.nodes, w.chunk)
    inter = W.draw(w, w.nodes * w.chunk, DEV, seed_offset=42).view(w.nodes, w.chunk)
    d_inter = pccl.device_pointer_array([inter[j] for j in range(w.nodes)])
    arena = W.draw(w, w.ranks * w.chunk, DEV, seed_offset=43).view(w.ranks, w.chunk)
    order = W.shuffled_slot_order(w.ranks, w.seed)
    d_slots = pccl.device_pointer_array([arena[order[s]] for s in range(w.ranks)])
    out = Guarded(w.ranks * w.chunk, w.dtype)
    pccl.pccl_phase2_reassemble_local(out.view, partial.view(-1), d_inter=d_inter, d_slots=d_slots, nodes=w.nodes,
                                      gpus_per_node=w.gpus, my_node=my_node, my_gpu=my_gpu)
    torch.cuda.synchronize()
    out.check()
    rows = [to_np(partial[n]) if n == my_node else to_np(inter[n]) for n in range(w.nodes)]
    slots = [to_np(arena[order[s]]) for s in range(w.ranks)]
    slots[my_gpu * w.nodes + my_node] = None
    want = oracle.phase2_reassemble(rows, slots, w.nodes, w.gpus, my_node, my_gpu, nthreads=16)
    got = to_np(out.view)
    assert same_bits(got, want), first_diff(got, want)
