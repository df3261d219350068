"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation),
so a whole all-reduce share can be captured into a HIP graph.  Every replay is checked against
the eager result, with eager work and synchronisations between replays."""
import pytest
import torch

import oracle
import paper_2504_18658_amd as pccl
from paper_2504_18658_amd import workloads as W
from util import same_bits, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_captured_all_reduce_share_replays_match_eager_and_oracle():
    w = W.cfg3(chunk=8192 + 8)
    w.nodes = 4
    P, C = w.ranks, w.chunk
    msg = W.draw(w, P * C, DEV, seed_offset=1)
    x = W.two_level_input(w, DEV, seed_offset=2)
    msgs = W.draw(w, w.gpus * P * C, DEV, seed_offset=3).view(w.gpus, P * C)
    inter = W.draw(w, w.nodes * C, DEV, seed_offset=4).view(w.nodes, C)
    d_inter = pccl.device_pointer_array([inter[n] for n in range(w.nodes)])
    gathered = W.draw(w, P * C, DEV, seed_offset=5)
    srcs = W.draw(w, 64 * 8 * 512, DEV, seed_offset=6).view(64 * 8, 512)
    ptrs = pccl.device_pointer_array([srcs[k] for k in range(64 * 8)])
    recv = W.draw(w, 7 * C, DEV, seed_offset=7).view(7, C)
    ring0 = W.draw(w, 8 * C, DEV, seed_offset=8).view(8, C)
    many = W.draw(w, 40 * 3001, DEV, seed_offset=9).view(40, 3001)        # 40 sources: the LDS-staged flat sum
    odd = W.draw(w, P * 1501 + 1, DEV, seed_offset=10)[1:]                # a message whose chunks start mid-word

    def buffers():
        return dict(packed=torch.empty_like(msg), partial=torch.empty(w.nodes * C, dtype=w.dtype, device=DEV),
                    shard=torch.empty(C, dtype=w.dtype, device=DEV), partial2=torch.empty(w.nodes * C, dtype=w.dtype, device=DEV),
                    shard2=torch.empty(C, dtype=w.dtype, device=DEV), out=torch.empty_like(gathered),
                    small=torch.empty(512, dtype=torch.float32, device=DEV), ring=torch.empty_like(ring0),
                    flat=torch.empty(3001, dtype=w.dtype, device=DEV), oddpacked=torch.empty(P * 1501, dtype=w.dtype, device=DEV),
                    shard3=torch.empty(C, dtype=w.dtype, device=DEV), partial3=torch.empty(w.nodes * C, dtype=w.dtype, device=DEV),
                    tail=torch.empty_like(gathered), halving=torch.empty_like(ring0), shard4=torch.empty(C, dtype=w.dtype, device=DEV),
                    acc_a=torch.empty(3001, dtype=w.dtype, device=DEV), acc_b=torch.empty(C, dtype=w.dtype, device=DEV))

    def step(b):
        pccl.pccl_hier_pack(b["packed"], msg, w.nodes, w.gpus)
        pccl.pccl_reduce_scatter_local(b["shard"], b["partial"], x, d_inter=d_inter, my_node=1, average=True)
        pccl.pccl_reduce_scatter_local_unpacked(b["shard2"], b["partial2"], msgs=msgs, d_inter=d_inter, nodes=w.nodes,
                                                gpus_per_node=w.gpus, my_node=2, my_gpu=5)
        pccl.pccl_allgather_reassemble(b["out"], src=gathered, nodes=w.nodes, gpus_per_node=w.gpus)
        pccl.pccl_local_reduce_ptrs_two_level(b["small"], ptrs, 64, 8, 512, w.dtype)
        b["ring"].copy_(ring0)                      # the replay mutates its message in place: reset it first
        pccl.pccl_ring_reduce_scatter_local(b["ring"], recv, 3)
        pccl.pccl_local_reduce(b["flat"], many)
        pccl.pccl_hier_pack(b["oddpacked"], odd, w.nodes, w.gpus)
        pccl.pccl_reduce_scatter_local_unpacked_batched(b["table"], 5)
        # the one-launch all-reduce tail (reads the partial of the second call above), the one-launch halving
        # replay, the share whose partial lives in the library's static workspace, and a batch of two steps
        pccl.pccl_phase2_reassemble_local(b["tail"], b["partial2"], d_inter=d_inter, src=gathered, nodes=w.nodes,
                                          gpus_per_node=w.gpus, my_node=2, my_gpu=5)
        b["halving"].copy_(ring0)
        pccl.pccl_halving_reduce_scatter_local(b["halving"], recv.view(-1), 6)
        pccl.pccl_reduce_scatter_local_static(b["shard4"], x, d_inter=d_inter, my_node=1, average=True)
        b["acc_a"].copy_(many[0])
        b["acc_b"].copy_(inter[0])
        pccl.pccl_accumulate_batched(b["acc_table"])

    def with_table(b):
        b["table"] = pccl.BucketTable([(b["shard3"], b["partial3"], msgs)], nodes=w.nodes)   # built outside the capture
        b["acc_table"] = pccl.AccumulateTable([(b["acc_a"], many[1]), (b["acc_b"], inter[1])])
        return b

    eager = with_table(buffers())
    step(eager)
    torch.cuda.synchronize()

    cap = with_table(buffers())
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(cap)                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        step(cap)
    for replay in range(4):
        for t in cap.values():
            if isinstance(t, torch.Tensor):
                t.view(torch.int16 if t.element_size() == 2 else torch.int32).fill_(0x5A5A)   # poison by an eager kernel
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in eager:
            if isinstance(eager[k], torch.Tensor):
                assert same_bits(to_np(cap[k]), to_np(eager[k])), (replay, k)
        step(with_table(buffers()))                 # eager work between replays
        torch.cuda.synchronize()
    # and the eager result itself is the oracle's
    ws, wp = oracle.reduce_scatter_local(to_np(x), my_node=1, inter=[to_np(inter[n]) for n in range(w.nodes)], average=True)
    assert same_bits(to_np(eager["shard"]), ws) and same_bits(to_np(eager["partial"]), wp.reshape(-1))
    assert same_bits(to_np(eager["packed"]), oracle.hier_pack(to_np(msg), w.nodes, w.gpus))
    assert same_bits(to_np(eager["ring"]), oracle.ring_rs_local(to_np(ring0), [to_np(recv[s]) for s in range(7)], 3))
    assert same_bits(to_np(eager["flat"]), oracle.flat_reduce([to_np(many[s]) for s in range(40)]))
    assert same_bits(to_np(eager["oddpacked"]), oracle.hier_pack(to_np(odd), w.nodes, w.gpus))
    ws, wp = oracle.reduce_scatter_local_unpacked([to_np(msgs[g]) for g in range(w.gpus)], w.nodes, w.gpus, 5)
    assert same_bits(to_np(eager["shard3"]), ws) and same_bits(to_np(eager["partial3"]), wp.reshape(-1))
    assert same_bits(to_np(eager["shard4"]), to_np(eager["shard"]))
    rows = [to_np(eager["partial2"].view(w.nodes, C)[n]) if n == 2 else to_np(inter[n]) for n in range(w.nodes)]
    slots = [to_np(gathered.view(P, C)[k]) for k in range(P)]
    assert same_bits(to_np(eager["tail"]), oracle.phase2_reassemble(rows, slots, w.nodes, w.gpus, 2, 5))
    flat = recv.reshape(-1)
    halves = [to_np(flat[:4 * C]), to_np(flat[4 * C:6 * C]), to_np(flat[6 * C:7 * C])]
    assert same_bits(to_np(eager["halving"]), oracle.halving_rs_local(to_np(ring0), halves, 6))
    assert same_bits(to_np(eager["acc_a"]), oracle.accumulate(to_np(many[0]), to_np(many[1])))
    assert same_bits(to_np(eager["acc_b"]), oracle.accumulate(to_np(inter[0]), to_np(inter[1])))
