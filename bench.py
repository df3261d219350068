#!/usr/bin/env python3
"""Benchmark of the local kernels of PCCL's hierarchical collectives on one MI355X.

A step is one GPU's share of a two-level all-reduce of one 256 MB bf16 message at
16 nodes x 8 GPUs (the 256 MB workload of the configuration list):
    pccl_hier_pack            256 MB rank-order message -> hierarchical order
    pccl_reduce_scatter_local phase 1: 8 x 32 MB -> 32 MB partial; phase 2: 16 x 2 MB -> 2 MB, both in
                              one launch (the 15 foreign chunks arrive through a device pointer array)
    pccl_allgather_reassemble 256 MB of gathered shards -> rank order
Inputs are seeded synthetic tensors already resident in HBM; every step works on the next of
several disjoint buffer sets so that the last-level cache cannot serve a re-run.

Prints ONE JSON line.  `value` = algorithmic bytes of a step / wall time of a step (no event is
recorded inside the timed steps).  `roofline` is for the dominant kernel (the chunk transpose):
after the timed steps, 24 pack and 24 reassemble launches run back to back over the rotating
buffer sets between ONE pair of HIP events on the launch stream, whatever --steps is; `calls`
holds the same measurement for each of the three calls, and next to it the figure with every
call bracketed by its own event pair (an event record stalls the stream for about 3 us, so that
figure is the larger one).  `size_sweep` repeats the kernels at 64 / 128 / 256 MB messages (the
metric's range; 16 MB - 1 GB with --sweep).  `cpu_baseline` times the CPU oracle on the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402
import torch  # noqa: E402

import paper_2504_18658_amd as pccl  # noqa: E402
from paper_2504_18658_amd import workloads as W  # noqa: E402

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak
# HBM bytes of one 256 MB k_permute launch, from profiles/k_permute_256MB_16x8.txt (two rocprofv3 --pmc
# runs of this file, FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each scaled by what the same counter
# reads for a plain 256 MiB copy: FETCH_SIZE x 2.000, WRITE_SIZE x 1.000).  A profiler figure, not measured here.
PROFILED_PERMUTE_FETCH_KIB, PROFILED_PERMUTE_WRITE_KIB = 131091.6, 262144.0
PROFILED_PERMUTE_TRAFFIC_BYTES = int((PROFILED_PERMUTE_FETCH_KIB * 2.000 + PROFILED_PERMUTE_WRITE_KIB * 1.000) * 1024)
MB = 1 << 20


def to_np(t):
    t = t.detach().cpu().contiguous()
    return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()


class AllReduceShare:
    """Buffers of one step of the headline workload (one of several rotating sets)."""

    def __init__(self, w, dev, k, my_node=5):
        self.w, self.my_node = w, my_node
        n = w.ranks * w.chunk
        self.msg = W.draw(w, n, dev, seed_offset=10 * k + 1)          # [node][gpu][chunk]
        self.packed = torch.empty_like(self.msg)                       # [gpu][node][chunk]
        self.x = W.two_level_input(w, dev, seed_offset=10 * k + 2)     # [gpu'][node][chunk] received
        self.partial = torch.empty(w.nodes * w.chunk, dtype=w.dtype, device=dev)
        self.shard = torch.empty(w.chunk, dtype=w.dtype, device=dev)
        self.inter = W.draw(w, w.nodes * w.chunk, dev, seed_offset=10 * k + 3).view(w.nodes, w.chunk)
        self.d_inter = pccl.device_pointer_array([self.inter[j] for j in range(w.nodes)])
        self.gathered = W.draw(w, n, dev, seed_offset=10 * k + 4)      # [gpu][node][chunk]
        self.out = torch.empty_like(self.gathered)

    def bytes_per_call(self):
        w = self.w
        e = w.esize
        m = w.ranks * w.chunk * e
        piece = w.nodes * w.chunk * e
        return {
            "pccl_hier_pack": 2 * m,
            "pccl_reduce_scatter_local": (w.gpus + 1) * piece + (w.nodes + 1) * w.chunk * e,
            "pccl_allgather_reassemble": 2 * m,
        }

    def run(self, events=None):
        w = self.w
        if events is not None:
            events[0].record()
        pccl.pccl_hier_pack(self.packed, self.msg, w.nodes, w.gpus)
        if events is not None:
            events[1].record()
        pccl.pccl_reduce_scatter_local(self.shard, self.partial, self.x, d_inter=self.d_inter,
                                       my_node=self.my_node)
        if events is not None:
            events[2].record()
        pccl.pccl_allgather_reassemble(self.out, src=self.gathered, nodes=w.nodes, gpus_per_node=w.gpus)
        if events is not None:
            events[3].record()

    def call(self, name):
        """One of the three calls of a step, as a function."""
        w = self.w
        return {
            "pccl_hier_pack": lambda: pccl.pccl_hier_pack(self.packed, self.msg, w.nodes, w.gpus),
            "pccl_reduce_scatter_local": lambda: pccl.pccl_reduce_scatter_local(
                self.shard, self.partial, self.x, d_inter=self.d_inter, my_node=self.my_node),
            "pccl_allgather_reassemble": lambda: pccl.pccl_allgather_reassemble(
                self.out, src=self.gathered, nodes=w.nodes, gpus_per_node=w.gpus),
        }[name]

    def oracle_step(self, host, nthreads=1):
        import oracle
        w = self.w
        packed = oracle.hier_pack(host["msg"], w.nodes, w.gpus)
        inter = [host["inter"][j] for j in range(w.nodes)]
        shard, partial = oracle.reduce_scatter_local(host["x"], my_node=self.my_node, inter=inter,
                                                     nthreads=nthreads)
        out = oracle.hier_unpack(host["gathered"], w.nodes, w.gpus)
        return packed, partial, shard, out

    def host_inputs(self):
        return {"msg": to_np(self.msg), "x": to_np(self.x), "inter": to_np(self.inter),
                "gathered": to_np(self.gathered)}


def time_calls(fn_list, trials=10, warm=3):
    """Mean/min milliseconds of fn_list[k % len]() over `trials` calls, events on the current stream."""
    for k in range(warm):
        fn_list[k % len(fn_list)]()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(trials)]
    torch.cuda.synchronize()
    # keep the GPU busy while the host enqueues, so that the timed calls run back to back and
    # an event pair brackets the kernels, not the host's launch latency
    torch.cuda._sleep(2_000_000)
    for k in range(trials):
        ev[k][0].record()
        fn_list[k % len(fn_list)]()
        ev[k][1].record()
    torch.cuda.synchronize()
    ms = [a.elapsed_time(b) for a, b in ev]
    # the same calls back to back inside ONE event pair: no event stall between launches
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda._sleep(2_000_000)
    a.record()
    for k in range(trials):
        fn_list[k % len(fn_list)]()
    b.record()
    torch.cuda.synchronize()
    return float(np.mean(ms)), float(np.min(ms)), float(np.std(ms)), a.elapsed_time(b) / trials


def back_to_back(fn_list, launches=24, warm=4):
    """Microseconds per call of `launches` calls fn_list[k % len]() enqueued back to back between ONE pair of
    events on the current stream (no event between the launches)."""
    for k in range(warm):
        fn_list[k % len(fn_list)]()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    torch.cuda._sleep(2_000_000)     # the GPU is busy while the host enqueues: the launches then run gap-free
    a.record()
    for k in range(launches):
        fn_list[k % len(fn_list)]()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / launches


def graph_replay_us(fn_list, rounds, replays=20):
    """Microseconds per call when `rounds` passes over fn_list are captured in one HIP graph and the
    graph is replayed (a launch-bound call issued from Python is bound by the host, not by the GPU)."""
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for fn in fn_list:
            fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(rounds):
            for fn in fn_list:
                fn()
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(replays):
        g.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / (replays * rounds * len(fn_list)) * 1e6


def other_workloads(dev):
    """The remaining configurations, each timed on its own (10 trials, rotating buffer sets)."""
    res = {}

    def entry(name, nbytes, mean_ms, min_ms, std_ms, burst_ms, **kw):
        # mean/min/std: every call bracketed by its own event pair (includes the event stall);
        # back_to_back: the same calls inside one pair
        res[name] = dict(bytes=nbytes, mean_us=round(mean_ms * 1e3, 2), min_us=round(min_ms * 1e3, 2),
                         std_us=round(std_ms * 1e3, 2), GBps=round(nbytes / (mean_ms * 1e-3) / 1e9, 1),
                         frac_of_peak=round(nbytes / (mean_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                         back_to_back_us=round(burst_ms * 1e3, 2),
                         back_to_back_GBps=round(nbytes / (burst_ms * 1e-3) / 1e9, 1), **kw)

    # cfg1: flat reduce of 8 x 512 KB fp32 (latency-sized)
    w = W.cfg1()
    sets = [(torch.empty(w.chunk, dtype=w.dtype, device=dev),
             W.draw(w, w.gpus * w.chunk, dev, seed_offset=k).view(w.gpus, w.chunk)) for k in range(8)]
    fns = [lambda s=s: pccl.pccl_local_reduce(s[0], s[1]) for s in sets]
    entry("cfg1_flat_reduce_p8_f32_512KB", (w.gpus + 1) * w.chunk * 4, *time_calls(fns),
          graph_replay_us=round(graph_replay_us(fns, 4), 2))
    del sets, fns
    # cfg2: all-gather reassembly, 4 x 8, 64 MB bf16
    w = W.cfg2()
    n = w.ranks * w.chunk
    sets = [(torch.empty(n, dtype=w.dtype, device=dev), W.draw(w, n, dev, seed_offset=k)) for k in range(8)]
    entry("cfg2_hier_unpack_4x8_bf16_64MB", 2 * n * 2,
          *time_calls([lambda s=s: pccl.pccl_hier_unpack(s[0], s[1], w.nodes, w.gpus) for s in sets]))
    del sets
    # cfg4: 2048 x 64 KB fp32 through a shuffled pointer array, then reassembly of 128 MB
    w = W.cfg4()
    sets = []
    for k in range(4):
        arena = W.draw(w, w.ranks * w.chunk, dev, seed_offset=k).view(w.ranks, w.chunk)
        order = W.shuffled_slot_order(w.ranks, w.seed + k)
        ptrs = pccl.device_pointer_array([arena[order[s]] for s in range(w.ranks)])
        sets.append((torch.empty(w.chunk, dtype=w.dtype, device=dev), ptrs, arena,
                     torch.empty(w.ranks * w.chunk, dtype=w.dtype, device=dev)))
    entry("cfg4_reduce_ptrs_two_level_256x8_f32_128MB", (w.ranks + 1) * w.chunk * 4,
          *time_calls([lambda s=s: pccl.pccl_local_reduce_ptrs_two_level(
              s[0], s[1], w.nodes, w.gpus, w.chunk, w.dtype) for s in sets], trials=24, warm=8))
    entry("cfg4_allgather_reassemble_256x8_f32_128MB", 2 * w.ranks * w.chunk * 4,
          *time_calls([lambda s=s: pccl.pccl_allgather_reassemble(
              s[3], src=s[2], nodes=w.nodes, gpus_per_node=w.gpus) for s in sets], trials=24, warm=8))
    del sets
    # op = average and fp16 messages on the 256 MB two-level share (same bytes as the headline's reduce call)
    w = W.cfg3()
    nb = (w.gpus + 1) * w.nodes * w.chunk * 2 + (w.nodes + 1) * w.chunk * 2
    for tag, dt, avg in (("bf16_average", torch.bfloat16, True), ("f16_sum", torch.float16, False)):
        sets = []
        for k in range(4):
            x = W.uniform_pm1(w.gpus * w.nodes * w.chunk, 300 + k, dev, dt).view(w.gpus, w.nodes, w.chunk)
            inter = W.uniform_pm1(w.nodes * w.chunk, 310 + k, dev, dt).view(w.nodes, w.chunk)
            sets.append((torch.empty(w.chunk, dtype=dt, device=dev), torch.empty(w.nodes * w.chunk, dtype=dt, device=dev),
                         x, pccl.device_pointer_array([inter[j] for j in range(w.nodes)]), inter))
        entry("cfg3_reduce_scatter_local_%s_256MB" % tag, nb,
              *time_calls([lambda s=s: pccl.pccl_reduce_scatter_local(s[0], s[1], s[2], d_inter=s[3], my_node=5,
                                                                      average=avg) for s in sets]))
        del sets
    # a DDP gradient bucket (Section II-A: 48-80 MB of fp32 gradients per all-reduce): one rank's share of
    # a two-level all-reduce of a 64 MB fp32 bucket at 128 nodes x 8 GPUs (64 KB chunks)
    n_nodes, n_gpus, c = 128, 8, 16384
    P = n_nodes * n_gpus
    sets = []
    for k in range(8):
        msg = W.normal(P * c, 600 + k, 1e-3, dev)
        x = W.normal(n_gpus * n_nodes * c, 610 + k, 1e-3, dev).view(n_gpus, n_nodes, c)
        inter = W.normal(n_nodes * c, 620 + k, 1e-3, dev).view(n_nodes, c)
        sets.append(dict(msg=msg, packed=torch.empty_like(msg), x=x, inter=inter,
                         d_inter=pccl.device_pointer_array([inter[j] for j in range(n_nodes)]),
                         partial=torch.empty(n_nodes * c, device=dev), shard=torch.empty(c, device=dev),
                         gathered=W.normal(P * c, 630 + k, 1e-3, dev), out=torch.empty(P * c, device=dev)))

    def ddp_share(s):
        pccl.pccl_hier_pack(s["packed"], s["msg"], n_nodes, n_gpus)
        pccl.pccl_reduce_scatter_local(s["shard"], s["partial"], s["x"], d_inter=s["d_inter"], my_node=77, average=True)
        pccl.pccl_allgather_reassemble(s["out"], src=s["gathered"], nodes=n_nodes, gpus_per_node=n_gpus)

    ddp_bytes = 2 * P * c * 4 + (n_gpus + 1) * n_nodes * c * 4 + (n_nodes + 1) * c * 4 + 2 * P * c * 4
    entry("ddp_bucket_64MB_f32_allreduce_share_128x8_average", ddp_bytes,
          *time_calls([lambda s=s: ddp_share(s) for s in sets], trials=16, warm=8), launches_per_call=4)
    del sets
    # the headline message at the paper's scale (Section V-A runs up to 2048 GCDs): one rank's share
    # of a two-level all-reduce of 256 MB of bf16 at 128 nodes x 8 GPUs (256 KB chunks), with the
    # pre-shuffle and straight from the node-mates' rank-order messages
    n_nodes, n_gpus = 128, 8
    P = n_nodes * n_gpus
    c = (256 << 20) // P // 2
    sets = []
    for k in range(3):
        msgs = W.uniform_pm1(n_gpus * P * c, 700 + k, dev, torch.bfloat16).view(n_gpus, P * c)          # 8 x 256 MB
        inter = W.uniform_pm1(n_nodes * c, 710 + k, dev, torch.bfloat16).view(n_nodes, c)
        sets.append(dict(msgs=msgs, packed=torch.empty(P * c, dtype=torch.bfloat16, device=dev),
                         x=msgs.view(-1)[: n_gpus * n_nodes * c].view(n_gpus, n_nodes, c), inter=inter,
                         d_inter=pccl.device_pointer_array([inter[j] for j in range(n_nodes)]),
                         partial=torch.empty(n_nodes * c, dtype=torch.bfloat16, device=dev),
                         shard=torch.empty(c, dtype=torch.bfloat16, device=dev),
                         out=torch.empty(P * c, dtype=torch.bfloat16, device=dev)))

    def big_share(s):
        pccl.pccl_hier_pack(s["packed"], s["msgs"][0], n_nodes, n_gpus)
        pccl.pccl_reduce_scatter_local(s["shard"], s["partial"], s["x"], d_inter=s["d_inter"], my_node=77)
        pccl.pccl_allgather_reassemble(s["out"], src=s["msgs"][1], nodes=n_nodes, gpus_per_node=n_gpus)

    def big_share_unpacked(s):
        pccl.pccl_reduce_scatter_local_unpacked(s["shard"], s["partial"], msgs=s["msgs"], d_inter=s["d_inter"],
                                                nodes=n_nodes, gpus_per_node=n_gpus, my_node=77, my_gpu=3)
        pccl.pccl_allgather_reassemble(s["out"], src=s["msgs"][1], nodes=n_nodes, gpus_per_node=n_gpus)

    share_bytes = (n_gpus + 1) * n_nodes * c * 2 + (n_nodes + 1) * c * 2
    entry("allreduce_share_256MB_bf16_128x8", 4 * P * c * 2 + share_bytes,
          *time_calls([lambda s=s: big_share(s) for s in sets], trials=12, warm=6), launches_per_call=4)
    entry("allreduce_share_256MB_bf16_128x8_no_pack", 2 * P * c * 2 + share_bytes,
          *time_calls([lambda s=s: big_share_unpacked(s) for s in sets], trials=12, warm=6), launches_per_call=3)
    del sets
    # the paper's literal two-source step (acc += recv) and one rank's replay of its inter-node algorithms
    w = W.cfg3()
    n = 64 * MB                                                     # 128 MB of bf16
    sets = [(W.draw(w, n, dev, seed_offset=40 + k), W.draw(w, n, dev, seed_offset=50 + k)) for k in range(4)]
    entry("step_accumulate_bf16_128MB", 3 * n * 2,
          *time_calls([lambda s=s: pccl.pccl_accumulate(s[0], s[1]) for s in sets]))
    del sets
    p8, c8 = 8, 16 * MB                                             # flat ring over 8 ranks, 256 MB message
    sets = [(W.draw(w, p8 * c8, dev, seed_offset=60 + k).view(p8, c8),
             W.draw(w, (p8 - 1) * c8, dev, seed_offset=70 + k).view(p8 - 1, c8)) for k in range(4)]
    entry("step_ring_rs_local_8_ranks_bf16_256MB", 3 * (p8 - 1) * c8 * 2,
          *time_calls([lambda s=s: pccl.pccl_ring_reduce_scatter_local(s[0], s[1], 3) for s in sets]),
          launches_per_call=1)
    del sets
    sets = [(W.draw(w, w.nodes * w.chunk, dev, seed_offset=80 + k).view(w.nodes, w.chunk),
             W.draw(w, (w.nodes - 1) * w.chunk, dev, seed_offset=90 + k).view(w.nodes - 1, w.chunk))
            for k in range(8)]
    entry("step_ring_rs_local_16_nodes_bf16_32MB", 3 * (w.nodes - 1) * w.chunk * 2,
          *time_calls([lambda s=s: pccl.pccl_ring_reduce_scatter_local(s[0], s[1], 5) for s in sets]),
          launches_per_call=1)
    # one launch: the first kept half is read and written once (2 * p/2 chunks), every received chunk read once (p - 1)
    entry("step_halving_rs_local_16_nodes_bf16_32MB", (2 * w.nodes - 1) * w.chunk * 2,
          *time_calls([lambda s=s: pccl.pccl_halving_reduce_scatter_local(s[0], s[1].view(-1), 5) for s in sets]),
          launches_per_call=1, bytes_if_launched_per_step=3 * (w.nodes - 1) * w.chunk * 2)
    del sets
    # cfg5: 40 ZeRO-3-shaped buckets in one batched call
    w = W.cfg5()
    sizes = w.extra["bucket_bytes"]
    buckets, nbytes = [], 0
    for k, b in enumerate(sizes):
        chunk = b // (w.ranks * w.esize)
        x = W.two_level_input(w, dev, seed_offset=k + 1, chunk=chunk)
        buckets.append((torch.empty(chunk, dtype=w.dtype, device=dev),
                        torch.empty(w.nodes * chunk, dtype=w.dtype, device=dev), x))
        nbytes += (w.gpus + 1) * w.nodes * chunk * 2 + (w.nodes + 1) * chunk * 2
    table = pccl.BucketTable(buckets)
    entry("cfg5_rs_batched_40_buckets_8x8_bf16", nbytes,
          *time_calls([lambda: pccl.pccl_reduce_scatter_local_batched(table)], trials=5, warm=2),
          total_bucket_MB=round(sum(sizes) / MB, 1))
    del table, buckets
    torch.cuda.empty_cache()
    # the same 40 buckets straight from the eight node-mates' rank-order messages (no pre-shuffle of any
    # bucket): 8 x 5 GB of messages resident, same algorithmic bytes
    buckets = []
    for k, b in enumerate(sizes):
        chunk = b // (w.ranks * w.esize)
        msgs = W.normal(w.gpus * w.ranks * chunk, 300 + k, 1e-3, dev, w.dtype).view(w.gpus, w.ranks * chunk)
        buckets.append((torch.empty(chunk, dtype=w.dtype, device=dev),
                        torch.empty(w.nodes * chunk, dtype=w.dtype, device=dev), msgs))
    table = pccl.BucketTable(buckets, nodes=w.nodes)
    entry("cfg5_rs_unpacked_batched_40_buckets_8x8_bf16", nbytes,
          *time_calls([lambda: pccl.pccl_reduce_scatter_local_unpacked_batched(table, 3)], trials=5, warm=2),
          total_bucket_MB=round(sum(sizes) / MB, 1))
    del table, buckets
    torch.cuda.empty_cache()
    # the all-gather side of the same 40 buckets: every bucket's shuffle into rank order, one launch
    pairs = []
    for k, b in enumerate(sizes):
        src = W.random_bits16(b // 2, 500 + k, dev)
        pairs.append((torch.empty_like(src), src))
    ptable = pccl.PermuteTable(pairs, w.nodes, w.gpus)
    entry("cfg5_allgather_reassemble_batched_40_buckets_8x8", 2 * sum(sizes),
          *time_calls([lambda: pccl.pccl_allgather_reassemble_batched(ptable)], trials=5, warm=2),
          total_bucket_MB=round(sum(sizes) / MB, 1))
    return res


def fused_leg(dev, steps, warmup, nsets=4, my_node=5, my_gpu=3):
    """The same all-reduce share in two launches instead of four: phase 1 reads the eight node-mates'
    rank-order 256 MB messages through the node stride (pccl_reduce_scatter_local_unpacked with no shard:
    no pccl_hier_pack pass, 512 MB less traffic), then pccl_phase2_reassemble_local sums the inter-node
    phase straight into the rank's own chunk of the all-gather result while the other chunks are shuffled
    in (no separate phase-2 launch, no copy of the shard).  Timed next to the other two-launch form, the
    whole share in one launch and a plain reassemble (pccl_reduce_scatter_local_unpacked with received
    chunks + pccl_allgather_reassemble), which moves the shard once more."""
    w = W.cfg3()
    n = w.ranks * w.chunk
    sets = []
    for k in range(nsets):
        msgs = W.draw(w, w.gpus * n, dev, seed_offset=200 + k).view(w.gpus, n)
        inter = W.draw(w, w.nodes * w.chunk, dev, seed_offset=210 + k).view(w.nodes, w.chunk)
        sets.append(dict(msgs=msgs, inter=inter,
                         d_inter=pccl.device_pointer_array([inter[j] for j in range(w.nodes)]),
                         partial=torch.empty(w.nodes * w.chunk, dtype=w.dtype, device=dev),
                         shard=torch.empty(w.chunk, dtype=w.dtype, device=dev),
                         gathered=W.draw(w, n, dev, seed_offset=220 + k),
                         out=torch.empty(n, dtype=w.dtype, device=dev)))

    def phase1(s):
        pccl.pccl_reduce_scatter_local_unpacked(None, s["partial"], msgs=s["msgs"], nodes=w.nodes,
                                                gpus_per_node=w.gpus, my_node=my_node, my_gpu=my_gpu)

    def tail(s):
        pccl.pccl_phase2_reassemble_local(s["out"], s["partial"], d_inter=s["d_inter"], src=s["gathered"],
                                          nodes=w.nodes, gpus_per_node=w.gpus, my_node=my_node, my_gpu=my_gpu)

    def run(s):
        phase1(s)
        tail(s)

    def run_share_then_reassemble(s):
        pccl.pccl_reduce_scatter_local_unpacked(s["shard"], s["partial"], msgs=s["msgs"], d_inter=s["d_inter"],
                                                nodes=w.nodes, gpus_per_node=w.gpus, my_node=my_node, my_gpu=my_gpu)
        pccl.pccl_allgather_reassemble(s["out"], src=s["gathered"], nodes=w.nodes, gpus_per_node=w.gpus)

    def wall(fn):
        for k in range(warmup):
            fn(sets[k % nsets])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            fn(sets[k % nsets])
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms, ms3 = wall(run), wall(run_share_then_reassemble)
    e = w.esize
    p1_bytes = (w.gpus + 1) * w.nodes * w.chunk * e
    tail_bytes = (w.nodes + 1) * w.chunk * e + 2 * (n - w.chunk) * e     # the own chunk is summed, not copied
    nbytes = p1_bytes + tail_bytes
    p1_us = back_to_back([lambda s=s: phase1(s) for s in sets])
    tail_us = back_to_back([lambda s=s: tail(s) for s in sets])
    share_us = back_to_back([lambda s=s: pccl.pccl_reduce_scatter_local_unpacked(
        s["shard"], s["partial"], msgs=s["msgs"], d_inter=s["d_inter"], nodes=w.nodes, gpus_per_node=w.gpus,
        my_node=my_node, my_gpu=my_gpu) for s in sets])
    share_bytes = p1_bytes + (w.nodes + 1) * w.chunk * e
    return dict(what="pccl_reduce_scatter_local_unpacked (phase 1 only, no pccl_hier_pack pass) + "
                     "pccl_phase2_reassemble_local (inter-node phase and all-gather shuffle in one launch)",
                launches_per_step=2, ms_per_step=round(ms, 4), algorithmic_bytes_per_step=nbytes,
                GBps=round(nbytes / (ms * 1e-3) / 1e9, 1),
                phase1_from_rank_order_messages_us=round(p1_us, 2),
                phase1_from_rank_order_messages_GBps=round(p1_bytes / (p1_us * 1e-6) / 1e9, 1),
                phase2_reassemble_us=round(tail_us, 2), phase2_reassemble_GBps=round(tail_bytes / (tail_us * 1e-6) / 1e9, 1),
                whole_share_from_rank_order_messages_us=round(share_us, 2),
                whole_share_from_rank_order_messages_GBps=round(share_bytes / (share_us * 1e-6) / 1e9, 1),
                share_then_reassemble_ms_per_step=round(ms3, 4))


def size_sweep(dev, sizes_mb=(64, 128, 256)):
    """Message sizes through the three kernels: chunk transpose (16 x 8 ranks), 8-source bf16 reduce
    (phase 1) and the two-source step; back-to-back launches over rotating buffer sets.  By default the
    metric's range (64 - 256 MB); the paper's whole range (16 MB - 1 GB, Section V-A) with --sweep."""
    w = W.cfg3()
    out = []
    for mb in sizes_mb:
        m = mb * MB
        n = m // 2                                              # bf16 elements of the message
        nsets = max(2, min(8, (1024 * MB) // m + 1))             # rotate over at least ~1 GB of inputs
        row = {"message_MB": mb, "buffer_sets": nsets}
        sets = [(torch.empty(n, dtype=w.dtype, device=dev), W.draw(w, n, dev, seed_offset=400 + k)) for k in range(nsets)]
        t = time_calls([lambda s=s: pccl.pccl_hier_pack(s[0], s[1], w.nodes, w.gpus) for s in sets], trials=2 * nsets)
        row["hier_pack_us"] = round(t[3] * 1e3, 2)
        row["hier_pack_GBps"] = round(2 * m / (t[3] * 1e-3) / 1e9, 1)
        row["hier_pack_frac_of_peak"] = round(2 * m / (t[3] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        # phase 1 of the share of this message: 8 pieces of m/8 -> m/8
        t = time_calls([lambda s=s: pccl.pccl_local_reduce(s[0][: n // 8], s[1].view(8, n // 8)) for s in sets],
                       trials=2 * nsets)
        row["reduce8_us"] = round(t[3] * 1e3, 2)
        row["reduce8_GBps"] = round((m + m // 8) / (t[3] * 1e-3) / 1e9, 1)
        row["reduce8_frac_of_peak"] = round((m + m // 8) / (t[3] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        # first halving step on this message: m/2 += m/2
        t = time_calls([lambda s=s: pccl.pccl_accumulate(s[0][: n // 2], s[1][: n // 2]) for s in sets], trials=2 * nsets)
        row["accumulate_us"] = round(t[3] * 1e3, 2)
        row["accumulate_GBps"] = round(3 * (m // 2) / (t[3] * 1e-3) / 1e9, 1)
        row["accumulate_frac_of_peak"] = round(3 * (m // 2) / (t[3] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        out.append(row)
        del sets
        torch.cuda.empty_cache()
    return out


def scale_sweep(dev):
    """Message size x node count (8 GPUs per node), the two axes of the paper's heat maps
    (Section IV-B, Section V-A: 16 MB - 1 GB, up to 2048 GCDs), through the four calls of an
    all-reduce share (the other nodes' chunks received in buffers of their own): bf16, back-to-back
    launches over rotating buffer sets."""
    gpus, dt = 8, torch.bfloat16
    out = []
    for mb in (16, 64, 256, 1024):
        m = mb * MB
        n = m // 2
        nsets = 2 if mb >= 256 else 4
        sets = []
        for k in range(nsets):
            msgs = W.uniform_pm1(gpus * n, 800 + k, dev, dt).view(gpus, n)
            sets.append(dict(msgs=msgs, packed=torch.empty(n, dtype=dt, device=dev), out=torch.empty(n, dtype=dt, device=dev),
                             partial=torch.empty(n // gpus, dtype=dt, device=dev), shard=torch.empty(n // (4 * gpus), dtype=dt, device=dev),
                             inter=W.uniform_pm1(n // gpus, 900 + k, dev, dt)))   # the chunks received from the other nodes
        for nodes in (4, 16, 64, 256):
            c = n // (nodes * gpus)
            share_bytes = (gpus + 1) * nodes * c * 2 + (nodes + 1) * c * 2
            row = {"message_MB": mb, "nodes": nodes, "chunk_KB": c * 2 // 1024}

            def put(name, nbytes, t):
                row[name + "_us"] = round(t[3] * 1e3, 2)
                row[name + "_GBps"] = round(nbytes / (t[3] * 1e-3) / 1e9, 1)

            for s in sets:
                s["d_inter"] = pccl.device_pointer_array([s["inter"][j * c:(j + 1) * c] for j in range(nodes)])
            put("hier_pack", 2 * m, time_calls(
                [lambda s=s: pccl.pccl_hier_pack(s["packed"], s["msgs"][0], nodes, gpus) for s in sets], trials=4 * nsets))
            put("reduce_scatter_local", share_bytes, time_calls(
                [lambda s=s: pccl.pccl_reduce_scatter_local(s["shard"][:c], s["partial"], s["msgs"][0].view(gpus, nodes, c),
                                                            d_inter=s["d_inter"], my_node=nodes // 3)
                 for s in sets], trials=4 * nsets))
            put("reduce_scatter_local_unpacked", share_bytes, time_calls(
                [lambda s=s: pccl.pccl_reduce_scatter_local_unpacked(s["shard"][:c], s["partial"], msgs=s["msgs"], nodes=nodes,
                                                                     gpus_per_node=gpus, my_gpu=3, d_inter=s["d_inter"],
                                                                     my_node=nodes // 3) for s in sets], trials=4 * nsets))
            put("allgather_reassemble", 2 * m, time_calls(
                [lambda s=s: pccl.pccl_allgather_reassemble(s["out"], src=s["msgs"][1], nodes=nodes, gpus_per_node=gpus)
                 for s in sets], trials=4 * nsets))
            out.append(row)
        del sets
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--sets", type=int, default=4, help="disjoint buffer sets rotated over (cold cache)")
    ap.add_argument("--kernel-launches", type=int, default=24,
                    help="back-to-back launches per call in the kernel timing loops after the timed steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the other four configurations")
    ap.add_argument("--sweep", action="store_true", help="time the kernels over 16 MB - 1 GB messages and 4 - 256 nodes "
                                                         "(the default run covers 64 - 256 MB only)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run plain 256 MB device-to-device copies (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is the single-GPU local path of the collectives; "
              "--gpus %d is not supported (nothing here uses a second GPU)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    dev = "cuda:0"
    pccl.lib()

    w = W.cfg3()
    sets = [AllReduceShare(w, dev, k) for k in range(args.sets)]
    per_call = sets[0].bytes_per_call()
    step_bytes = sum(per_call.values())

    for k in range(args.warmup):
        sets[k % len(sets)].run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        sets[k % len(sets)].run()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # kernel timing loops, independent of --steps: every call back to back between one pair of events on the
    # launch stream; then a few steps with every call bracketed by its own pair (the figure that includes the stall)
    names = ["pccl_hier_pack", "pccl_reduce_scatter_local", "pccl_allgather_reassemble"]
    nl = max(20, args.kernel_launches)
    calls = {}
    for n in names:
        us = back_to_back([s.call(n) for s in sets], launches=nl)
        calls[n] = dict(bytes=per_call[n], launches=nl, back_to_back_us=round(us, 2),
                        GBps=round(per_call[n] / (us * 1e-6) / 1e9, 1),
                        frac_of_peak=round(per_call[n] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4))
    bracketed = {n: [] for n in names}
    for k in range(3 * len(sets)):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        sets[k % len(sets)].run(ev)
        torch.cuda.synchronize()
        for j, n in enumerate(names):
            bracketed[n].append(ev[j].elapsed_time(ev[j + 1]) * 1e3)
    for n in names:
        calls[n]["event_bracketed_us"] = round(float(np.mean(bracketed[n][len(sets):])), 2)   # first round: warm-up
    perm_us = 0.5 * (calls["pccl_hier_pack"]["back_to_back_us"] + calls["pccl_allgather_reassemble"]["back_to_back_us"])
    achieved = per_call["pccl_hier_pack"] / (perm_us * 1e-6) / 1e9
    roofline = dict(kernel="k_permute (pccl_hier_pack / pccl_allgather_reassemble, 256 MB each)",
                    bound="hbm", achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4), traffic=PROFILED_PERMUTE_TRAFFIC_BYTES,
                    traffic_source="profiles/k_permute_256MB_16x8.txt (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; not measured in this run)",
                    algorithmic_bytes_per_launch=per_call["pccl_hier_pack"], avg_launch_us=round(perm_us, 2),
                    launches=2 * nl, timing="HIP events around back-to-back launches on the launch stream, rotating buffer sets",
                    event_bracketed_frac=round(per_call["pccl_hier_pack"] / (0.5 * (
                        calls["pccl_hier_pack"]["event_bracketed_us"] + calls["pccl_allgather_reassemble"]["event_bracketed_us"])
                        * 1e-6) / 1e9 / HBM_PEAK_GBS, 4))
    red = calls["pccl_reduce_scatter_local"]
    roofline["reduce"] = dict(kernel="k_share_fused: phase 1 (8 x 32 MB) and phase 2 (16 x 2 MB), one call, one launch",
                              bound="hbm", achieved=red["GBps"], peak=HBM_PEAK_GBS, unit="GB/s", frac=red["frac_of_peak"])

    # parity of the timed configuration + CPU baseline: the oracle on the very same buffers
    cpu_baseline, parity = None, None
    if not args.no_cpu_baseline:
        s0 = sets[0]
        s0.run()
        torch.cuda.synchronize()
        host = s0.host_inputs()
        got = [to_np(s0.packed), to_np(s0.partial), to_np(s0.shard), to_np(s0.out)]
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 50:
            c0 = time.perf_counter()
            want = s0.oracle_step(host, nthreads=1)
            t_cpu += time.perf_counter() - c0
            reps += 1
        parity = all(g.tobytes() == np.ascontiguousarray(x).tobytes() for g, x in zip(got, want))
        cpu_baseline = dict(value=round(step_bytes * reps / t_cpu / 1e9, 3), unit="GB/s", cores=1, kind="oracle",
                            sample="%d whole steps of the same workload (pack, two-level reduce, reassemble), "
                                   "%.1f s, single thread of %d host cores" % (reps, t_cpu, os.cpu_count() or 0),
                            ms_per_step=round(t_cpu / reps * 1e3, 1))
        # the same oracle with its element loops split over the box's share of host cores (the byte
        # copies of its permutations stay on one thread); a second reported baseline, about 5 s
        nthr = min(16, os.cpu_count() or 1)
        reps2, t2 = 0, 0.0
        while t2 < 5.0 and reps2 < 50:
            c0 = time.perf_counter()
            want2 = s0.oracle_step(host, nthreads=nthr)
            t2 += time.perf_counter() - c0
            reps2 += 1
        parity = parity and all(np.ascontiguousarray(a).tobytes() == np.ascontiguousarray(b).tobytes()
                                for a, b in zip(want, want2))
        cpu_baseline["all_threads"] = dict(value=round(step_bytes * reps2 / t2 / 1e9, 3), unit="GB/s", cores=nthr,
                                           ms_per_step=round(t2 / reps2 * 1e3, 1),
                                           sample="%d whole steps, %.1f s" % (reps2, t2))
        # warm numbers, labelled: the same buffer set over and over (the 256 MB last-level cache holds part of it)
        warm = {}
        for name in ("pccl_hier_pack", "pccl_reduce_scatter_local"):
            us = back_to_back([s0.call(name)], launches=20)
            warm[name] = dict(back_to_back_us=round(us, 2), GBps=round(per_call[name] / (us * 1e-6) / 1e9, 1))
        calls["warm_same_buffers"] = warm
    del sets
    torch.cuda.empty_cache()

    fused = None if args.no_others else fused_leg(dev, args.steps, args.warmup)
    if fused is not None:
        fused["speedup_vs_three_call_step"] = round(ms_per_step / fused["ms_per_step"], 3)
    torch.cuda.empty_cache()
    sweep = size_sweep(dev, (16, 32, 64, 128, 256, 512, 1024) if args.sweep else (64, 128, 256))
    others = None if args.no_others else other_workloads(dev)
    scale = scale_sweep(dev) if args.sweep else None
    if args.calibration_copy:
        a = torch.empty(256 * MB, dtype=torch.uint8, device=dev)
        b = torch.ones(256 * MB, dtype=torch.uint8, device=dev)
        for _ in range(5):
            a.copy_(b)
        torch.cuda.synchronize()

    out = {
        "metric": "achieved HBM GB/s (and % of peak) for local reduce + hier permute, 64\u2013256 MB",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "config": {"workload": w.name + ": pack 256 MB + two-level reduce (8 x 32 MB, 16 x 2 MB) + reassemble 256 MB",
                   "nodes": w.nodes, "gpus_per_node": w.gpus, "message_MB": w.ranks * w.chunk * w.esize // MB,
                   "accumulate": "f32", "algorithmic_bytes_per_step": step_bytes, "buffer_sets": args.sets,
                   "kernel_events_in_timed_region": False, "kernel_timing_launches_per_call": nl},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "parity_vs_oracle": parity,
        "calls": calls, "fused_step": fused, "size_sweep": sweep, "other_workloads": others, "scale_sweep": scale,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
