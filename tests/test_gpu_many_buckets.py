"""Batches of 64 - 512 buckets (the most the descriptor tables hold): every batched entry point against
the oracle, bucket by bucket, with empty buckets in runs (equal entries in the tile prefix a block
bisects) and sizes from one element to several tiles."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_18658_amd as pccl
from paper_2504_18658_amd import workloads as W
from util import first_diff, same_bits, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda"
F32, BF16 = torch.float32, torch.bfloat16


def _sizes(n, seed):
    rng = np.random.default_rng(seed)
    s = rng.choice([0, 0, 1, 7, 64, 513, 1024, 2049, 5000], size=n).tolist()
    s[0] = 0                    # a leading run of empty buckets, and a trailing one
    s[1] = 0
    s[-1] = 0
    s[n // 2] = 4096 * 3 + 5    # several tiles
    return [int(x) for x in s]


@pytest.mark.parametrize("n", [64, 65, 200, 512])
def test_many_buckets_reduce_scatter_share(n):
    nodes, gpus = 3, 4
    chunks = _sizes(n, n)
    big = W.normal(sum(chunks) * nodes * gpus + 8, n, 1.0, "cpu", BF16)
    big_d = big.to(DEV)
    buckets, hosts, at = [], [], 0
    for c in chunks:
        x_h = big[at:at + gpus * nodes * c].view(gpus, nodes, c)
        x = big_d[at:at + gpus * nodes * c].view(gpus, nodes, c)
        at += gpus * nodes * c
        buckets.append((torch.full((c,), 7.0, dtype=BF16, device=DEV), torch.full((nodes * c,), 7.0, dtype=BF16, device=DEV), x))
        hosts.append(x_h)
    pccl.pccl_reduce_scatter_local_batched(pccl.BucketTable(buckets))
    torch.cuda.synchronize()
    for k, c in enumerate(chunks):
        if c:
            ws, wp = oracle.reduce_scatter_local(to_np(hosts[k]))
            assert same_bits(to_np(buckets[k][0]), ws), (k, c, first_diff(to_np(buckets[k][0]), ws))
            assert same_bits(to_np(buckets[k][1]), wp.reshape(-1)), (k, c)


@pytest.mark.parametrize("n", [65, 300, 512])
def test_many_buckets_share_from_rank_order_messages(n):
    nodes, gpus, my_gpu = 2, 3, 1
    P = nodes * gpus
    chunks = _sizes(n, n + 1)
    buckets, wants = [], []
    for k, c in enumerate(chunks):
        m_h = W.normal(gpus * P * c + 2, 1000 + k, 1.0, "cpu", F32)[: gpus * P * c].view(gpus, P * c)
        buckets.append((torch.zeros(c, dtype=F32, device=DEV), torch.zeros(nodes * c, dtype=F32, device=DEV), m_h.to(DEV)))
        wants.append(oracle.reduce_scatter_local_unpacked([to_np(m_h[g]) for g in range(gpus)], nodes, gpus, my_gpu) if c else None)
    pccl.pccl_reduce_scatter_local_unpacked_batched(pccl.BucketTable(buckets, nodes=nodes), my_gpu)
    torch.cuda.synchronize()
    for k, c in enumerate(chunks):
        if c:
            ws, wp = wants[k]
            assert same_bits(to_np(buckets[k][0]), ws), (k, c, first_diff(to_np(buckets[k][0]), ws))
            assert same_bits(to_np(buckets[k][1]), wp.reshape(-1)), (k, c)


@pytest.mark.parametrize("n", [65, 256, 512])
def test_many_buckets_shuffles(n):
    nodes, gpus = 4, 2
    P = nodes * gpus
    chunk_bytes = [2 * c for c in _sizes(n, n + 2)]
    srcs_h = [W.random_bits16(P * cb // 2 + 8, 50 + k).view(torch.uint8)[: P * cb] for k, cb in enumerate(chunk_bytes)]
    srcs = [s.to(DEV) for s in srcs_h]
    for fn, ref in ((pccl.pccl_allgather_reassemble_batched, oracle.hier_unpack), (pccl.pccl_hier_pack_batched, oracle.hier_pack)):
        dsts = [torch.full((P * cb,), 0x5A, dtype=torch.uint8, device=DEV) for cb in chunk_bytes]
        fn(pccl.PermuteTable(list(zip(dsts, srcs)), nodes, gpus))
        torch.cuda.synchronize()
        for k, cb in enumerate(chunk_bytes):
            if cb:
                want = ref(srcs_h[k].numpy(), nodes, gpus)
                assert same_bits(to_np(dsts[k]), want), (k, cb, first_diff(to_np(dsts[k]), want))


@pytest.mark.parametrize("n", [65, 512])
def test_many_pairs_accumulate(n):
    counts = _sizes(n, n + 3)
    hosts = [(W.normal(c, 300 + k, 1.0, "cpu", BF16), W.normal(c, 900 + k, 1e-2, "cpu", BF16)) for k, c in enumerate(counts)]
    accs = [a.to(DEV) for a, _ in hosts]
    recvs = [r.to(DEV) for _, r in hosts]
    pccl.pccl_accumulate_batched(pccl.AccumulateTable(list(zip(accs, recvs))))
    torch.cuda.synchronize()
    for k, (a, r) in enumerate(hosts):
        if counts[k]:
            want = oracle.accumulate(to_np(a), to_np(r))
            assert same_bits(to_np(accs[k]), want), (k, first_diff(to_np(accs[k]), want))
