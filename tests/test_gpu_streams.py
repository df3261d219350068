"""The library keeps no state between calls: calls made from several host threads, each on a
stream of its own, run side by side and every result is bit-exact against the oracle; a call
runs on the stream it is given (it sees work queued on that stream before it)."""
import threading

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


def _job(kind, seed):
    """(inputs on host, run(stream) -> outputs on device, want) for one kind of call."""
    if kind == "reduce":
        dtype, odt = BF16, oracle.BF16
        host = W.normal(8 * 70001, seed, 1.0, "cpu", dtype).view(8, 70001)
        dev = host.to(DEV)
        out = torch.empty(70001, dtype=dtype, device=DEV)
        want = oracle.flat_reduce([to_np(host[s]) for s in range(8)], odt)

        def run():
            pccl.pccl_local_reduce(out, dev)
        return run, lambda: to_np(out), want
    if kind == "share":
        n, g, c = 6, 4, 9001
        host = W.normal(g * n * c, seed, 1.0, "cpu", BF16).view(g, n, c)
        dev = host.to(DEV)
        shard = torch.empty(c, dtype=BF16, device=DEV)
        partial = torch.empty(n * c, dtype=BF16, device=DEV)
        ws, wp = oracle.reduce_scatter_local(to_np(host))

        def run():
            pccl.pccl_reduce_scatter_local(shard, partial, dev)
        return run, lambda: np.concatenate([to_np(shard), to_np(partial)]), np.concatenate([ws, wp.reshape(-1)])
    if kind == "pack":
        n, g, cb = 5, 3, 40000 + 16
        gen = torch.Generator()
        gen.manual_seed(seed)
        host = torch.randint(0, 256, (n * g * cb,), generator=gen, dtype=torch.uint8)
        dev = host.to(DEV)
        out = torch.empty_like(dev)
        want = oracle.hier_pack(host.numpy(), n, g)

        def run():
            pccl.pccl_hier_pack(out, dev, n, g)
        return run, lambda: to_np(out), want
    if kind == "accumulate":
        a = W.normal(50003, seed, 1.0, "cpu", F32)
        r = W.normal(50003, seed + 1, 1.0, "cpu", F32)
        acc, recv = a.to(DEV), r.to(DEV)
        state = {"n": 0}

        def run():
            pccl.pccl_accumulate(acc, recv)
            state["n"] += 1

        def want():
            w = to_np(a)
            for _ in range(state["n"]):
                w = oracle.accumulate(w, to_np(r))
            return w
        return run, lambda: to_np(acc), want
    raise ValueError(kind)


def test_calls_from_four_threads_on_four_streams():
    kinds = ["reduce", "share", "pack", "accumulate"]
    jobs = [_job(k, 100 + i) for i, k in enumerate(kinds)]
    streams = [torch.cuda.Stream() for _ in kinds]
    torch.cuda.synchronize()
    errors = []
    start = threading.Barrier(len(kinds))

    def worker(i):
        try:
            start.wait()
            with torch.cuda.stream(streams[i]):
                for _ in range(25):
                    jobs[i][0]()
            streams[i].synchronize()
        except Exception as e:  # noqa: BLE001 - reported by the main thread
            errors.append((kinds[i], repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(len(kinds))]
    for t in threads:
        t.start()
    for t in threads:
        t.join(120)
    assert not any(t.is_alive() for t in threads)
    assert not errors, errors
    torch.cuda.synchronize()
    for kind, (_, got, want) in zip(kinds, jobs):
        w = want() if callable(want) else want
        assert same_bits(got(), w), kind


def test_a_call_is_ordered_after_earlier_work_on_its_stream():
    n = 1 << 22
    side = torch.cuda.Stream()
    src = torch.zeros(2, n, dtype=F32, device=DEV)
    dst = torch.empty(n, dtype=F32, device=DEV)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for k in range(20):                                 # a queue of fills, then the reduce behind them
            src[0].fill_(float(k))
            src[1].fill_(float(2 * k))
        pccl.pccl_local_reduce(dst, src)
        src[0].fill_(-1.0)                                  # queued behind the reduce: must not be seen by it
    side.synchronize()
    assert bool((dst == 57.0).all())
