"""pccl_reduce_scatter_local_static -- the share for callers that cannot allocate device memory
(the phase-1 result stays in a static device array of the library) -- against
pccl_reduce_scatter_local on the same inputs, through the C ABI: the shards must agree bit
for bit.  Two calls in a row on the one workspace, the second smaller than the first, so that
what the first call left behind must not reach the second's result; then the limit."""
import ctypes

import pytest
import torch

import oracle
import paper_2504_18658_amd as pccl
from paper_2504_18658_amd import workloads as W
from util import Guarded, first_diff, same_bits, to_np

pytestmark = pytest.mark.gpu

DEV = "cuda"
ODT = {torch.float32: oracle.F32, torch.bfloat16: oracle.BF16}


def _both(nodes, gpus, chunk, dtype, seed, my_node, with_inter, average=False):
    """(shard of the static entry point, shard of the existing entry point), raw C ABI calls."""
    L = pccl.lib()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    x = W.uniform_pm1(gpus * nodes * chunk, seed, DEV, dtype).view(gpus, nodes, chunk)
    d_inter, inter = None, None
    if with_inter:
        inter = W.uniform_pm1(nodes * chunk, seed + 1, DEV, dtype).view(nodes, chunk)
        d_inter = pccl.device_pointer_array([inter[j] for j in range(nodes)])
    es = x.element_size()
    got = Guarded(chunk, dtype)
    want = torch.empty(chunk, dtype=dtype, device=DEV)
    partial = torch.empty(nodes * chunk, dtype=dtype, device=DEV)
    dp = None if d_inter is None else ctypes.c_void_p(d_inter.data_ptr())
    code, op = pccl.binding.dtype_code(dtype), pccl.PCCL_AVG if average else pccl.PCCL_SUM
    print("static share", nodes, gpus, chunk, dtype, "inter" if with_inter else "self", flush=True)
    rc = L.pccl_reduce_scatter_local_static(got.view.data_ptr(), x.data_ptr(), nodes * chunk * es, dp, nodes, gpus,
                                            my_node, chunk, code, op, st)
    assert rc == pccl.PCCL_OK, pccl.status_string(rc)
    rc = L.pccl_reduce_scatter_local(want.data_ptr(), partial.data_ptr(), x.data_ptr(), nodes * chunk * es, dp,
                                     nodes, gpus, my_node, chunk, code, op, st)
    assert rc == pccl.PCCL_OK, pccl.status_string(rc)
    torch.cuda.synchronize()
    got.check()
    return to_np(got.view), to_np(want), x, inter


def test_static_share_two_calls_in_a_row_second_smaller():
    # first call: 16 x 8 ranks, ragged chunk (several tiles and a tail), received chunks through d_inter
    a, b, x, inter = _both(16, 8, 70000 + 13, torch.bfloat16, 11, 5, True)
    assert same_bits(a, b), first_diff(a, b)
    # ... and against the oracle, so that both entry points cannot be wrong together
    want, _ = oracle.reduce_scatter_local(to_np(x), my_node=5, inter=[to_np(inter[j]) for j in range(16)])
    assert same_bits(a, want), first_diff(a, want)
    # second call, smaller in every extent: the workspace still holds the first call's partial
    a, b, x, _ = _both(4, 8, 4096 + 24, torch.bfloat16, 12, 2, False)
    assert same_bits(a, b), first_diff(a, b)
    want, _ = oracle.reduce_scatter_local(to_np(x))
    assert same_bits(a, want), first_diff(a, want)
    # a third, fp32 with the average, many nodes (the LDS-staged flat kernel in phase 2)
    a, b, _, _ = _both(64, 4, 1000, torch.float32, 13, 63, True, average=True)
    assert same_bits(a, b), first_diff(a, b)


def test_static_share_at_the_limit_and_beyond():
    # the 256 MB workload's share fills the workspace exactly: 16 x 1 Mi bf16 = 32 MiB of partial
    w = W.cfg3()
    assert w.nodes * w.chunk * 2 == pccl.PCCL_STATIC_SCRATCH_BYTES
    a, b, _, _ = _both(w.nodes, w.gpus, w.chunk, torch.bfloat16, 14, 7, True)
    assert same_bits(a, b), first_diff(a, b)
    # one element more per chunk is refused on the host, before anything is launched
    L = pccl.lib()
    c = w.chunk + 1
    x = torch.zeros(w.gpus * w.nodes * c, dtype=torch.bfloat16, device=DEV)
    out = torch.full((c,), 7.0, dtype=torch.bfloat16, device=DEV)
    rc = L.pccl_reduce_scatter_local_static(out.data_ptr(), x.data_ptr(), w.nodes * c * 2, None, w.nodes, w.gpus, 0,
                                            c, pccl.PCCL_BF16, pccl.PCCL_SUM, None)
    assert rc == pccl.PCCL_ERR_SCRATCH
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    # a smaller call afterwards still works
    a, b, _, _ = _both(2, 2, 300, torch.float32, 15, 1, False)
    assert same_bits(a, b), first_diff(a, b)
