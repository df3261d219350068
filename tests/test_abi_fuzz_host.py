"""Property test of the host-side argument checks, on machines without a GPU only (a call that
passes the checks would launch on made-up addresses; with no device the launch simply fails
with PCCL_ERR_HIP).  Whatever the arguments, a call returns a status code -- no crash, no
wrap-around in the size arithmetic: a call is only ever accepted when every range it describes
fits the address space."""
import ctypes

import pytest
from hypothesis import given, settings, strategies as st

import paper_2504_18658_amd as pccl
from paper_2504_18658_amd import binding

A = 1 << 20
STATUSES = {pccl.PCCL_OK, pccl.PCCL_ERR_NULL, pccl.PCCL_ERR_INVALID, pccl.PCCL_ERR_UNSUPPORTED, pccl.PCCL_ERR_OVERLAP,
            pccl.PCCL_ERR_HIP, pccl.PCCL_ERR_ADDRESS}
ACCEPTED = {pccl.PCCL_OK, pccl.PCCL_ERR_HIP}          # passed every check (the launch then fails: no device)
SIZE_MAX = (1 << 64) - 1


@pytest.fixture(autouse=True)
def _only_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("host argument fuzzing runs on machines without a GPU")


ptr = st.sampled_from([0, A, 2 * A, 3 * A + 2, 5 * A + 1, 1 << 40, (1 << 63) + A])
size = st.one_of(st.integers(0, 4096), st.sampled_from([1 << 31, (1 << 32) + 6, 1 << 62, (1 << 63) + 8, SIZE_MAX, SIZE_MAX - 1]))
small = st.integers(-2, 70)
count_like = st.one_of(st.integers(-3, 300), st.sampled_from([1 << 15, 65535, 65536, (1 << 31) - 1]))
code = st.integers(-1, 4)


def _es(dt):
    return 4 if dt == pccl.PCCL_F32 else 2


@settings(max_examples=400, deadline=None)
@given(ptr, ptr, size, count_like, size, code, code, code)
def test_local_reduce(dst, src, stride, nsrc, count, in_dt, out_dt, op):
    rc = binding.lib().pccl_local_reduce(dst, src, stride, nsrc, count, in_dt, out_dt, op, None)
    assert rc in STATUSES
    if rc in ACCEPTED:
        assert dst and src and nsrc >= 1 and in_dt in (0, 1, 2) and out_dt in (0, 1, 2) and op in (0, 1)
        assert count * max(_es(in_dt), _es(out_dt)) <= SIZE_MAX
        if nsrc > 1:
            assert stride >= count * _es(in_dt) and (nsrc - 1) * stride + count * _es(in_dt) <= SIZE_MAX


@settings(max_examples=400, deadline=None)
@given(ptr, ptr, count_like, count_like, size, st.sampled_from(["pccl_hier_pack", "pccl_hier_unpack"]))
def test_shuffles(dst, src, nodes, gpus, chunk_bytes, name):
    rc = getattr(binding.lib(), name)(dst, src, nodes, gpus, chunk_bytes, None)
    assert rc in STATUSES
    if rc in ACCEPTED:
        assert dst and src and nodes >= 1 and gpus >= 1
        assert nodes * gpus * chunk_bytes <= SIZE_MAX


@settings(max_examples=400, deadline=None)
@given(ptr, ptr, ptr, size, ptr, count_like, count_like, small, size, code, code)
def test_reduce_scatter_local(shard, partial, intra, stride, d_inter, nodes, gpus, my_node, chunk, dt, op):
    rc = binding.lib().pccl_reduce_scatter_local(shard, partial, intra, stride, d_inter or None, nodes, gpus, my_node, chunk,
                                                 dt, op, None)
    assert rc in STATUSES
    if rc in ACCEPTED:
        assert shard and partial and intra and nodes >= 1 and gpus >= 1 and 0 <= my_node < nodes
        assert dt in (0, 1, 2) and op in (0, 1) and nodes * chunk * _es(dt) <= SIZE_MAX
        if gpus > 1:
            assert stride >= nodes * chunk * _es(dt) and (gpus - 1) * stride + nodes * chunk * _es(dt) <= SIZE_MAX


@settings(max_examples=400, deadline=None)
@given(ptr, ptr, ptr, size, count_like, count_like, small, small, size, code, code)
def test_reduce_scatter_local_unpacked(shard, partial, msgs, stride, nodes, gpus, my_node, my_gpu, chunk, dt, op):
    rc = binding.lib().pccl_reduce_scatter_local_unpacked(shard, partial, msgs, stride, None, None, nodes, gpus, my_node,
                                                          my_gpu, chunk, dt, op, None)
    assert rc in STATUSES
    if rc in ACCEPTED:
        assert shard and partial and msgs and 1 <= nodes <= 65535 and gpus >= 1
        assert 0 <= my_node < nodes and 0 <= my_gpu < gpus and dt in (0, 1, 2) and op in (0, 1)
        msg = nodes * gpus * chunk * _es(dt)
        assert msg <= SIZE_MAX and (gpus == 1 or (stride >= msg and (gpus - 1) * stride + msg <= SIZE_MAX))


@settings(max_examples=300, deadline=None)
@given(ptr, ptr, size, code, code)
def test_accumulate(acc, recv, count, dt, op):
    rc = binding.lib().pccl_accumulate(acc, recv, count, dt, op, None)
    assert rc in STATUSES
    if rc in ACCEPTED:
        assert acc and recv and dt in (0, 1, 2) and op == 0 and count * _es(dt) <= SIZE_MAX


@settings(max_examples=300, deadline=None)
@given(st.lists(st.tuples(ptr, ptr, ptr, size, size), min_size=0, max_size=4), count_like, count_like, small, code, code,
       st.booleans())
def test_batched_shares(rows, nodes, gpus, my_gpu, dt, op, from_messages):
    L = binding.lib()
    n = len(rows)
    host = (pccl.pccl_bucket_t * max(n, 1))(*[pccl.pccl_bucket_t(*r) for r in rows])
    h = ctypes.addressof(host)
    if from_messages:
        rc = L.pccl_reduce_scatter_local_unpacked_batched(A, h, n, nodes, gpus, my_gpu, dt, op, None)
    else:
        rc = L.pccl_reduce_scatter_local_batched(A, h, n, nodes, gpus, dt, op, None)
    assert rc in STATUSES
    if rc in ACCEPTED and any(r[4] for r in rows):
        assert nodes >= 1 and gpus >= 1 and dt in (0, 1, 2) and op in (0, 1)
        for shard, partial, base, stride, chunk in rows:
            if chunk:
                assert shard and partial and base
                src = nodes * chunk * _es(dt) * (gpus if from_messages else 1)
                assert src <= SIZE_MAX and (gpus == 1 or stride >= src)
