"""pccl_reduce_scatter_local with received inter-node chunks runs both phases in ONE launch (the
own node's row of the partial goes straight on into phase 2); PCCL_SHARE_LAUNCHES=2 keeps one
launch per phase.  Both forms against the oracle, bit for bit: shard and the whole partial."""
import pytest
import torch

import oracle
import paper_2504_18658_amd as pccl
from paper_2504_18658_amd import workloads as W
from util import Guarded, first_diff, same_bits, to_np

pytestmark = pytest.mark.gpu

DEV = "cuda"
F32, BF16, F16 = torch.float32, torch.bfloat16, torch.float16


@pytest.fixture(params=["one launch", "launch per phase", "chooser"])
def launches(request, monkeypatch):
    # "1" takes the one-launch form wherever it exists (the chooser leaves small messages at many
    # nodes to a launch per phase), "2" never
    if request.param != "chooser":
        monkeypatch.setenv("PCCL_SHARE_LAUNCHES", "1" if request.param == "one launch" else "2")
        pccl.diag_reload_env()
    return request.param


def _run(dtype, nodes, gpus, chunk, my_node, seed, average=False, piece_pad=0, off=0, static=False):
    x_h = W.normal(gpus * (nodes * chunk + piece_pad), seed, 1.0, "cpu", dtype).view(gpus, nodes * chunk + piece_pad)
    inter_h = W.normal(nodes * (chunk + 3), seed + 1, 1.0, "cpu", dtype).view(nodes, chunk + 3)
    x = x_h.to(DEV)[:, : nodes * chunk].view(gpus, nodes, chunk) if piece_pad == 0 else None
    xd = x_h.to(DEV)
    if x is None:
        x = xd.as_strided((gpus, nodes, chunk), (nodes * chunk + piece_pad, chunk, 1))
    inter = inter_h.to(DEV)
    d_inter = pccl.device_pointer_array([inter[n, :chunk] for n in range(nodes)])
    g16 = dtype == F16
    shard = torch.empty(chunk, dtype=dtype, device=DEV) if g16 else Guarded(chunk, dtype, offset_elems=off)
    partial = torch.empty(nodes * chunk, dtype=dtype, device=DEV) if g16 else Guarded(nodes * chunk, dtype, offset_elems=off)
    sv = shard if g16 else shard.view
    pv = partial if g16 else partial.view
    if static:
        pccl.pccl_reduce_scatter_local_static(sv, x, d_inter=d_inter, my_node=my_node, average=average)
    else:
        pccl.pccl_reduce_scatter_local(sv, pv, x, d_inter=d_inter, my_node=my_node, average=average)
    torch.cuda.synchronize()
    if not g16:
        shard.check()
        partial.check()
    xs = to_np(x_h[:, : nodes * chunk].reshape(gpus, nodes, chunk))
    want_s, want_p = oracle.reduce_scatter_local(xs, my_node=my_node, inter=[to_np(inter_h[n, :chunk]) for n in range(nodes)],
                                                 average=average)
    assert same_bits(to_np(sv), want_s), first_diff(to_np(sv), want_s)
    if not static:
        assert same_bits(to_np(pv), want_p.reshape(-1)), first_diff(to_np(pv), want_p.reshape(-1))


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
@pytest.mark.parametrize("nodes", [1, 2, 3, 8, 16, 17, 33, 130])
@pytest.mark.parametrize("gpus", [1, 2, 4, 8, 16, 5])
def test_share_shapes(launches, dtype, nodes, gpus):
    print("share", launches, dtype, nodes, gpus, flush=True)
    for chunk, my_node in ((1, 0), (1000, nodes - 1), (4096 * 2 + 5, nodes // 2)):
        _run(dtype, nodes, gpus, chunk, my_node, seed=nodes * 100 + gpus * 7 + chunk)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_share_unaligned_and_strided(launches, dtype):
    _run(dtype, 4, 8, 2049, 2, seed=5, off=1)                  # shard and partial off 16 bytes, odd chunk
    _run(dtype, 16, 8, 1000, 15, seed=6, piece_pad=40)         # pieces further apart than their size
    _run(dtype, 8, 4, 777, 0, seed=7, off=3, average=True)


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
def test_share_average(launches, dtype):
    _run(dtype, 16, 8, 5000, 7, seed=8, average=True)


def test_share_many_nodes_beyond_the_chooser_threshold(launches):
    """128 x 8 ranks with 64 KB chunks (a 64 MB bf16 message: the chooser picks a launch per phase)
    and with 160 KB chunks (160 MB: one launch), own node first, in the middle of a round, last."""
    for chunk, my_node in ((32768, 0), (81920, 37), (81920 + 8, 127)):
        _run(BF16, 128, 8, chunk, my_node, seed=40 + my_node)


def test_static_share_takes_the_same_path(launches):
    _run(BF16, 16, 8, 3000 + 8, 9, seed=9, static=True)
    _run(F32, 3, 2, 100, 1, seed=10, static=True, average=True)


# ---- the same straight from rank-order messages (pccl_reduce_scatter_local_unpacked with received chunks)
def _run_unpacked(dtype, nodes, gpus, chunk, my_node, my_gpu, seed, average=False, msg_pad=0, off=0, pointers=False):
    n = nodes * gpus * chunk
    m_h = W.normal(gpus * (n + msg_pad), seed, 1.0, "cpu", dtype).view(gpus, n + msg_pad)
    inter_h = W.normal(nodes * (chunk + 3), seed + 1, 1.0, "cpu", dtype).view(nodes, chunk + 3)
    md = m_h.to(DEV)
    msgs = md[:, :n]
    inter = inter_h.to(DEV)
    d_inter = pccl.device_pointer_array([inter[k, :chunk] for k in range(nodes)])
    g16 = dtype == F16
    shard = torch.empty(chunk, dtype=dtype, device=DEV) if g16 else Guarded(chunk, dtype, offset_elems=off)
    partial = torch.empty(nodes * chunk, dtype=dtype, device=DEV) if g16 else Guarded(nodes * chunk, dtype, offset_elems=off)
    sv = shard if g16 else shard.view
    pv = partial if g16 else partial.view
    if pointers:
        pccl.pccl_reduce_scatter_local_unpacked(sv, pv, d_msgs=pccl.device_pointer_array([msgs[g] for g in range(gpus)]),
                                                d_inter=d_inter, nodes=nodes, gpus_per_node=gpus, my_node=my_node,
                                                my_gpu=my_gpu, average=average)
    else:
        pccl.pccl_reduce_scatter_local_unpacked(sv, pv, msgs=msgs, d_inter=d_inter, nodes=nodes, gpus_per_node=gpus,
                                                my_node=my_node, my_gpu=my_gpu, average=average)
    torch.cuda.synchronize()
    if not g16:
        shard.check()
        partial.check()
    want_s, want_p = oracle.reduce_scatter_local_unpacked(
        [to_np(m_h[g, :n]) for g in range(gpus)], nodes, gpus, my_gpu, my_node=my_node,
        inter=[to_np(inter_h[k, :chunk]) for k in range(nodes)], average=average)
    assert same_bits(to_np(sv), want_s), first_diff(to_np(sv), want_s)
    assert same_bits(to_np(pv), want_p.reshape(-1)), first_diff(to_np(pv), want_p.reshape(-1))


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
@pytest.mark.parametrize("nodes", [1, 2, 3, 16, 17, 40])
@pytest.mark.parametrize("gpus", [1, 2, 8, 16, 5])
def test_unpacked_share_shapes(launches, dtype, nodes, gpus):
    print("unpacked share", launches, dtype, nodes, gpus, flush=True)
    for chunk, my_node, my_gpu in ((1, 0, 0), (1000, nodes - 1, gpus - 1), (2048 * 2 + 5, nodes // 2, gpus // 2),
                                   (4096, nodes // 3, 0)):
        _run_unpacked(dtype, nodes, gpus, chunk, my_node, my_gpu, seed=nodes * 100 + gpus * 7 + chunk)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_unpacked_share_unaligned_strided_and_pointers(launches, dtype):
    _run_unpacked(dtype, 4, 8, 2049, 2, 3, seed=5, off=1)                 # odd chunk, outputs off 16 bytes
    _run_unpacked(dtype, 16, 8, 1000, 15, 7, seed=6, msg_pad=40)          # messages further apart than their size
    _run_unpacked(dtype, 8, 4, 776, 0, 1, seed=7, off=3, average=True)    # 16-byte chunks, not line-sized
    _run_unpacked(dtype, 8, 8, 4096, 5, 2, seed=8, pointers=True)         # messages through a pointer array: launch per phase


def test_unpacked_share_many_nodes(launches):
    for chunk, my_node in ((8192, 0), (20480, 37), (20480 + 8, 127)):      # 128 x 8: 16 MB and 40 MB messages
        _run_unpacked(BF16, 128, 8, chunk, my_node, 5, seed=60 + my_node)
