"""The LDS-staged two-level reduction where its whole tiles of whole element slices keep loads in
flight across tile boundaries and chain half a tile behind them (the nodes past the last whole
tile and a ragged last slice take the plain loop; PCCL_TWO_LEVEL_PIPE=0 keeps the plain loop
throughout): both forms against the oracle, bit for bit."""
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


@pytest.fixture(params=["piped", "plain"])
def pipe(request, monkeypatch):
    if request.param == "plain":
        monkeypatch.setenv("PCCL_TWO_LEVEL_PIPE", "0")
    return request.param


def _sources(nsrc, count, dtype, seed):
    """nsrc chunks in shuffled slots of one arena: the pointer array is not monotone."""
    host = W.normal(nsrc * count, seed, 1.0, "cpu", dtype)
    arena = host.to(DEV)
    order = W.shuffled_slot_order(nsrc, seed)
    dev = [arena[order[s] * count:(order[s] + 1) * count] for s in range(nsrc)]
    cpu = [to_np(host[order[s] * count:(order[s] + 1) * count]) for s in range(nsrc)]
    return arena, dev, cpu


# a tile = 16 wavefronts x (nodes per wavefront: 8 for up to 8 fp32 sources per node, 2 for 16), a slice =
# 64 fp32: first shapes made of whole tiles and slices only, then the ragged ones
@pytest.mark.parametrize("out_dt", [F32, BF16])
@pytest.mark.parametrize("nodes,gpus,count,npt4", [
    (128, 1, 192, False), (256, 2, 128, False), (128, 4, 64, False), (256, 8, 256, False), (384, 8, 64, False),
    (128, 8, 4096, False), (64, 8, 128, True), (192, 8, 64, True), (32, 16, 64, False), (96, 16, 128, False),
    # whole tiles followed by a partial one, a ragged last slice, fewer nodes than a tile, fewer elements than a slice
    (133, 8, 64 * 3 + 7, False), (255, 2, 100, False), (257, 4, 64, False), (127, 8, 128, False), (300, 1, 5, False),
    (70, 8, 200, True), (40, 16, 130, False)])
def test_two_level_ptrs_shapes(pipe, monkeypatch, out_dt, nodes, gpus, count, npt4):
    print("case", pipe, out_dt, nodes, gpus, count, npt4, flush=True)
    monkeypatch.setenv("PCCL_FORCE_TWO_LEVEL_KERNEL", "lds")
    if npt4:
        monkeypatch.setenv("PCCL_TWO_LEVEL_NPT", "4")
    pccl.diag_reload_env()
    arena, dev, cpu = _sources(nodes * gpus, count, F32, seed=nodes * 13 + gpus + count)
    ptrs = pccl.device_pointer_array(dev)
    dst = Guarded(count, out_dt)
    pccl.pccl_local_reduce_ptrs_two_level(dst.view, ptrs, nodes, gpus, count, F32)
    torch.cuda.synchronize()
    want = oracle.two_level_reduce(cpu, nodes, gpus, ODT[out_dt])
    assert same_bits(to_np(dst.view), want), first_diff(to_np(dst.view), want)
    dst.check()


def test_two_level_ptrs_average(pipe, monkeypatch):
    monkeypatch.setenv("PCCL_FORCE_TWO_LEVEL_KERNEL", "lds")
    pccl.diag_reload_env()
    nodes, gpus, count = 128, 8, 320
    arena, dev, cpu = _sources(nodes * gpus, count, F32, seed=99)
    dst = Guarded(count, F32)
    pccl.pccl_local_reduce_ptrs_two_level(dst.view, pccl.device_pointer_array(dev), nodes, gpus, count, F32, average=True)
    torch.cuda.synchronize()
    want = oracle.two_level_reduce(cpu, nodes, gpus, oracle.F32, average=True)
    assert same_bits(to_np(dst.view), want), first_diff(to_np(dst.view), want)
    dst.check()


# a flat sum sent through the same kernel (one source per "node"): strided sources, where 16-bit
# ones on 32-bit words qualify as well (tiles of 64 sources, slices of 128 elements)
@pytest.mark.parametrize("in_dt,out_dt,nsrc,count,pad", [
    (F32, F32, 128, 128, 0), (F32, BF16, 256, 64, 64), (BF16, BF16, 64, 256, 0), (BF16, F32, 128, 128, 128),
    (F16, F16, 192, 128, 0), (BF16, BF16, 64, 128, 1),   # pad 1: rows start in mid-word, so the plain loop runs
    (F32, F32, 300, 77, 3), (BF16, BF16, 150, 300, 2)])
def test_flat_strided_through_two_level_kernel(pipe, monkeypatch, in_dt, out_dt, nsrc, count, pad):
    print("case", pipe, in_dt, out_dt, nsrc, count, pad, flush=True)
    monkeypatch.setenv("PCCL_FORCE_FLAT_KERNEL", "two-level")
    pccl.diag_reload_env()
    host = W.normal(nsrc * (count + pad), nsrc + count, 1.0, "cpu", in_dt).view(nsrc, count + pad)
    src = host.to(DEV)[:, :count]
    dst = Guarded(count, out_dt)
    pccl.pccl_local_reduce(dst.view, src)
    torch.cuda.synchronize()
    want = oracle.flat_reduce([to_np(host[s, :count]) for s in range(nsrc)], ODT[out_dt])
    assert same_bits(to_np(dst.view), want), first_diff(to_np(dst.view), want)
    dst.check()


@pytest.mark.parametrize("my_node", [0, 77, 127])
def test_phase2_own_slot_through_two_level_kernel(pipe, monkeypatch, my_node):
    """Phase 2 over received chunks (a pointer array whose slot my_node is replaced by the own partial
    row) as a launch of its own through this kernel: the replacement happens when the addresses are
    used, a tile after they were fetched."""
    monkeypatch.setenv("PCCL_FORCE_FLAT_KERNEL", "two-level")
    monkeypatch.setenv("PCCL_SHARE_LAUNCHES", "2")
    pccl.diag_reload_env()
    nodes, gpus, chunk = 128, 2, 192
    x_h = W.normal(gpus * nodes * chunk, 5 + my_node, 1.0, "cpu", F32).view(gpus, nodes, chunk)
    inter_h = W.normal(nodes * chunk, 6 + my_node, 1.0, "cpu", F32).view(nodes, chunk)
    x, inter = x_h.to(DEV), inter_h.to(DEV)
    # the own slot of the table points at memory no kernel may read: a guard band checks nothing is written
    d_inter = pccl.device_pointer_array([inter[n] for n in range(nodes)])
    shard, partial = Guarded(chunk, F32), Guarded(nodes * chunk, F32)
    pccl.pccl_reduce_scatter_local(shard.view, partial.view, x, d_inter=d_inter, my_node=my_node)
    torch.cuda.synchronize()
    want_s, want_p = oracle.reduce_scatter_local(to_np(x_h), my_node=my_node,
                                                 inter=[to_np(inter_h[n]) for n in range(nodes)])
    assert same_bits(to_np(shard.view), want_s), first_diff(to_np(shard.view), want_s)
    assert same_bits(to_np(partial.view), want_p.reshape(-1))
    shard.check()
    partial.check()


@pytest.mark.parametrize("dtype,nsrc,count,odd", [
    (F32, 128, 16384, ()), (F32, 2048, 1024, ()), (F32, 300, 25600, ()), (F32, 1000, 999, ()), (F32, 256, 65536, ()),
    (F32, 127, 4096, ()), (BF16, 128, 32768, ()), (BF16, 2048, 1024, ()), (BF16, 300, 2000, (290,)), (F16, 256, 16384, (7, 200)),
    (BF16, 127, 4096, ()), (BF16, 512, 65536, ())])
def test_flat_ptrs_many_short_sources(pipe, dtype, nsrc, count, odd):
    """The kernel chooser sends flat sums of many short sources through this kernel (one source per
    node): whatever it picks, the bits are the flat order's."""
    print("case", pipe, dtype, nsrc, count, odd, flush=True)
    pccl.diag_reload_env()
    arena, dev, cpu = _sources_some_mid_word(nsrc, count, dtype, seed=nsrc + count, odd=set(odd))
    dst = Guarded(count, dtype)
    pccl.pccl_local_reduce_ptrs(dst.view, pccl.device_pointer_array(dev), count, dtype)
    torch.cuda.synchronize()
    want = oracle.flat_reduce(cpu, ODT[dtype])
    assert same_bits(to_np(dst.view), want), first_diff(to_np(dst.view), want)
    dst.check()


def _sources_some_mid_word(nsrc, count, dtype, seed, odd):
    """As _sources, but the sources whose index is in `odd` start one 16-bit element into their slot:
    in the middle of a 32-bit word."""
    slot = count + 2
    host = W.normal(nsrc * slot, seed, 1.0, "cpu", dtype)
    arena = host.to(DEV)
    order = W.shuffled_slot_order(nsrc, seed)
    lo = [order[s] * slot + (1 if s in odd else 0) for s in range(nsrc)]
    return arena, [arena[a:a + count] for a in lo], [to_np(host[a:a + count]) for a in lo]


# tiles of 64 nodes for 16-bit sources: the block leaves the in-flight loop at the first tile that holds
# a source in mid-word (tile 0: never enters it; none: never leaves it)
@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("odd", [(), (0,), (3,), (64 * 8 + 5,), (130 * 8,), (255 * 8 + 7,), (70 * 8, 200 * 8 + 1)])
def test_two_level_ptrs_16_bit_sources_vote_on_alignment(pipe, monkeypatch, dtype, odd):
    print("case", pipe, dtype, odd, flush=True)
    monkeypatch.setenv("PCCL_FORCE_TWO_LEVEL_KERNEL", "lds")
    pccl.diag_reload_env()
    nodes, gpus, count = 256, 8, 256 + 128
    arena, dev, cpu = _sources_some_mid_word(nodes * gpus, count, dtype, seed=len(odd) * 17 + 3, odd=set(odd))
    dst = Guarded(count, dtype)
    pccl.pccl_local_reduce_ptrs_two_level(dst.view, pccl.device_pointer_array(dev), nodes, gpus, count, dtype)
    torch.cuda.synchronize()
    want = oracle.two_level_reduce(cpu, nodes, gpus, ODT[dtype])
    assert same_bits(to_np(dst.view), want), first_diff(to_np(dst.view), want)
    dst.check()


@pytest.mark.parametrize("odd", [(), (1,), (130,), (255,)])
def test_flat_ptrs_16_bit_through_two_level_kernel(pipe, monkeypatch, odd):
    monkeypatch.setenv("PCCL_FORCE_FLAT_KERNEL", "two-level")
    pccl.diag_reload_env()
    nsrc, count = 256, 512
    arena, dev, cpu = _sources_some_mid_word(nsrc, count, BF16, seed=41 + len(odd), odd=set(odd))
    dst = Guarded(count, BF16)
    pccl.pccl_local_reduce_ptrs(dst.view, pccl.device_pointer_array(dev), count, BF16)
    torch.cuda.synchronize()
    want = oracle.flat_reduce(cpu, oracle.BF16)
    assert same_bits(to_np(dst.view), want), first_diff(to_np(dst.view), want)
    dst.check()
