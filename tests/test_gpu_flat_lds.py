"""The LDS-staged flat sum (phase 2 at large node counts) against the oracle, forced through
PCCL_FORCE_FLAT_KERNEL so that shapes the chooser would hand to another kernel run through it
too: source counts around the tile sizes of both block shapes, ragged element counts, every
dtype pair, misaligned sources and outputs, pointer arrays with the caller's own slot
overridden, and op = average."""
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


_np = to_np                                               # fp16 travels as numpy float16, bf16 as uint16 bit patterns


def _out(n, dtype, offset=0):
    """A guarded output and its typed view (the guard poisons 16-bit types through the bf16 pattern)."""
    g = Guarded(n, dtype if dtype != F16 else BF16, offset_elems=offset)
    return g, (g.view.view(dtype) if dtype == F16 else g.view)


@pytest.fixture(autouse=True)
def _force_flat(monkeypatch):
    monkeypatch.setenv("PCCL_FORCE_FLAT_KERNEL", "flat")
    pccl.diag_reload_env()


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
@pytest.mark.parametrize("nsrc", [1, 2, 7, 8, 9, 31, 32, 33, 63, 64, 65, 127, 128, 129, 257, 300])
def test_strided_sources(dtype, nsrc):
    for count in (1, 63, 127, 128, 129, 1000, 4099):
        host = W.normal(nsrc * count, nsrc * 7 + count, 1.0, "cpu", dtype).view(nsrc, count)
        dst, view = _out(count, dtype)
        pccl.pccl_local_reduce(view, host.to(DEV))
        torch.cuda.synchronize()
        want = oracle.flat_reduce([_np(host[s]) for s in range(nsrc)], ODT[dtype])
        assert same_bits(_np(view), want), (count, first_diff(_np(view), want))
        dst.check()


@pytest.mark.parametrize("in_dt,out_dt", [(BF16, F32), (F32, BF16), (F16, F32), (F32, F16)])
def test_mixed_dtype_pairs_and_average(in_dt, out_dt):
    for nsrc, count in ((40, 777), (130, 129)):
        host = W.normal(nsrc * count, 5, 1.0, "cpu", in_dt).view(nsrc, count)
        for average in (False, True):
            dst, view = _out(count, out_dt)
            pccl.pccl_local_reduce(view, host.to(DEV), average=average)
            torch.cuda.synchronize()
            want = oracle.flat_reduce([_np(host[s]) for s in range(nsrc)], ODT[out_dt], average=average)
            assert same_bits(_np(view), want), (nsrc, count, average)
            dst.check()


@pytest.mark.parametrize("dtype", [BF16, F32])
def test_pointer_array_misaligned_sources_and_output(dtype):
    nsrc, count = 70, 1537
    host = W.normal(nsrc * (count + 3), 11, 1.0, "cpu", dtype).view(nsrc, count + 3)
    dev = host.to(DEV)
    for off in (0, 1):                                    # sources one element off 4-byte alignment
        srcs = [dev[s, off:off + count] for s in range(nsrc)]
        ptrs = pccl.device_pointer_array(srcs)
        for dst_off in (0, 1):
            dst = Guarded(count, dtype, offset_elems=dst_off)
            pccl.pccl_local_reduce_ptrs(dst.view, ptrs, count, dtype)
            torch.cuda.synchronize()
            want = oracle.flat_reduce([_np(host[s, off:off + count]) for s in range(nsrc)], ODT[dtype])
            assert same_bits(_np(dst.view), want), (off, dst_off)
            dst.check()


@pytest.mark.parametrize("nodes", [24, 100])
def test_phase_two_of_a_share_with_received_chunks(nodes):
    gpus, c, my_node = 2, 2000 + 3, 5
    x_h = W.normal(gpus * nodes * c, 21, 1.0, "cpu", BF16).view(gpus, nodes, c)
    inter_h = W.normal(nodes * c, 22, 1.0, "cpu", BF16).view(nodes, c)
    inter = inter_h.to(DEV)
    slots = [inter[k] for k in range(nodes)]
    d_inter = pccl.device_pointer_array(slots)
    d_inter[my_node] = 0x10                                # never dereferenced: the partial's own row is used
    shard, partial = Guarded(c, BF16), Guarded(nodes * c, BF16)
    pccl.pccl_reduce_scatter_local(shard.view, partial.view, x_h.to(DEV), d_inter=d_inter, my_node=my_node, average=True)
    torch.cuda.synchronize()
    ws, wp = oracle.reduce_scatter_local(to_np(x_h), my_node=my_node, inter=[to_np(inter_h[k]) for k in range(nodes)],
                                         average=True)
    assert same_bits(to_np(shard.view), ws) and same_bits(to_np(partial.view), wp.reshape(-1))
    shard.check()
    partial.check()


@pytest.mark.parametrize("nsrc", [40, 200])
def test_launch_split_over_x_and_z(monkeypatch, nsrc):
    """A tiny x extent makes a small problem take the x/z-split launch that only buffers of tens of
    GiB would otherwise take: blocks past the last slice must leave, every slice must be summed once."""
    monkeypatch.setenv("PCCL_GRID_X_LIMIT", "4096")
    pccl.diag_reload_env()
    count = 100003
    host = W.normal(nsrc * count, 31, 1.0, "cpu", BF16).view(nsrc, count)
    dst, view = _out(count, BF16)
    pccl.pccl_local_reduce(view, host.to(DEV))
    torch.cuda.synchronize()
    want = oracle.flat_reduce([_np(host[s]) for s in range(nsrc)], ODT[BF16])
    assert same_bits(_np(view), want), first_diff(_np(view), want)
    dst.check()


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
def test_special_values(dtype):
    """Subnormals are kept, -0 survives when every source holds it, infinities propagate, NaN stays NaN."""
    nsrc = 40
    col = {F32: [1e-45, -0.0, float("inf"), 3e-39, float("nan"), -1e-40, 3.0e38, 1.0],
           BF16: [1e-40, -0.0, float("inf"), 3e-39, float("nan"), -1e-40, 3.0e38, 1.0],
           F16: [6e-8, -0.0, float("inf"), 3e-6, float("nan"), -6e-8, 6.0e4, 1.0]}[dtype]
    host = torch.tensor(col, dtype=torch.float32).to(dtype).repeat(nsrc, 40)        # 320 elements per source
    host[1::2, 2::8] = 1.0                                                           # inf + finite stays inf
    host[3, 7::8] = float("-inf")                                                    # finite ... + -inf
    dst, view = _out(host.shape[1], dtype)
    pccl.pccl_local_reduce(view, host.to(DEV))
    torch.cuda.synchronize()
    want = oracle.flat_reduce([_np(host[s]) for s in range(nsrc)], ODT[dtype])
    got = _np(view)
    wf = want.astype(np.float32) if dtype == F16 else (want if dtype == F32 else (want.astype(np.uint32) << 16).view(np.float32))
    gf = got.astype(np.float32) if dtype == F16 else (got if dtype == F32 else (got.astype(np.uint32) << 16).view(np.float32))
    nan = np.isnan(wf)
    assert nan.any() and np.isinf(wf).any() and np.array_equal(np.isnan(gf), nan)
    assert same_bits(got[~nan], want[~nan]), first_diff(got[~nan], want[~nan])
    assert np.signbit(gf[1]) and gf[1] == 0.0                                        # -0 + -0 + ... = -0
    dst.check()


@pytest.mark.parametrize("mode", ["0", "1"])
@pytest.mark.parametrize("tiny_grid", [False, True])
def test_slice_order_and_load_kind(monkeypatch, mode, tiny_grid):
    """Slices dealt XCD-major with cached loads (1, the default) or linearly with streaming loads
    (0): the same sums; with a tiny x extent the XCD-major launch is also rounded up over x and z."""
    monkeypatch.setenv("PCCL_FLAT_LOCAL", mode)
    pccl.diag_reload_env()
    if tiny_grid:
        monkeypatch.setenv("PCCL_GRID_X_LIMIT", "4096")
        pccl.diag_reload_env()
    for nsrc, count, dtype in ((40, 100003, BF16), (130, 1000, F32), (17, 64 * 9 + 1, BF16), (300, 127, F16)):
        host = W.normal(nsrc * (count + 1), 41, 1.0, "cpu", dtype)[: nsrc * count].view(nsrc, count)
        dst, view = _out(count, dtype)
        pccl.pccl_local_reduce(view, host.to(DEV))
        torch.cuda.synchronize()
        want = oracle.flat_reduce([_np(host[s]) for s in range(nsrc)], ODT[dtype])
        assert same_bits(_np(view), want), (nsrc, count, first_diff(_np(view), want))
        dst.check()
