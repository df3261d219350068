"""Parity of the fp16 message dtype and of op = average against the CPU oracle, through the
C ABI, bit for bit (NaNs by NaN-ness and sign)."""
import os

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


def _sync():
    torch.cuda.synchronize()


def _draw(n, dtype, seed, scale=1.0):
    return W.normal(n, seed, scale, "cpu", dtype)


def _guarded_out(n, dtype, offset=0):
    # Guarded poisons with an int pattern; fp16 uses the 16-bit one like bf16
    return Guarded(n, dtype if dtype != F16 else BF16, offset_elems=offset)


def _view(g, dtype):
    return g.view.view(dtype) if dtype == F16 else g.view


# ------------------------------------------------------------------------------- fp16
@pytest.mark.parametrize("in_dt,out_dt", [(F16, F16), (F16, F32), (F32, F16)])
@pytest.mark.parametrize("nsrc", [1, 2, 3, 8, 13, 16])
@pytest.mark.parametrize("count", [1, 7, 1000, 4096 * 3 + 5])
def test_f16_local_reduce_matches_oracle(in_dt, out_dt, nsrc, count):
    print("case", in_dt, out_dt, nsrc, count, flush=True)
    host = _draw(nsrc * count, in_dt, 7 * nsrc + count, 8.0).view(nsrc, count)
    dst = _guarded_out(count, out_dt)
    pccl.pccl_local_reduce(_view(dst, out_dt), host.to(DEV))
    _sync()
    want = oracle.flat_reduce([to_np(host[s]) for s in range(nsrc)], ODT[out_dt])
    got = to_np(_view(dst, out_dt))
    assert same_bits(got, want), first_diff(got, want)
    dst.check()


def test_f16_unaligned_and_overflowing_sums():
    count = 1001
    host = _draw(4 * (count + 3), F16, 5, 30000.0)                      # sums overflow to +-inf often
    src = torch.as_strided(host.to(DEV), (4, count), (count + 3, 1), 1)
    dst = _guarded_out(count, F16, offset=1)
    pccl.pccl_local_reduce(_view(dst, F16), src)
    _sync()
    want = oracle.flat_reduce([to_np(src[s]) for s in range(4)])
    got = to_np(_view(dst, F16))
    assert np.isinf(want.astype(np.float32)).any()
    nan = np.isnan(want.astype(np.float32))
    assert np.array_equal(np.isnan(got.astype(np.float32)), nan)
    assert same_bits(got[~nan], want[~nan]), first_diff(got[~nan], want[~nan])
    dst.check()


def test_f16_rounding_exhaustive_on_gpu():
    """Every binary32 pattern through the library's fp32 -> fp16 store (nsrc = 1 converting copy)
    against the oracle; NaNs by NaN-ness and sign."""
    step = 1 << 26
    base = torch.arange(step, dtype=torch.int64, device=DEV)
    dst = torch.empty(step, dtype=F16, device=DEV)
    for start in range(0, 1 << 32, step):
        u = (base + start).to(torch.int32) if start < (1 << 31) else (base + (start - (1 << 32))).to(torch.int32)
        pccl.pccl_local_reduce(dst, u.view(F32).view(1, step))
        _sync()
        got = to_np(dst).view(np.uint16)
        bits = u.cpu().numpy().view(np.uint32)
        want = oracle.f32_to_f16(bits.view(np.float32)).view(np.uint16)
        if (start >> 23) & 0xFF != 0xFF:
            assert same_bits(got, want), (hex(start), first_diff(got, want))
            continue
        nan = (bits & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
        assert same_bits(got[~nan], want[~nan]), hex(start)
        assert np.all((got[nan] & 0x7FFF) > 0x7C00), "NaN must stay NaN"
        assert np.array_equal(got[nan] >> 15, (bits[nan] >> 31).astype(np.uint16)), "NaN keeps its sign"


def test_f16_widening_exhaustive_on_gpu():
    bits = torch.arange(1 << 16, dtype=torch.int32).to(torch.int16).to(DEV)
    dst = torch.empty(1 << 16, dtype=F32, device=DEV)
    pccl.pccl_local_reduce(dst, bits.view(F16).view(1, -1))
    _sync()
    want = oracle.f16_to_f32(bits.cpu().numpy().view(np.uint16))
    got = to_np(dst)
    nan = np.isnan(want)
    assert same_bits(got[~nan], want[~nan])
    assert np.all(np.isnan(got[nan]))


@pytest.mark.parametrize("force", ["stream", "lds"])
@pytest.mark.parametrize("out_dt", [F16, F32])
@pytest.mark.parametrize("nodes,gpus,count", [(4, 8, 1000), (33, 8, 130), (70, 16, 96), (17, 3, 260), (129, 1, 200)])
def test_f16_two_level_ptrs_matches_oracle(force, out_dt, nodes, gpus, count):
    print("case", force, out_dt, nodes, gpus, count, flush=True)
    nsrc = nodes * gpus
    host = _draw(nsrc * count, F16, nsrc + count, 4.0).view(nsrc, count)
    dev = host.to(DEV)
    ptrs = pccl.device_pointer_array([dev[s] for s in range(nsrc)])
    dst = _guarded_out(count, out_dt)
    os.environ["PCCL_FORCE_TWO_LEVEL_KERNEL"] = force
    pccl.diag_reload_env()
    try:
        pccl.pccl_local_reduce_ptrs_two_level(_view(dst, out_dt), ptrs, nodes, gpus, count, F16)
        _sync()
    finally:
        os.environ.pop("PCCL_FORCE_TWO_LEVEL_KERNEL", None)
        pccl.diag_reload_env()
    want = oracle.two_level_reduce([to_np(host[s]) for s in range(nsrc)], nodes, gpus, ODT[out_dt])
    got = to_np(_view(dst, out_dt))
    assert same_bits(got, want), first_diff(got, want)
    dst.check()


@pytest.mark.parametrize("nodes,gpus,chunk", [(2, 2, 3), (4, 8, 1000), (16, 8, 2048 + 8), (3, 5, 333)])
def test_f16_reduce_scatter_local_batched_and_steps(nodes, gpus, chunk):
    x_h = _draw(gpus * nodes * chunk, F16, 99 + chunk, 2.0).view(gpus, nodes, chunk)
    x = x_h.to(DEV)
    partial = torch.empty(nodes * chunk, dtype=F16, device=DEV)
    shard = torch.empty(chunk, dtype=F16, device=DEV)
    pccl.pccl_reduce_scatter_local(shard, partial, x)
    _sync()
    want_shard, want_partial = oracle.reduce_scatter_local(to_np(x_h))
    assert same_bits(to_np(partial), want_partial.reshape(-1)) and same_bits(to_np(shard), want_shard)
    # the same through the batched entry (two buckets, the second a prefix of the first)
    c2 = max(1, chunk // 2)
    x2_h = x_h[:, :, :c2].contiguous()
    p2 = torch.empty(nodes * c2, dtype=F16, device=DEV)
    s2 = torch.empty(c2, dtype=F16, device=DEV)
    p1 = torch.empty_like(partial)
    s1 = torch.empty_like(shard)
    table = pccl.BucketTable([(s1, p1, x), (s2, p2, x2_h.to(DEV))])
    pccl.pccl_reduce_scatter_local_batched(table)
    _sync()
    assert same_bits(to_np(s1), want_shard) and same_bits(to_np(p1), want_partial.reshape(-1))
    ws2, wp2 = oracle.reduce_scatter_local(to_np(x2_h))
    assert same_bits(to_np(s2), ws2) and same_bits(to_np(p2), wp2.reshape(-1))
    # one literal step and a halving replay in fp16
    a_h, r_h = x_h[0].reshape(-1), x_h[1 % gpus].reshape(-1)
    a = a_h.to(DEV).clone()
    pccl.pccl_accumulate(a, r_h.to(DEV))
    _sync()
    assert same_bits(to_np(a), oracle.accumulate(to_np(a_h), to_np(r_h)))


# ------------------------------------------------------------------------------- average
def test_average_hand_cases_on_gpu(golden_dir):
    for line in open(os.path.join(golden_dir, "avg_cases.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        shape, terms, expected = [p.strip() for p in line.split("|")]
        nodes, gpus = map(int, shape.split())
        f = lambda t: float.fromhex(t) if "0x" in t.lower() else float(t)
        vals = np.array([f(t) for t in terms.split()], dtype=np.float32)
        want = np.array([f(expected)], dtype=np.float32)
        src = torch.from_numpy(vals).to(DEV).view(nodes * gpus, 1)
        ptrs = pccl.device_pointer_array([src[k] for k in range(nodes * gpus)])
        for force in ("stream", "lds"):
            dst = torch.empty(1, dtype=F32, device=DEV)
            os.environ["PCCL_FORCE_TWO_LEVEL_KERNEL"] = force
            pccl.diag_reload_env()
            try:
                pccl.pccl_local_reduce_ptrs_two_level(dst, ptrs, nodes, gpus, 1, F32, average=True)
                _sync()
            finally:
                os.environ.pop("PCCL_FORCE_TWO_LEVEL_KERNEL", None)
                pccl.diag_reload_env()
            assert same_bits(to_np(dst), want), (line, force, to_np(dst))
        if nodes == 1:
            dst = torch.empty(1, dtype=F32, device=DEV)
            pccl.pccl_local_reduce(dst, src, average=True)
            _sync()
            assert same_bits(to_np(dst), want), (line, to_np(dst))


@pytest.mark.parametrize("in_dt,out_dt", [(F32, F32), (BF16, BF16), (F16, F16), (BF16, F32), (F32, F16)])
@pytest.mark.parametrize("nsrc", [1, 2, 3, 7, 8, 24])
def test_average_local_reduce_matches_oracle(in_dt, out_dt, nsrc):
    count = 4096 * 2 + 11
    host = _draw(nsrc * count, in_dt, 31 * nsrc, 3.0).view(nsrc, count)
    dst = _guarded_out(count, out_dt)
    pccl.pccl_local_reduce(_view(dst, out_dt), host.to(DEV), average=True)
    _sync()
    want = oracle.flat_reduce([to_np(host[s]) for s in range(nsrc)], ODT[out_dt], average=True)
    got = to_np(_view(dst, out_dt))
    assert same_bits(got, want), first_diff(got, want)
    dst.check()


@pytest.mark.parametrize("divisor", [3, 5, 6, 7, 10, 24])
def test_division_over_random_bit_patterns(divisor):
    """x / divisor for 2^24 random binary32 patterns (x + 0 + ... + 0, so the sum is x itself)."""
    n = 1 << 24
    g = torch.Generator(device=DEV)
    g.manual_seed(1234 + divisor)
    bits = torch.randint(-(1 << 31), (1 << 31) - 1, (n,), generator=g, device=DEV, dtype=torch.int64).to(torch.int32)
    x = bits.view(F32)
    zeros = torch.zeros(n, dtype=F32, device=DEV)
    ptrs = pccl.device_pointer_array([x] + [zeros] * (divisor - 1))
    dst = torch.empty(n, dtype=F32, device=DEV)
    pccl.pccl_local_reduce_ptrs(dst, ptrs, n, F32, average=True)
    _sync()
    xh = to_np(x)
    want = oracle.flat_reduce([xh] + [np.zeros(n, dtype=np.float32)] * (divisor - 1), average=True, nthreads=8)
    got = to_np(dst)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert same_bits(got[~nan], want[~nan]), first_diff(got[~nan], want[~nan])


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
def test_average_in_the_reduce_scatter_entry_points(dtype):
    nodes, gpus, chunk, my_n, my_g = 6, 4, 1000 + 8, 4, 1
    P = nodes * gpus
    x_h = _draw(gpus * nodes * chunk, dtype, 555, 2.0).view(gpus, nodes, chunk)
    inter_h = _draw(nodes * chunk, dtype, 556, 2.0).view(nodes, chunk)
    x, inter = x_h.to(DEV), inter_h.to(DEV)
    d_inter = pccl.device_pointer_array([inter[n] for n in range(nodes)])
    partial = torch.empty(nodes * chunk, dtype=dtype, device=DEV)
    shard = torch.empty(chunk, dtype=dtype, device=DEV)
    pccl.pccl_reduce_scatter_local(shard, partial, x, d_inter=d_inter, my_node=my_n, average=True)
    _sync()
    ws, wp = oracle.reduce_scatter_local(to_np(x_h), my_node=my_n, inter=[to_np(inter_h[n]) for n in range(nodes)],
                                         average=True)
    assert same_bits(to_np(shard), ws), first_diff(to_np(shard), ws)
    assert same_bits(to_np(partial), wp.reshape(-1))
    # self-simulated, batched
    s1, p1 = torch.empty_like(shard), torch.empty_like(partial)
    pccl.pccl_reduce_scatter_local_batched(pccl.BucketTable([(s1, p1, x)]), average=True)
    _sync()
    ws, wp = oracle.reduce_scatter_local(to_np(x_h), average=True)
    assert same_bits(to_np(s1), ws) and same_bits(to_np(p1), wp.reshape(-1))
    # straight from rank-order messages
    msgs_h = _draw(gpus * P * chunk, dtype, 557, 2.0).view(gpus, P * chunk)
    pccl.pccl_reduce_scatter_local_unpacked(shard, partial, msgs=msgs_h.to(DEV), d_inter=d_inter, nodes=nodes,
                                            gpus_per_node=gpus, my_node=my_n, my_gpu=my_g, average=True)
    _sync()
    ws, wp = oracle.reduce_scatter_local_unpacked([to_np(msgs_h[g]) for g in range(gpus)], nodes, gpus, my_g,
                                                  my_node=my_n, inter=[to_np(inter_h[n]) for n in range(nodes)],
                                                  average=True)
    assert same_bits(to_np(shard), ws) and same_bits(to_np(partial), wp.reshape(-1))


@pytest.mark.parametrize("force", ["stream", "lds"])
@pytest.mark.parametrize("in_dt,out_dt", [(F32, F32), (BF16, BF16), (F16, F32)])
def test_average_two_level_ptrs_matches_oracle(force, in_dt, out_dt):
    nodes, gpus, count = 70, 8, 300
    nsrc = nodes * gpus
    host = _draw(nsrc * count, in_dt, 808, 1.0).view(nsrc, count)
    dev = host.to(DEV)
    ptrs = pccl.device_pointer_array([dev[s] for s in range(nsrc)])
    dst = _guarded_out(count, out_dt)
    os.environ["PCCL_FORCE_TWO_LEVEL_KERNEL"] = force
    pccl.diag_reload_env()
    try:
        pccl.pccl_local_reduce_ptrs_two_level(_view(dst, out_dt), ptrs, nodes, gpus, count, in_dt, average=True)
        _sync()
    finally:
        os.environ.pop("PCCL_FORCE_TWO_LEVEL_KERNEL", None)
        pccl.diag_reload_env()
    want = oracle.two_level_reduce([to_np(host[s]) for s in range(nsrc)], nodes, gpus, ODT[out_dt], average=True)
    got = to_np(_view(dst, out_dt))
    assert same_bits(got, want), first_diff(got, want)
    dst.check()
