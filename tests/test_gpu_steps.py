"""Parity of the step-wise reduction entry points (acc += recv, ring and recursive-halving
replays of one rank) against the CPU oracle, through the C ABI, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_18658_amd as pccl
from paper_2504_18658_amd import workloads as W
from util import Guarded, first_diff, same_bits, to_np

pytestmark = pytest.mark.gpu

DEV = "cuda"
F32, BF16 = torch.float32, torch.bfloat16


def _sync():
    torch.cuda.synchronize()


def _guarded_copy(host, offset=0):
    g = Guarded(host.numel(), host.dtype, offset_elems=offset)
    g.view.copy_(host.reshape(-1).to(DEV))
    return g


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("count", [1, 7, 8, 1000, 4096 * 5 + 3, 1 << 20])
@pytest.mark.parametrize("offs", [(0, 0), (1, 0), (0, 3), (1, 1)])
def test_accumulate_matches_oracle(dtype, count, offs):
    print("case", dtype, count, offs, flush=True)
    a = W.normal(count, 17 + count, 1.0, "cpu", dtype)
    r = W.normal(count, 18 + count, 1e-2, "cpu", dtype)
    acc = _guarded_copy(a, offs[0])
    recv = _guarded_copy(r, offs[1])
    pccl.pccl_accumulate(acc.view, recv.view)
    _sync()
    want = oracle.accumulate(to_np(a), to_np(r))
    assert same_bits(to_np(acc.view), want), first_diff(to_np(acc.view), want)
    assert same_bits(to_np(recv.view), to_np(r))      # the received buffer is only read
    acc.check()
    recv.check()


def test_accumulate_hand_cases_on_gpu(golden_dir):
    import os
    a, r, w, b = [], [], [], []
    for line in open(os.path.join(golden_dir, "accumulate_cases.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        dt, x, y, z = [p.strip() for p in line.split("|")]
        f = lambda t: float.fromhex(t) if "0x" in t.lower() else float(t)
        a.append(f(x)); r.append(f(y)); w.append(f(z)); b.append(dt == "bf16")
    for bf in (False, True):
        dt = BF16 if bf else F32
        sel = [k for k in range(len(a)) if b[k] == bf]
        acc = torch.tensor([a[k] for k in sel], dtype=torch.float32).to(dt).to(DEV)
        recv = torch.tensor([r[k] for k in sel], dtype=torch.float32).to(dt).to(DEV)
        want = torch.tensor([w[k] for k in sel], dtype=torch.float32).to(dt)
        pccl.pccl_accumulate(acc, recv)
        _sync()
        assert same_bits(to_np(acc), to_np(want)), (to_np(acc), to_np(want))


def test_accumulate_special_values():
    inf, nan = float("inf"), float("nan")
    for dt in (F32, BF16):
        acc = torch.tensor([inf, -inf, inf, nan, 1.0, -0.0, 3.0e38, 1e-40], dtype=torch.float32).to(dt).to(DEV)
        recv = torch.tensor([1.0, 2.0, -inf, 1.0, nan, 0.0, 3.0e38, 1e-40], dtype=torch.float32).to(dt).to(DEV)
        a0, r0 = to_np(acc), to_np(recv)
        pccl.pccl_accumulate(acc, recv)
        _sync()
        got = acc.float().cpu().numpy()
        want_bits = oracle.accumulate(a0, r0)
        want = oracle.bf16_to_f32(want_bits) if dt == BF16 else want_bits
        assert np.array_equal(np.isnan(got), np.isnan(want))
        ok = ~np.isnan(want)
        assert same_bits(got[ok].astype(np.float32), want[ok].astype(np.float32))


@pytest.fixture(params=["one launch", "launch per step"])
def launches(request, monkeypatch):
    """Both forms of the replays: every step in one launch (the default) and one launch per step."""
    if request.param == "launch per step":
        monkeypatch.setenv("PCCL_STEP_LAUNCHES", "1")
        pccl.diag_reload_env()
    return request.param


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("p,chunk", [(2, 5), (3, 1000), (8, 4096 + 8), (16, 333), (1, 64), (7, 1029), (33, 520)])
def test_ring_local_matches_oracle(dtype, p, chunk, launches):
    print("case", dtype, p, chunk, launches, flush=True)
    for rank in sorted({0, p // 2, p - 1}):
        msg_h = W.uniform_pm1(p * chunk, 31 + p, "cpu", dtype).view(p, chunk)
        recv_h = W.uniform_pm1(max(p - 1, 1) * chunk, 32 + p, "cpu", dtype).view(max(p - 1, 1), chunk)
        msg = _guarded_copy(msg_h)
        recv = _guarded_copy(recv_h)
        pccl.pccl_ring_reduce_scatter_local(msg.view.view(p, chunk), recv.view.view(-1, chunk)[:max(p - 1, 1)], rank)
        _sync()
        want = oracle.ring_rs_local(to_np(msg_h), [to_np(recv_h[s]) for s in range(p - 1)], rank)
        assert same_bits(to_np(msg.view).reshape(p, chunk), want), first_diff(to_np(msg.view), want)
        msg.check()
        recv.check()


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("p,chunk", [(1, 10), (2, 7), (4, 1000), (16, 2048 + 8), (64, 65), (8, 1031), (256, 24)])
def test_halving_local_matches_oracle(dtype, p, chunk, launches):
    print("case", dtype, p, chunk, launches, flush=True)
    for rank in sorted({0, p // 3, p - 1, p // 2}):
        msg_h = W.uniform_pm1(p * chunk, 41 + p, "cpu", dtype).view(p, chunk)
        recv_h = W.uniform_pm1(max(p - 1, 1) * chunk, 42 + p, "cpu", dtype)
        msg = _guarded_copy(msg_h)
        recv = _guarded_copy(recv_h)
        pccl.pccl_halving_reduce_scatter_local(msg.view.view(p, chunk), recv.view[:max(p - 1, 0) * chunk] if p > 1 else recv.view, rank)
        _sync()
        halves, off = [], 0
        t = 0
        while (p >> (t + 1)) >= 1:
            ln = p >> (t + 1)
            halves.append(to_np(recv_h[off * chunk:(off + ln) * chunk]))
            off += ln
            t += 1
        want = oracle.halving_rs_local(to_np(msg_h), halves, rank)
        assert same_bits(to_np(msg.view).reshape(p, chunk), want), first_diff(to_np(msg.view), want)
        msg.check()
        recv.check()


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("off", [1, 3])
def test_ring_and_halving_unaligned_buffers(dtype, off):
    """Buffers that start off a 16-byte boundary take the element-wise capable paths: same bits."""
    p, chunk = 8, 777
    msg_h = W.uniform_pm1(p * chunk, 61, "cpu", dtype).view(p, chunk)
    recv_h = W.uniform_pm1((p - 1) * chunk, 62, "cpu", dtype).view(p - 1, chunk)
    for rank in (0, 5):
        msg = _guarded_copy(msg_h, off)
        recv = _guarded_copy(recv_h, off + 1)
        pccl.pccl_ring_reduce_scatter_local(msg.view.view(p, chunk), recv.view.view(p - 1, chunk), rank)
        _sync()
        want = oracle.ring_rs_local(to_np(msg_h), [to_np(recv_h[s]) for s in range(p - 1)], rank)
        assert same_bits(to_np(msg.view).reshape(p, chunk), want), first_diff(to_np(msg.view), want)
        msg.check()
        msg = _guarded_copy(msg_h, off)
        pccl.pccl_halving_reduce_scatter_local(msg.view.view(p, chunk), recv.view, rank)
        _sync()
        flat = recv_h.reshape(-1)
        halves = [to_np(flat[0:4 * chunk]), to_np(flat[4 * chunk:6 * chunk]), to_np(flat[6 * chunk:7 * chunk])]
        want = oracle.halving_rs_local(to_np(msg_h), halves, rank)
        assert same_bits(to_np(msg.view).reshape(p, chunk), want), first_diff(to_np(msg.view), want)
        msg.check()
        recv.check()


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_accumulate_batched_matches_oracle(dtype):
    """Pairs of different sizes (empty, ragged, unaligned, several blocks) in one launch, each against
    the oracle's single step; two pairs may share a received buffer."""
    counts = [1000, 0, 7, 4096 * 5 + 3, 8, 1 << 18, 129]
    offs = [0, 0, 1, 0, 3, 0, 2]
    accs, recvs, hosts = [], [], []
    for k, (c, o) in enumerate(zip(counts, offs)):
        a = W.normal(c, 300 + k, 1.0, "cpu", dtype)
        r = W.normal(c, 400 + k, 1e-2, "cpu", dtype)
        accs.append(_guarded_copy(a, o))
        recvs.append(_guarded_copy(r, o))
        hosts.append((a, r))
    # an eighth pair that reads pair 0's received buffer again
    a = W.normal(counts[0], 500, 1.0, "cpu", dtype)
    accs.append(_guarded_copy(a))
    recvs.append(recvs[0])
    hosts.append((a, hosts[0][1]))
    table = pccl.AccumulateTable([(x.view, y.view) for x, y in zip(accs, recvs)])
    pccl.pccl_accumulate_batched(table)
    _sync()
    for k, (a, r) in enumerate(hosts):
        want = oracle.accumulate(to_np(a), to_np(r))
        assert same_bits(to_np(accs[k].view), want), (k, first_diff(to_np(accs[k].view), want))
        assert same_bits(to_np(recvs[k].view), to_np(r))
        accs[k].check()
        recvs[k].check()
    pccl.pccl_accumulate_batched(pccl.AccumulateTable([]))      # an empty batch launches nothing


def test_ring_and_halving_full_size_inter_node_phase():
    """The inter-node phase of the 256 MB workload (16 nodes, 2 MB bf16 chunks) in the paper's
    own step-wise algorithms: 15 ring steps of 2 MB, and halving steps of 16, 8, 4, 2 MB."""
    w = W.cfg3()
    p, chunk = w.nodes, w.chunk
    msg_h = W.draw(w, p * chunk, "cpu", seed_offset=5).view(p, chunk)
    recv_h = W.draw(w, (p - 1) * chunk, "cpu", seed_offset=6).view(p - 1, chunk)
    rank = 5
    msg = _guarded_copy(msg_h)
    recv = recv_h.to(DEV)
    pccl.pccl_ring_reduce_scatter_local(msg.view.view(p, chunk), recv, rank)
    _sync()
    want = oracle.ring_rs_local(to_np(msg_h), [to_np(recv_h[s]) for s in range(p - 1)], rank, nthreads=8)
    assert same_bits(to_np(msg.view).reshape(p, chunk), want)
    msg.check()
    msg = _guarded_copy(msg_h)
    pccl.pccl_halving_reduce_scatter_local(msg.view.view(p, chunk), recv.view(-1), rank)
    _sync()
    flat = recv_h.reshape(-1)
    halves = [to_np(flat[0:8 * chunk]), to_np(flat[8 * chunk:12 * chunk]), to_np(flat[12 * chunk:14 * chunk]),
              to_np(flat[14 * chunk:15 * chunk])]
    want = oracle.halving_rs_local(to_np(msg_h), halves, rank, nthreads=8)
    assert same_bits(to_np(msg.view).reshape(p, chunk), want)
    msg.check()


def test_accumulate_full_size_128mb():
    """First halving step of a 256 MB bf16 message: 128 MB += 128 MB, sampled against the oracle."""
    n = 64 * 1024 * 1024
    a = W.uniform_pm1(n, 51, DEV, BF16)
    r = W.uniform_pm1(n, 52, DEV, BF16)
    a0 = a.clone()
    pccl.pccl_accumulate(a, r)
    _sync()
    for lo in (0, 12345678, n - 4096):
        sl = slice(lo, lo + 4096)
        want = oracle.accumulate(to_np(a0[sl]), to_np(r[sl]))
        assert same_bits(to_np(a[sl]), want)
    # property that holds at any size: the result equals torch's own bf16 add everywhere
    assert torch.equal((a0 + r).view(torch.int16), a.view(torch.int16))
