"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same seeded
inputs.  Bars: permutations and gathers bit-exact; reductions bit-exact as well, because
the library uses exactly the oracle's summation order (that is stricter than the stated
tolerances: relative error <= 1e-6 for fp32 output, <= 1 bf16 ulp for bf16 output)."""
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
F32, BF16 = torch.float32, torch.bfloat16
ODT = {F32: oracle.F32, BF16: oracle.BF16}


def _sync():
    torch.cuda.synchronize()


def _draw(n, dtype, seed, kind="uniform"):
    if kind == "uniform":
        return W.uniform_pm1(n, seed, "cpu", dtype)
    if kind == "normal":
        return W.normal(n, seed, 1.0, "cpu", dtype)
    if kind == "int":
        return W.small_integers(n, seed, "cpu", dtype)
    raise ValueError(kind)


# ------------------------------------------------------------------------------- flat reduce
@pytest.mark.parametrize("in_dt,out_dt", [(F32, F32), (BF16, BF16), (BF16, F32), (F32, BF16)])
@pytest.mark.parametrize("nsrc", [1, 2, 3, 4, 5, 8, 13, 16, 17])
@pytest.mark.parametrize("count", [1, 7, 1000, 4096 * 3 + 5])
def test_local_reduce_matches_oracle(in_dt, out_dt, nsrc, count):
    print("case", in_dt, out_dt, nsrc, count, flush=True)
    pad = 24  # elements between sources: keeps rows 16-byte aligned for count % 8 == 0 only
    host = _draw(nsrc * (count + pad), in_dt, seed=nsrc * 100003 + count).view(nsrc, count + pad)
    src = host.to(DEV)[:, :count]
    dst = Guarded(count, out_dt)
    pccl.pccl_local_reduce(dst.view, src)
    _sync()
    want = oracle.flat_reduce([to_np(host[s, :count]) for s in range(nsrc)], ODT[out_dt])
    got = to_np(dst.view)
    assert same_bits(got, want), first_diff(got, want)
    dst.check()


@pytest.mark.parametrize("in_dt,out_dt", [(F32, F32), (BF16, BF16), (BF16, F32), (F32, BF16)])
@pytest.mark.parametrize("src_off,dst_off", [(1, 0), (0, 1), (1, 1), (3, 2)])
def test_local_reduce_unaligned_buffers(in_dt, out_dt, src_off, dst_off):
    nsrc, count = 8, 5000
    row = count + 40 + 1  # odd row stride in elements as well
    host = _draw(nsrc * row, in_dt, seed=77 + src_off).view(nsrc, row)
    src = host.to(DEV)[:, src_off:src_off + count]
    dst = Guarded(count, out_dt, offset_elems=dst_off)
    pccl.pccl_local_reduce(dst.view, src)
    _sync()
    want = oracle.flat_reduce([to_np(host[s, src_off:src_off + count]) for s in range(nsrc)], ODT[out_dt])
    assert same_bits(to_np(dst.view), want), first_diff(to_np(dst.view), want)
    dst.check()


def test_cfg1_flat_reduce_full_size():
    w = W.cfg1()
    host = W.draw(w, w.gpus * w.chunk).view(w.gpus, w.chunk)
    dst = Guarded(w.chunk, F32)
    pccl.pccl_local_reduce(dst.view, host.to(DEV))
    _sync()
    want = oracle.flat_reduce([to_np(host[s]) for s in range(w.gpus)])
    assert same_bits(to_np(dst.view), want), first_diff(to_np(dst.view), want)
    dst.check()


def _golden_lines(name):
    here = os.path.dirname(os.path.abspath(__file__))
    with open(os.path.join(here, "golden", name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line


def _pf(tok):
    return float.fromhex(tok) if "0x" in tok.lower() else float(tok)


def test_hand_worked_order_cases_on_gpu():
    """The IEEE order cases of tests/golden run through the library: flat ones through
    pccl_local_reduce, two-level ones through the pointer-array entry point (both kernels)."""
    for line in _golden_lines("fp32_order_cases.txt"):
        shape, terms, expected = [p.strip() for p in line.split("|")]
        nodes, gpus = map(int, shape.split())
        vals = torch.tensor([_pf(t) for t in terms.split()], dtype=F32)
        want = np.array([_pf(expected)], dtype=np.float32)
        # each term is a source of 9 equal elements (vector path + ragged tail)
        src = vals.view(-1, 1).repeat(1, 9).contiguous().to(DEV)
        if nodes == 1:
            dst = torch.empty(9, dtype=F32, device=DEV)
            pccl.pccl_local_reduce(dst, src)
            _sync()
            assert same_bits(to_np(dst), np.repeat(want, 9)), line
        ptrs = pccl.device_pointer_array([src[k] for k in range(nodes * gpus)])
        for force in ("stream", "lds"):
            os.environ["PCCL_FORCE_TWO_LEVEL_KERNEL"] = force
            pccl.diag_reload_env()
            try:
                dst = torch.empty(9, dtype=F32, device=DEV)
                pccl.pccl_local_reduce_ptrs_two_level(dst, ptrs, nodes, gpus, 9, F32)
                _sync()
            finally:
                del os.environ["PCCL_FORCE_TWO_LEVEL_KERNEL"]
                pccl.diag_reload_env()
            assert same_bits(to_np(dst), np.repeat(want, 9)), (line, force, to_np(dst))


def test_bf16_partial_rounding_cases_on_gpu():
    for line in _golden_lines("bf16_partial_rounding_cases.txt"):
        shape, terms, expected, _ = [p.strip() for p in line.split("|")]
        nodes, gpus = map(int, shape.split())
        vals = torch.tensor([_pf(t) for t in terms.split()], dtype=F32).to(BF16)
        src = vals.view(-1, 1).repeat(1, 19).contiguous().to(DEV)
        ptrs = pccl.device_pointer_array([src[k] for k in range(nodes * gpus)])
        for force in ("stream", "lds"):
            os.environ["PCCL_FORCE_TWO_LEVEL_KERNEL"] = force
            pccl.diag_reload_env()
            try:
                dst = torch.empty(19, dtype=BF16, device=DEV)
                pccl.pccl_local_reduce_ptrs_two_level(dst, ptrs, nodes, gpus, 19, BF16)
                _sync()
            finally:
                del os.environ["PCCL_FORCE_TWO_LEVEL_KERNEL"]
                pccl.diag_reload_env()
            assert bool((dst.float().cpu() == _pf(expected)).all()), (line, force)


def test_special_values_flow_through():
    """Subnormals are kept, -0 survives, inf propagates, NaN stays NaN."""
    rows = torch.tensor([[1e-45, -0.0, float("inf"), 1.0, 3e-39, float("nan"), -1e-40, 65504.0],
                         [1e-45, -0.0, 1.0, float("-inf"), 2e-39, 1.0, -1e-40, 1e38]], dtype=F32)
    dst = torch.empty(8, dtype=F32, device=DEV)
    pccl.pccl_local_reduce(dst, rows.to(DEV))
    _sync()
    want = oracle.flat_reduce([to_np(rows[0]), to_np(rows[1])])
    got = to_np(dst)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert same_bits(got[~nan], want[~nan]), first_diff(got[~nan], want[~nan])
    assert got[0] == np.float32(2.8e-45) and np.signbit(got[1])


def test_bf16_rounding_exhaustive_on_gpu():
    """Every binary32 pattern through the library's fp32 -> bf16 store (nsrc = 1 converting
    copy) against the oracle's round-to-nearest-even; NaNs compared by NaN-ness and sign."""
    step = 1 << 26
    base = torch.arange(step, dtype=torch.int64, device=DEV)
    dst = torch.empty(step, dtype=BF16, device=DEV)
    for start in range(0, 1 << 32, step):
        u = (base + start).to(torch.int32) if start < (1 << 31) else (base + (start - (1 << 32))).to(torch.int32)
        src = u.view(F32).view(1, step)
        pccl.pccl_local_reduce(dst, src)
        _sync()
        got = to_np(dst)
        bits = u.cpu().numpy().view(np.uint32)
        want = oracle.f32_to_bf16(bits.view(np.float32))
        if (start >> 23) & 0xFF != 0xFF:
            assert same_bits(got, want), (hex(start), first_diff(got, want))
            continue
        nan = (bits & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
        assert same_bits(got[~nan], want[~nan]), hex(start)
        assert np.all((got[nan] & 0x7FFF) > 0x7F80), "NaN must stay NaN"
        assert np.array_equal(got[nan] >> 15, (bits[nan] >> 31).astype(np.uint16)), "NaN keeps its sign"


# ------------------------------------------------------------------------------- pointer arrays
def _arena_sources(nsrc, count, dtype, seed, kind="normal", align_elems=8, shift=0):
    """nsrc chunks in one arena, placed in shuffled slots so the pointer array is not monotone."""
    slot = (count + align_elems - 1) // align_elems * align_elems + shift
    host = _draw(nsrc * slot + 8, dtype, seed, kind)
    arena = host.to(DEV)
    order = W.shuffled_slot_order(nsrc, seed)
    dev = [arena[order[s] * slot + shift: order[s] * slot + shift + count] for s in range(nsrc)]
    cpu = [to_np(host[order[s] * slot + shift: order[s] * slot + shift + count]) for s in range(nsrc)]
    return arena, dev, cpu


@pytest.mark.parametrize("in_dt,out_dt", [(F32, F32), (BF16, BF16), (BF16, F32)])
@pytest.mark.parametrize("nsrc,count", [(1, 100), (8, 4096), (16, 70000), (37, 1000), (300, 129), (2048, 64)])
def test_local_reduce_ptrs_matches_oracle(in_dt, out_dt, nsrc, count):
    print("case", in_dt, out_dt, nsrc, count, flush=True)
    arena, dev, cpu = _arena_sources(nsrc, count, in_dt, seed=nsrc + count)
    ptrs = pccl.device_pointer_array(dev)
    dst = Guarded(count, out_dt)
    pccl.pccl_local_reduce_ptrs(dst.view, ptrs, count, in_dt)
    _sync()
    want = oracle.flat_reduce(cpu, ODT[out_dt])
    assert same_bits(to_np(dst.view), want), first_diff(to_np(dst.view), want)
    dst.check()


@pytest.mark.parametrize("force", ["stream", "lds", None])
@pytest.mark.parametrize("in_dt,out_dt", [(F32, F32), (BF16, BF16), (BF16, F32), (F32, BF16)])
@pytest.mark.parametrize("nodes,gpus,count,shift", [
    (2, 2, 5, 0), (4, 8, 1000, 0), (16, 8, 4096, 0), (3, 5, 777, 1), (33, 8, 130, 0),
    (256, 8, 300, 0), (300, 2, 200, 1), (9, 1, 64, 0), (1, 8, 640, 0), (40, 4, 255, 3),
    (130, 8, 100, 0), (70, 16, 96, 0), (129, 1, 200, 1), (65, 4, 128, 0), (17, 3, 260, 1), (33, 11, 64, 0)])
def test_two_level_ptrs_matches_oracle(force, in_dt, out_dt, nodes, gpus, count, shift):
    print("case", force, in_dt, out_dt, nodes, gpus, count, shift, flush=True)
    nsrc = nodes * gpus
    arena, dev, cpu = _arena_sources(nsrc, count, in_dt, seed=nsrc * 7 + count, shift=shift)
    ptrs = pccl.device_pointer_array(dev)
    dst = Guarded(count, out_dt, offset_elems=shift)
    if force:
        os.environ["PCCL_FORCE_TWO_LEVEL_KERNEL"] = force
        pccl.diag_reload_env()
    try:
        pccl.pccl_local_reduce_ptrs_two_level(dst.view, ptrs, nodes, gpus, count, in_dt)
        _sync()
    finally:
        os.environ.pop("PCCL_FORCE_TWO_LEVEL_KERNEL", None)
        pccl.diag_reload_env()
    want = oracle.two_level_reduce(cpu, nodes, gpus, ODT[out_dt])
    assert same_bits(to_np(dst.view), want), first_diff(to_np(dst.view), want)
    dst.check()


def test_cfg4_allreduce_share_full_size():
    """2048 ranks x 64 KB fp32 through a shuffled pointer array, node-major two-level order,
    then the all-gather half: 2048 gathered shards back into rank order."""
    w = W.cfg4()
    nsrc = w.ranks
    arena, dev, cpu = _arena_sources(nsrc, w.chunk, F32, seed=w.seed, kind="normal")
    ptrs = pccl.device_pointer_array(dev)
    shard = Guarded(w.chunk, F32)
    pccl.pccl_local_reduce_ptrs_two_level(shard.view, ptrs, w.nodes, w.gpus, w.chunk, F32)
    _sync()
    want = oracle.two_level_reduce(cpu, w.nodes, w.gpus, nthreads=8)
    assert same_bits(to_np(shard.view), want), first_diff(to_np(shard.view), want)
    shard.check()
    # all-gather half: own shard sits in its hierarchical slot, the others are seeded data
    gathered = W.normal(nsrc * w.chunk, w.seed + 1, 1.0, DEV).view(nsrc, w.chunk)
    my_slot = 3 * w.nodes + 17  # this GPU is rank (n=17, g=3)
    gathered[my_slot].copy_(shard.view)
    out = Guarded(nsrc * w.chunk, F32)
    pccl.pccl_allgather_reassemble(out.view, src=gathered, nodes=w.nodes, gpus_per_node=w.gpus)
    _sync()
    want = oracle.hier_unpack(to_np(gathered), w.nodes, w.gpus)
    assert same_bits(to_np(out.view), want)
    out.check()
    assert same_bits(to_np(out.view).reshape(nsrc, w.chunk)[17 * w.gpus + 3], to_np(shard.view))
    # and through a pointer array of slots
    slots = pccl.device_pointer_array([gathered[k] for k in range(nsrc)])
    out2 = Guarded(nsrc * w.chunk, F32)
    pccl.pccl_allgather_reassemble(out2.view, d_slots=slots, nodes=w.nodes, gpus_per_node=w.gpus)
    _sync()
    assert same_bits(to_np(out2.view), want)
    out2.check()


# ------------------------------------------------------------------------------- permutations
@pytest.mark.parametrize("nodes,gpus,chunk_bytes", [
    (2, 3, 1), (4, 8, 2), (3, 2, 6), (4, 8, 16), (4, 8, 4096), (16, 8, 16384 + 48), (5, 3, 17),
    (7, 2, 16384 * 2 + 3), (256, 8, 260), (1, 8, 100), (8, 1, 100), (2, 2, 100000), (70000, 1, 4),
    (2, 66000, 2), (3, 3, 1024), (3, 3, 1040), (3, 3, 1023)])
@pytest.mark.parametrize("offset", [0, 1, 4])
def test_pack_unpack_match_oracle(nodes, gpus, chunk_bytes, offset):
    print("case", nodes, gpus, chunk_bytes, offset, flush=True)
    total = nodes * gpus * chunk_bytes
    g = torch.Generator().manual_seed(total + offset)
    host = torch.randint(0, 256, (total + 16,), generator=g, dtype=torch.uint8)
    src = host.to(DEV)[offset:offset + total]
    src_np = host[offset:offset + total].numpy()
    for fn, ofn in ((pccl.pccl_hier_unpack, oracle.hier_unpack), (pccl.pccl_hier_pack, oracle.hier_pack)):
        raw = torch.full((total + 64,), 0xA5, dtype=torch.uint8, device=DEV)
        dst = raw[16 + offset:16 + offset + total]
        fn(dst, src, nodes, gpus)
        _sync()
        want = ofn(src_np, nodes, gpus)
        assert same_bits(dst.cpu().numpy(), want), first_diff(dst.cpu().numpy(), want)
        r = raw.cpu()
        assert bool((r[:16 + offset] == 0xA5).all()) and bool((r[16 + offset + total:] == 0xA5).all())
    # round trip through the library alone
    a = torch.empty_like(src)
    b = torch.empty_like(src)
    pccl.pccl_hier_pack(a, src, nodes, gpus)
    pccl.pccl_hier_unpack(b, a, nodes, gpus)
    _sync()
    assert bool((b == src).all())


def test_cfg2_allgather_reassembly_full_size():
    w = W.cfg2()
    host = W.draw(w, w.ranks * w.chunk)  # [g][n][chunk] random 16-bit patterns
    src = host.to(DEV)
    dst = Guarded(w.ranks * w.chunk, BF16)
    pccl.pccl_hier_unpack(dst.view, src, w.nodes, w.gpus)
    _sync()
    want = oracle.hier_unpack(to_np(host), w.nodes, w.gpus)
    assert same_bits(to_np(dst.view), want)
    dst.check()
    back = torch.empty_like(src)
    pccl.pccl_hier_pack(back, dst.view, w.nodes, w.gpus)
    _sync()
    assert same_bits(to_np(back), to_np(host))
    # every rank's chunk lands exactly once: compare per-chunk fingerprints
    got = to_np(dst.view).reshape(w.ranks, w.chunk)
    src_np = to_np(host).reshape(w.gpus, w.nodes, w.chunk)
    for n in range(w.nodes):
        for g in range(w.gpus):
            assert same_bits(got[n * w.gpus + g][:64], src_np[g][n][:64])


@pytest.mark.parametrize("nodes,gpus,chunk_elems", [(2, 3, 5), (4, 8, 1000), (16, 4, 4096), (64, 8, 33)])
def test_reassemble_from_slot_pointers(nodes, gpus, chunk_elems):
    P = nodes * gpus
    arena, dev, cpu = _arena_sources(P, chunk_elems, F32, seed=P, kind="normal", shift=P % 2)
    slots = pccl.device_pointer_array(dev)
    dst = Guarded(P * chunk_elems, F32)
    pccl.pccl_allgather_reassemble(dst.view, d_slots=slots, nodes=nodes, gpus_per_node=gpus)
    _sync()
    want = oracle.allgather_reassemble(cpu, nodes, gpus)
    assert same_bits(to_np(dst.view), want)
    dst.check()


# ------------------------------------------------------------------------------- two-level reduce-scatter
@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("nodes,gpus,chunk", [(2, 2, 3), (4, 8, 1000), (16, 8, 2048 + 8), (3, 5, 333),
                                               (1, 8, 100), (8, 1, 100), (5, 16, 64), (2, 3, 20001)])
def test_reduce_scatter_local_matches_oracle(dtype, nodes, gpus, chunk):
    print("case", dtype, nodes, gpus, chunk, flush=True)
    host = _draw(gpus * nodes * chunk, dtype, seed=nodes * 31 + gpus * 7 + chunk).view(gpus, nodes, chunk)
    x = host.to(DEV)
    partial = Guarded(nodes * chunk, dtype)
    shard = Guarded(chunk, dtype)
    pccl.pccl_reduce_scatter_local(shard.view, partial.view, x)
    _sync()
    want_shard, want_partial = oracle.reduce_scatter_local(to_np(host))
    assert same_bits(to_np(partial.view), want_partial), first_diff(to_np(partial.view), want_partial)
    assert same_bits(to_np(shard.view), want_shard), first_diff(to_np(shard.view), want_shard)
    partial.check()
    shard.check()


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_reduce_scatter_local_with_received_inter_chunks(dtype):
    nodes, gpus, chunk, my = 6, 4, 1500, 2
    host = _draw(gpus * nodes * chunk, dtype, seed=5).view(gpus, nodes, chunk)
    arena, dev, cpu = _arena_sources(nodes, chunk, dtype, seed=6, kind="uniform")
    d_inter = pccl.device_pointer_array(dev)
    partial = Guarded(nodes * chunk, dtype)
    shard = Guarded(chunk, dtype)
    pccl.pccl_reduce_scatter_local(shard.view, partial.view, host.to(DEV), d_inter=d_inter, my_node=my)
    _sync()
    want_shard, want_partial = oracle.reduce_scatter_local(to_np(host), my_node=my, inter=cpu)
    assert same_bits(to_np(partial.view), want_partial)
    assert same_bits(to_np(shard.view), want_shard), first_diff(to_np(shard.view), want_shard)
    shard.check()


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("nodes,gpus,chunk", [(64, 2, 1000), (256, 8, 96), (300, 1, 515), (40, 32, 64)])
def test_reduce_scatter_local_many_sources_short_chunks(dtype, nodes, gpus, chunk):
    """Shapes whose phase 2 (and, with 32 GPUs per node, phase 1) is a long chain over short
    buffers: the flat sums go through the LDS-staged kernel."""
    x_h = _draw(gpus * nodes * chunk, dtype, 4242 + nodes).view(gpus, nodes, chunk)
    inter_h = _draw(nodes * chunk, dtype, 4243 + nodes).view(nodes, chunk)
    x, inter = x_h.to(DEV), inter_h.to(DEV)
    my_node = nodes // 3
    for d_inter in (None, pccl.device_pointer_array([inter[n] for n in range(nodes)])):
        partial = Guarded(nodes * chunk, dtype)
        shard = Guarded(chunk, dtype)
        pccl.pccl_reduce_scatter_local(shard.view, partial.view, x, d_inter=d_inter, my_node=my_node)
        _sync()
        want_shard, want_partial = oracle.reduce_scatter_local(
            to_np(x_h), my_node=my_node, inter=None if d_inter is None else [to_np(inter_h[n]) for n in range(nodes)])
        assert same_bits(to_np(partial.view), want_partial.reshape(-1)), first_diff(to_np(partial.view), want_partial)
        assert same_bits(to_np(shard.view), want_shard), first_diff(to_np(shard.view), want_shard)
        partial.check()
        shard.check()
    # the strided flat entry with many short sources
    src_h = _draw(200 * 333, dtype, 99).view(200, 333)
    dst = Guarded(333, dtype)
    pccl.pccl_local_reduce(dst.view, src_h.to(DEV))
    _sync()
    assert same_bits(to_np(dst.view), oracle.flat_reduce([to_np(src_h[k]) for k in range(200)]))
    dst.check()


def test_reduce_scatter_local_strided_pieces():
    """Pieces that do not touch each other in memory (row stride larger than a piece)."""
    nodes, gpus, chunk = 4, 8, 512
    host = _draw(gpus * (nodes * chunk + 64), BF16, seed=9).view(gpus, nodes * chunk + 64)
    x = host.to(DEV)[:, :nodes * chunk].unflatten(1, (nodes, chunk))
    partial = torch.empty(nodes * chunk, dtype=BF16, device=DEV)
    shard = torch.empty(chunk, dtype=BF16, device=DEV)
    pccl.pccl_reduce_scatter_local(shard, partial, x)
    _sync()
    want_shard, want_partial = oracle.reduce_scatter_local(
        to_np(host[:, :nodes * chunk]).reshape(gpus, nodes, chunk))
    assert same_bits(to_np(partial), want_partial) and same_bits(to_np(shard), want_shard)


def test_cfg3_two_level_reduce_scatter_full_size():
    """16 x 8 ranks, 256 MB bf16 message: phase 1 sums 8 x 32 MB, phase 2 sums 16 x 2 MB."""
    w = W.cfg3()
    x = W.two_level_input(w, DEV)
    partial = Guarded(w.nodes * w.chunk, BF16)
    shard = Guarded(w.chunk, BF16)
    pccl.pccl_reduce_scatter_local(shard.view, partial.view, x)
    _sync()
    want_shard, want_partial = oracle.reduce_scatter_local(to_np(x), nthreads=16)
    assert same_bits(to_np(partial.view), want_partial), first_diff(to_np(partial.view), want_partial)
    assert same_bits(to_np(shard.view), want_shard), first_diff(to_np(shard.view), want_shard)
    partial.check()
    shard.check()
    # the reduce-scatter pre-shuffle at the same size: a 256 MB rank-order message
    msg = x.view(-1)  # reuse the bytes as [node=16][gpu=8][chunk]
    packed = Guarded(msg.numel(), BF16)
    pccl.pccl_hier_pack(packed.view, msg, w.nodes, w.gpus)
    _sync()
    assert same_bits(to_np(packed.view), oracle.hier_pack(to_np(msg), w.nodes, w.gpus))
    packed.check()


def test_cfg3_in_the_benchmarked_launch_configuration():
    """The call sequence bench.py times, at full size: pack, reduce-scatter share with the 15
    foreign chunks behind a device pointer array, reassemble."""
    w = W.cfg3()
    n = w.ranks * w.chunk
    my = 5
    msg = W.draw(w, n, DEV, seed_offset=1)
    x = W.two_level_input(w, DEV, seed_offset=2)
    inter = W.draw(w, w.nodes * w.chunk, DEV, seed_offset=3).view(w.nodes, w.chunk)
    d_inter = pccl.device_pointer_array([inter[j] for j in range(w.nodes)])
    gathered = W.draw(w, n, DEV, seed_offset=4)
    packed, out = Guarded(n, BF16), Guarded(n, BF16)
    partial, shard = Guarded(w.nodes * w.chunk, BF16), Guarded(w.chunk, BF16)
    pccl.pccl_hier_pack(packed.view, msg, w.nodes, w.gpus)
    pccl.pccl_reduce_scatter_local(shard.view, partial.view, x, d_inter=d_inter, my_node=my)
    pccl.pccl_allgather_reassemble(out.view, src=gathered, nodes=w.nodes, gpus_per_node=w.gpus)
    _sync()
    assert same_bits(to_np(packed.view), oracle.hier_pack(to_np(msg), w.nodes, w.gpus))
    want_shard, want_partial = oracle.reduce_scatter_local(
        to_np(x), my_node=my, inter=[to_np(inter[j]) for j in range(w.nodes)], nthreads=16)
    assert same_bits(to_np(partial.view), want_partial)
    assert same_bits(to_np(shard.view), want_shard), first_diff(to_np(shard.view), want_shard)
    assert same_bits(to_np(out.view), oracle.hier_unpack(to_np(gathered), w.nodes, w.gpus))
    for gbuf in (packed, out, partial, shard):
        gbuf.check()


# ------------------------------------------------------------------------------- batched buckets
def _make_buckets(w, sizes_bytes, device):
    buckets, hosts = [], []
    for k, nbytes in enumerate(sizes_bytes):
        chunk = nbytes // (w.ranks * w.esize)
        x = W.two_level_input(w, device, seed_offset=k + 1, chunk=chunk)
        partial = torch.empty(w.nodes * chunk, dtype=w.dtype, device=device)
        shard = torch.empty(chunk, dtype=w.dtype, device=device)
        buckets.append((shard, partial, x))
    return buckets


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("use_ptrs", [False, True])
@pytest.mark.parametrize("nodes,gpus,chunk,my_n,my_g", [(2, 2, 3, 0, 1), (4, 8, 1000, 3, 7), (16, 8, 2048 + 8, 5, 0),
                                                         (3, 5, 333, 2, 4), (1, 4, 100, 0, 2), (5, 1, 64, 4, 0)])
def test_unpacked_reduce_scatter_matches_oracle(dtype, use_ptrs, nodes, gpus, chunk, my_n, my_g):
    print("case", dtype, use_ptrs, nodes, gpus, chunk, my_n, my_g, flush=True)
    P = nodes * gpus
    msgs_h = _draw(gpus * P * chunk, dtype, 900 + P + chunk).view(gpus, P * chunk)
    inter_h = _draw(nodes * chunk, dtype, 901 + P + chunk).view(nodes, chunk)
    msgs = msgs_h.to(DEV)
    inter = inter_h.to(DEV)
    d_inter = pccl.device_pointer_array([inter[n] for n in range(nodes)])
    partial = Guarded(nodes * chunk, dtype)
    shard = Guarded(chunk, dtype)
    if use_ptrs:
        separate = [msgs[g].clone() for g in reversed(range(gpus))][::-1]   # own allocations, not monotone
        pccl.pccl_reduce_scatter_local_unpacked(shard.view, partial.view, d_msgs=pccl.device_pointer_array(separate),
                                                d_inter=d_inter, nodes=nodes, gpus_per_node=gpus, my_node=my_n,
                                                my_gpu=my_g)
    else:
        pccl.pccl_reduce_scatter_local_unpacked(shard.view, partial.view, msgs=msgs, d_inter=d_inter, nodes=nodes,
                                                gpus_per_node=gpus, my_node=my_n, my_gpu=my_g)
    _sync()
    want_shard, want_partial = oracle.reduce_scatter_local_unpacked(
        [to_np(msgs_h[g]) for g in range(gpus)], nodes, gpus, my_g, my_node=my_n,
        inter=[to_np(inter_h[n]) for n in range(nodes)])
    assert same_bits(to_np(partial.view), want_partial.reshape(-1)), first_diff(to_np(partial.view), want_partial)
    assert same_bits(to_np(shard.view), want_shard), first_diff(to_np(shard.view), want_shard)
    partial.check()
    shard.check()
    # and it is the packed path bit for bit
    packed = torch.empty_like(msgs)
    for g in range(gpus):
        pccl.pccl_hier_pack(packed[g], msgs[g], nodes, gpus)
    x = packed.view(gpus, gpus, nodes, chunk)[:, my_g]          # piece my_g of every message (strided rows)
    p2 = torch.empty(nodes * chunk, dtype=dtype, device=DEV)
    s2 = torch.empty(chunk, dtype=dtype, device=DEV)
    pccl.pccl_reduce_scatter_local(s2, p2, x, d_inter=d_inter, my_node=my_n)
    _sync()
    assert same_bits(to_np(p2), to_np(partial.view)) and same_bits(to_np(s2), to_np(shard.view))


def test_unpacked_reduce_scatter_unaligned_and_self_simulated():
    nodes, gpus, chunk, my_g = 3, 4, 1001, 2
    P = nodes * gpus
    raw = _draw(gpus * (P * chunk + 8) + 3, BF16, 77).to(DEV)
    msgs = torch.as_strided(raw, (gpus, P * chunk), (P * chunk + 8, 1), 3)   # odd element offset, padded rows
    partial = Guarded(nodes * chunk, BF16, offset_elems=1)
    shard = Guarded(chunk, BF16, offset_elems=1)
    pccl.pccl_reduce_scatter_local_unpacked(shard.view, partial.view, msgs=msgs, nodes=nodes, gpus_per_node=gpus,
                                            my_gpu=my_g)
    _sync()
    want_shard, want_partial = oracle.reduce_scatter_local_unpacked(
        [to_np(msgs[g]) for g in range(gpus)], nodes, gpus, my_g)
    assert same_bits(to_np(partial.view), want_partial.reshape(-1))
    assert same_bits(to_np(shard.view), want_shard)
    partial.check()
    shard.check()


@pytest.mark.parametrize("dtype", [BF16, F32])
def test_batched_small_buckets_match_unbatched_oracle(dtype):
    w = W.cfg5()
    w.dtype = dtype
    sizes = [1024, 3 * 1024, 64 * 1024, 1024, 0, 129 * 1024, 7 * 1024]
    buckets = _make_buckets(w, sizes, DEV)
    table = pccl.BucketTable(buckets)
    pccl.pccl_reduce_scatter_local_batched(table)
    _sync()
    for k, (shard, partial, x) in enumerate(buckets):
        if x.numel() == 0:
            continue
        want_shard, want_partial = oracle.reduce_scatter_local(to_np(x))
        assert same_bits(to_np(partial), want_partial), (k, first_diff(to_np(partial), want_partial))
        assert same_bits(to_np(shard), want_shard), (k, first_diff(to_np(shard), want_shard))


def test_batched_ragged_chunks_and_other_shapes():
    w = W.cfg5()
    w.nodes, w.gpus = 3, 5
    buckets = []
    for k, chunk in enumerate([1, 9, 1001, 4099]):
        x = W.two_level_input(w, DEV, seed_offset=k + 50, chunk=chunk)
        buckets.append((torch.empty(chunk, dtype=BF16, device=DEV),
                        torch.empty(w.nodes * chunk, dtype=BF16, device=DEV), x))
    table = pccl.BucketTable(buckets)
    pccl.pccl_reduce_scatter_local_batched(table)
    _sync()
    for k, (shard, partial, x) in enumerate(buckets):
        want_shard, want_partial = oracle.reduce_scatter_local(to_np(x))
        assert same_bits(to_np(partial), want_partial), k
        assert same_bits(to_np(shard), want_shard), k


def test_cfg5_zero3_buckets_full_size():
    """40 buckets of 16 - 512 MB in one batched call; three whole buckets (smallest, median,
    largest) and the head and tail of every shard are checked against the oracle, and every
    element of every partial and shard against the same sums written with torch on the GPU."""
    w = W.cfg5()
    sizes = w.extra["bucket_bytes"]
    buckets = _make_buckets(w, sizes, DEV)
    table = pccl.BucketTable(buckets)
    pccl.pccl_reduce_scatter_local_batched(table)
    _sync()
    order = sorted(range(len(sizes)), key=lambda k: sizes[k])
    for k in (order[0], order[len(order) // 2], order[-1]):
        shard, partial, x = buckets[k]
        want_shard, want_partial = oracle.reduce_scatter_local(to_np(x), nthreads=16)
        assert same_bits(to_np(partial), want_partial), k
        assert same_bits(to_np(shard), want_shard), k
    for k, (shard, partial, x) in enumerate(buckets):
        head = min(4096, x.shape[2])
        tail = x.shape[2] - head
        for sl in (slice(0, head), slice(tail, tail + head)):
            want_shard, _ = oracle.reduce_scatter_local(to_np(x[:, :, sl]))
            assert same_bits(to_np(shard[sl]), want_shard), k
    # EVERY element of every bucket's partial and shard, on the GPU, against the same order written with
    # torch: binary32 adds one source after the other, torch's bf16 cast (round to nearest even; the
    # oracle's rounding is pinned against that cast over all 2^32 patterns) between and after the phases
    for k, (shard, partial, x) in enumerate(buckets):
        t = x[0].float()
        for g in range(1, x.shape[0]):
            t = t + x[g].float()
        ref_partial = t.to(BF16)                                   # [nodes][chunk]
        assert torch.equal(partial.view(torch.int16), ref_partial.view(torch.int16).reshape(-1)), ("partial", k)
        a = ref_partial[0].float()
        for n in range(1, x.shape[1]):
            a = a + ref_partial[n].float()
        assert torch.equal(shard.view(torch.int16), a.to(BF16).view(torch.int16)), ("shard", k)
        del t, a, ref_partial


# ------------------------------------------------------------------------------- empty inputs
def test_empty_inputs_launch_nothing_and_touch_nothing():
    """count == 0 / chunk == 0 succeed without a launch: poisoned outputs stay as they are."""
    for dtype in (F32, BF16):
        out = Guarded(16, dtype)
        before = to_np(out.raw).copy()
        empty_src = torch.empty(4, 0, dtype=dtype, device=DEV)
        L = pccl.lib()
        st = torch.cuda.current_stream().cuda_stream
        dt = pccl.binding.dtype_code(dtype)
        p = out.view.data_ptr()
        q = torch.empty(64, dtype=dtype, device=DEV).data_ptr()
        assert L.pccl_local_reduce(p, q, 0, 4, 0, dt, dt, 0, st) == pccl.PCCL_OK
        assert L.pccl_local_reduce_ptrs(p, q, 4, 0, dt, dt, 0, st) == pccl.PCCL_OK
        assert L.pccl_local_reduce_ptrs_two_level(p, q, 2, 2, 0, dt, dt, 0, st) == pccl.PCCL_OK
        assert L.pccl_hier_pack(p, q, 2, 2, 0, st) == pccl.PCCL_OK
        assert L.pccl_hier_unpack(p, q, 2, 2, 0, st) == pccl.PCCL_OK
        assert L.pccl_allgather_reassemble(p, q, None, 2, 2, 0, st) == pccl.PCCL_OK
        assert L.pccl_reduce_scatter_local(p, p + 1024, q, 0, None, 2, 2, 0, 0, dt, 0, st) == pccl.PCCL_OK
        assert L.pccl_reduce_scatter_local_unpacked(p, p + 1024, q, 0, None, None, 2, 2, 0, 1, 0, dt, 0, st) == pccl.PCCL_OK
        assert L.pccl_reduce_scatter_local_batched(None, None, 0, 2, 2, dt, 0, st) == pccl.PCCL_OK
        assert L.pccl_accumulate(p, q, 0, dt, 0, st) == pccl.PCCL_OK
        assert L.pccl_ring_reduce_scatter_local(p, q, 0, 4, 1, 0, dt, 0, st) == pccl.PCCL_OK
        assert L.pccl_halving_reduce_scatter_local(p, q, 4, 1, 0, dt, 0, st) == pccl.PCCL_OK
        _sync()
        assert same_bits(to_np(out.raw), before)
        del empty_src


def test_binding_refuses_host_tensors_and_mismatched_shapes():
    host = torch.zeros(4, 8)
    dev = torch.zeros(4, 8, device=DEV)
    with pytest.raises(ValueError):
        pccl.pccl_local_reduce(torch.zeros(8, device=DEV), host)
    with pytest.raises(ValueError):
        pccl.pccl_local_reduce(torch.zeros(7, device=DEV), dev)
    with pytest.raises(ValueError):
        pccl.pccl_hier_pack(torch.zeros(30, device=DEV), torch.zeros(32, device=DEV), 2, 4)
    with pytest.raises(TypeError):
        pccl.pccl_local_reduce(torch.zeros(8, device=DEV, dtype=torch.float64), dev.double())
    with pytest.raises(pccl.PcclError) as e:                       # in-place is refused by the library itself
        pccl.pccl_local_reduce(dev[0], dev)
    assert e.value.status == pccl.PCCL_ERR_OVERLAP
    with pytest.raises(pccl.PcclError) as e:                       # bf16 in, fp16 out: no such pair
        pccl.pccl_local_reduce(torch.zeros(8, device=DEV, dtype=torch.float16), dev.to(torch.bfloat16))
    assert e.value.status == pccl.PCCL_ERR_UNSUPPORTED


# ------------------------------------------------------------------------------- batched shuffles
@pytest.mark.parametrize("nodes,gpus", [(4, 8), (3, 5), (1, 7), (16, 2)])
def test_batched_shuffles_match_the_oracle_bucket_by_bucket(nodes, gpus):
    P = nodes * gpus
    chunk_bytes = [1024, 6, 0, 4096 + 48, 1, 100000, 16, 2050, 640 * 1024 + 48]   # ragged, tiny, empty, several tiles, rotated tiles
    for offset in (0, 1):                                              # 16-byte aligned and not
        srcs_h = [W.random_bits16((P * cb + 1) // 2 + 8, 50 + k).view(torch.uint8)[offset:offset + P * cb]
                  for k, cb in enumerate(chunk_bytes)]
        srcs = [s.to(DEV) for s in srcs_h]
        for name, fn, ref in (("unpack", pccl.pccl_allgather_reassemble_batched, oracle.hier_unpack),
                              ("pack", pccl.pccl_hier_pack_batched, oracle.hier_pack)):
            outs = [Guarded((P * cb + 3) // 4 + 2, F32) for cb in chunk_bytes]
            dsts = [o.view.view(torch.uint8)[offset:offset + P * cb] for o, cb in zip(outs, chunk_bytes)]
            table = pccl.PermuteTable(list(zip(dsts, srcs)), nodes, gpus)
            fn(table)
            _sync()
            for k, cb in enumerate(chunk_bytes):
                if cb:
                    want = ref(srcs_h[k].numpy(), nodes, gpus)
                    assert same_bits(to_np(dsts[k]), want), (name, k, cb, first_diff(to_np(dsts[k]), want))
                outs[k].check()


def test_batched_reassembly_of_the_zero3_bucket_list_full_size():
    """The 40 ZeRO-3-shaped buckets (16-512 MB, 8 x 8 ranks) through one batched all-gather shuffle:
    chunk by chunk equal to the definition on the GPU, three buckets and the head and tail of every
    bucket against the oracle."""
    w = W.cfg5()
    sizes = w.extra["bucket_bytes"]
    pairs = []
    for k, b in enumerate(sizes):
        src = W.random_bits16(b // 2, 700 + k, DEV)
        pairs.append((torch.empty_like(src), src))
    table = pccl.PermuteTable(pairs, w.nodes, w.gpus)
    pccl.pccl_allgather_reassemble_batched(table)
    _sync()
    for k, (dst, src) in enumerate(pairs):
        cb2 = src.numel() // w.ranks
        assert torch.equal(dst.view(torch.int16).view(w.nodes, w.gpus, cb2),
                           src.view(torch.int16).view(w.gpus, w.nodes, cb2).transpose(0, 1)), k
    for k in sorted(range(len(sizes)), key=lambda j: sizes[j])[:3]:
        dst, src = pairs[k]
        assert same_bits(to_np(dst), oracle.hier_unpack(to_np(src), w.nodes, w.gpus)), k


@pytest.mark.parametrize("dst_off", [0, 16, 48, 112, 512, 1008, 1023, 1024 + 16, 7])
@pytest.mark.parametrize("src_off", [0, 16, 100])
def test_shuffle_tiles_cut_at_destination_boundaries(dst_off, src_off):
    """Tiles are cut at 1 KB boundaries of the destination address: every combination of
    destination misalignment, source misalignment and chunk size around the tile size must
    still move every byte exactly once (single, pointer-array and batched forms)."""
    nodes, gpus = 2, 3
    P = nodes * gpus
    sizes = [1, 16, 1000, 1024, 1040, 2048, 3000, 5000, 1024 - 16]
    pairs, wants, outs = [], [], []
    for k, cb in enumerate(sizes):
        src_h = W.random_bits16((P * cb + 1) // 2 + 64, 900 + k).view(torch.uint8)[src_off:src_off + P * cb]
        src = src_h.to(DEV)                       # a fresh allocation: shift it to the wanted misalignment
        raw = torch.empty(P * cb + 256, dtype=torch.uint8, device=DEV)
        src = raw[src_off:src_off + P * cb].copy_(src)
        out = Guarded((P * cb + dst_off) // 4 + 8, F32)
        dst = out.view.view(torch.uint8)[dst_off:dst_off + P * cb]
        want = oracle.hier_unpack(src_h.numpy(), nodes, gpus)
        pccl.pccl_hier_unpack(dst, src, nodes, gpus)
        _sync()
        assert same_bits(to_np(dst), want), (cb, first_diff(to_np(dst), want))
        out.check()
        dst.zero_()
        slots = pccl.device_pointer_array([src[j * cb:(j + 1) * cb] for j in range(P)])
        pccl.pccl_allgather_reassemble(dst, d_slots=slots, nodes=nodes, gpus_per_node=gpus)
        _sync()
        assert same_bits(to_np(dst), want), ("slots", cb)
        out.check()
        dst.zero_()
        pairs.append((dst, src)); wants.append(want); outs.append(out)
    pccl.pccl_allgather_reassemble_batched(pccl.PermuteTable(pairs, nodes, gpus))
    _sync()
    for (dst, _), want, out, cb in zip(pairs, wants, outs, sizes):
        assert same_bits(to_np(dst), want), ("batched", cb)
        out.check()


# ------------------------------------------------------------------------------- batched share from messages
@pytest.mark.parametrize("dtype", [BF16, F32])
@pytest.mark.parametrize("nodes,gpus,my_gpu", [(4, 8, 3), (5, 3, 0), (1, 4, 3), (40, 2, 1), (3, 1, 0)])
def test_batched_share_from_rank_order_messages(dtype, nodes, gpus, my_gpu):
    """Buckets of different sizes (one empty, ragged and misaligned ones) through
    pccl_reduce_scatter_local_unpacked_batched: equal to the unbatched oracle bucket by bucket."""
    P = nodes * gpus
    chunks = [1000, 0, 7, 4096 + 3, 129, 20000]
    for average in (False, True):
        buckets, wants, guards = [], [], []
        for k, c in enumerate(chunks):
            msgs_h = W.normal(gpus * P * c + gpus, 80 + k, 1.0, "cpu", dtype)[: gpus * P * c].view(gpus, P * c)
            shard, partial = Guarded(c, dtype), Guarded(nodes * c, dtype, offset_elems=k % 2)
            buckets.append((shard.view, partial.view, msgs_h.to(DEV)))
            guards += [shard, partial]
            wants.append(oracle.reduce_scatter_local_unpacked([to_np(msgs_h[g]) for g in range(gpus)], nodes, gpus, my_gpu,
                                                              average=average) if c else None)
        table = pccl.BucketTable(buckets, nodes=nodes)
        pccl.pccl_reduce_scatter_local_unpacked_batched(table, my_gpu, average=average)
        _sync()
        for k, c in enumerate(chunks):
            if c:
                ws, wp = wants[k]
                assert same_bits(to_np(buckets[k][0]), ws), (k, c, average, first_diff(to_np(buckets[k][0]), ws))
                assert same_bits(to_np(buckets[k][1]), wp.reshape(-1)), (k, c, average)
        for g in guards:
            g.check()


def test_batched_share_from_messages_equals_pack_then_batched_share_at_size():
    """Ten ZeRO-3-shaped buckets (8 x 8 ranks, sizes of the 40-bucket list scaled by 1/4): the share
    straight from the messages equals pre-shuffling every message and taking the packed share,
    bit for bit on the GPU; the smallest bucket is also checked against the oracle."""
    w = W.cfg5(scale=0.25, nbuckets=10)
    sizes = w.extra["bucket_bytes"]
    nodes, gpus, my_gpu = w.nodes, w.gpus, 5
    P = nodes * gpus
    direct, packed, keep = [], [], []
    for k, b in enumerate(sizes):
        c = b // 2 // P
        msgs = W.normal(gpus * P * c, 90 + k, 1e-3, DEV, BF16).view(gpus, P * c)
        pieces = torch.empty(gpus, nodes * c, dtype=BF16, device=DEV)
        for g in range(gpus):                                   # piece g of the pre-shuffled message g2 = [my_gpu]
            tmp = torch.empty(P * c, dtype=BF16, device=DEV)
            pccl.pccl_hier_pack(tmp, msgs[g], nodes, gpus)
            pieces[g].copy_(tmp.view(gpus, nodes * c)[my_gpu])
        direct.append((torch.empty(c, dtype=BF16, device=DEV), torch.empty(nodes * c, dtype=BF16, device=DEV), msgs))
        packed.append((torch.empty(c, dtype=BF16, device=DEV), torch.empty(nodes * c, dtype=BF16, device=DEV),
                       pieces.view(gpus, nodes, c)))
    pccl.pccl_reduce_scatter_local_unpacked_batched(pccl.BucketTable(direct, nodes=nodes), my_gpu)
    pccl.pccl_reduce_scatter_local_batched(pccl.BucketTable(packed))
    _sync()
    for k in range(len(sizes)):
        assert torch.equal(direct[k][0].view(torch.int16), packed[k][0].view(torch.int16)), k
        assert torch.equal(direct[k][1].view(torch.int16), packed[k][1].view(torch.int16)), k
    k = min(range(len(sizes)), key=lambda j: sizes[j])
    ws, wp = oracle.reduce_scatter_local_unpacked([to_np(direct[k][2][g]) for g in range(gpus)], nodes, gpus, my_gpu)
    assert same_bits(to_np(direct[k][0]), ws) and same_bits(to_np(direct[k][1]), wp.reshape(-1))


def test_share_at_128_nodes_in_the_benchmarked_launch_configuration():
    """The 128 x 8 rank, 256 MB bf16 all-reduce share that bench.py times, at full size: the
    pre-shuffle of 256 KB chunks, phase 1 from pre-shuffled pieces and straight from the eight
    rank-order messages (128 rows), phase 2 over 128 received chunks, the reassembly."""
    nodes, gpus, my_node, my_gpu = 128, 8, 77, 3
    P = nodes * gpus
    c = (256 << 20) // P // 2
    msgs = W.uniform_pm1(gpus * P * c, 700, DEV, BF16).view(gpus, P * c)
    inter = W.uniform_pm1(nodes * c, 710, DEV, BF16).view(nodes, c)
    d_inter = pccl.device_pointer_array([inter[j] for j in range(nodes)])
    want_inter = [to_np(inter[j]) for j in range(nodes)]
    packed, out = Guarded(P * c, BF16), Guarded(P * c, BF16)
    pccl.pccl_hier_pack(packed.view, msgs[0], nodes, gpus)
    pccl.pccl_allgather_reassemble(out.view, src=msgs[1], nodes=nodes, gpus_per_node=gpus)
    _sync()
    assert same_bits(to_np(packed.view), oracle.hier_pack(to_np(msgs[0]), nodes, gpus))
    assert same_bits(to_np(out.view), oracle.hier_unpack(to_np(msgs[1]), nodes, gpus))
    packed.check()
    out.check()
    # from pre-shuffled pieces: the first message's bytes stand for [gpu][node][chunk]
    x = msgs[0].view(gpus, nodes, c)
    partial, shard = Guarded(nodes * c, BF16), Guarded(c, BF16)
    pccl.pccl_reduce_scatter_local(shard.view, partial.view, x, d_inter=d_inter, my_node=my_node)
    _sync()
    ws, wp = oracle.reduce_scatter_local(to_np(x), my_node=my_node, inter=want_inter, nthreads=16)
    assert same_bits(to_np(partial.view), wp.reshape(-1)) and same_bits(to_np(shard.view), ws)
    partial.check()
    shard.check()
    # straight from the messages
    partial2, shard2 = Guarded(nodes * c, BF16), Guarded(c, BF16)
    pccl.pccl_reduce_scatter_local_unpacked(shard2.view, partial2.view, msgs=msgs, d_inter=d_inter, nodes=nodes,
                                            gpus_per_node=gpus, my_node=my_node, my_gpu=my_gpu)
    _sync()
    ws, wp = oracle.reduce_scatter_local_unpacked([to_np(msgs[g]) for g in range(gpus)], nodes, gpus, my_gpu,
                                                  my_node=my_node, inter=want_inter, nthreads=16)
    assert same_bits(to_np(partial2.view), wp.reshape(-1)), first_diff(to_np(partial2.view), wp.reshape(-1))
    assert same_bits(to_np(shard2.view), ws)
    partial2.check()
    shard2.check()
