"""CPU oracle for the local kernels of PCCL's hierarchical collectives.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product path (the HIP library and its
Python binding) never imports this package, and this package never imports
the product.

All arithmetic lives in pccl_oracle.c; this module only marshals numpy arrays.
bf16 data is carried as numpy uint16 bit patterns, fp32 data as numpy float32, fp16 data as
numpy float16.
"""
import ctypes
import os

import numpy as np

from . import build as _build

F32 = 0
BF16 = 1
F16 = 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_build.build())
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.pccl_oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.pccl_oracle_f32_to_bf16.argtypes = [ctypes.c_uint32]
        L.pccl_oracle_f32_to_bf16_array.restype = None
        L.pccl_oracle_f32_to_bf16_array.argtypes = [vp, vp, sz]
        L.pccl_oracle_f32_to_f16.restype = ctypes.c_uint16
        L.pccl_oracle_f32_to_f16.argtypes = [ctypes.c_uint32]
        L.pccl_oracle_f32_to_f16_array.restype = None
        L.pccl_oracle_f32_to_f16_array.argtypes = [vp, vp, sz]
        L.pccl_oracle_f16_to_f32_array.restype = None
        L.pccl_oracle_f16_to_f32_array.argtypes = [vp, vp, sz]
        L.pccl_oracle_flat_reduce.argtypes = [vp, vp, i, sz, i, i, i, i]
        L.pccl_oracle_two_level_reduce.argtypes = [vp, vp, vp, i, i, sz, i, i, i, i]
        L.pccl_oracle_rs_phase1.argtypes = [vp, vp, i, i, sz, i, i]
        L.pccl_oracle_rs_phase2.argtypes = [vp, vp, i, sz, i, i, i, i]
        L.pccl_oracle_accumulate.argtypes = [vp, vp, sz, i, i]
        L.pccl_oracle_hier_pack.argtypes = [vp, vp, i, i, sz]
        L.pccl_oracle_hier_unpack.argtypes = [vp, vp, i, i, sz]
        L.pccl_oracle_allgather_reassemble.argtypes = [vp, vp, i, i, sz]
        _lib = L
    return _lib


def _dt(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float16:
        return F16
    raise TypeError("oracle takes float32 (fp32), uint16 (bf16 bits) or float16 arrays, got %s" % a.dtype)


def _np_dtype(code):
    return {F32: np.float32, BF16: np.uint16, F16: np.float16}[code]


def _flat(a):
    a = np.ascontiguousarray(a)
    return a.reshape(-1)


def _ptr_array(arrs):
    arr = (ctypes.c_void_p * len(arrs))()
    for k, a in enumerate(arrs):
        arr[k] = a.ctypes.data
    return arr


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s: bad argument (rc=%d)" % (what, rc))


def f32_to_bf16(x):
    """Round float32 values to bf16 bit patterns (round to nearest, ties to even)."""
    x = _flat(np.asarray(x, dtype=np.float32))
    out = np.empty(x.shape, dtype=np.uint16)
    lib().pccl_oracle_f32_to_bf16_array(out.ctypes.data, x.ctypes.data, x.size)
    return out


def f32_to_f16(x):
    """Round float32 values to binary16 (round to nearest, ties to even); returns numpy float16."""
    x = _flat(np.asarray(x, dtype=np.float32))
    out = np.empty(x.shape, dtype=np.uint16)
    lib().pccl_oracle_f32_to_f16_array(out.ctypes.data, x.ctypes.data, x.size)
    return out.view(np.float16)


def f16_to_f32(h):
    """Widen binary16 values (numpy float16 or uint16 bit patterns) to float32 (exact)."""
    h = _flat(np.asarray(h)).view(np.uint16)
    out = np.empty(h.shape, dtype=np.uint32)
    lib().pccl_oracle_f16_to_f32_array(out.ctypes.data, h.ctypes.data, h.size)
    return out.view(np.float32)


def bf16_to_f32(bits):
    """Widen bf16 bit patterns to float32 (exact)."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def flat_reduce(srcs, out_dt=None, nthreads=1, average=False):
    """out[e] = ((x0[e] + x1[e]) + ...) in fp32, sources in the order given; with average the
    finished sum is divided by the number of sources before the output rounding."""
    srcs = [_flat(s) for s in srcs]
    in_dt = _dt(srcs[0])
    out_dt = in_dt if out_dt is None else out_dt
    count = srcs[0].size
    assert all(s.size == count and _dt(s) == in_dt for s in srcs)
    out = np.empty(count, dtype=_np_dtype(out_dt))
    rc = lib().pccl_oracle_flat_reduce(out.ctypes.data, _ptr_array(srcs), len(srcs), count,
                                       in_dt, out_dt, len(srcs) if average else 0, nthreads)
    _check(rc, "flat_reduce")
    return out


def two_level_reduce(srcs, nodes, gpus, out_dt=None, want_partials=False, nthreads=1, average=False):
    """Two-level sum of nodes*gpus sources given node-major (srcs[n*gpus+g]); with average the
    finished sum is divided by nodes*gpus (the partials stay plain sums)."""
    srcs = [_flat(s) for s in srcs]
    assert len(srcs) == nodes * gpus
    in_dt = _dt(srcs[0])
    out_dt = in_dt if out_dt is None else out_dt
    count = srcs[0].size
    assert all(s.size == count and _dt(s) == in_dt for s in srcs)
    out = np.empty(count, dtype=_np_dtype(out_dt))
    partials = np.empty((nodes, count), dtype=_np_dtype(in_dt)) if want_partials else None
    rc = lib().pccl_oracle_two_level_reduce(
        out.ctypes.data, partials.ctypes.data if want_partials else None, _ptr_array(srcs),
        nodes, gpus, count, in_dt, out_dt, nodes * gpus if average else 0, nthreads)
    _check(rc, "two_level_reduce")
    return (out, partials) if want_partials else out


def rs_phase1(pieces, nodes, chunk, nthreads=1):
    """partial[n][e] = round_io(sum over g of pieces[g][n][e]); pieces[g] is [nodes][chunk]."""
    pieces = [_flat(p) for p in pieces]
    io_dt = _dt(pieces[0])
    assert all(p.size == nodes * chunk and _dt(p) == io_dt for p in pieces)
    partial = np.empty((nodes, chunk), dtype=_np_dtype(io_dt))
    rc = lib().pccl_oracle_rs_phase1(partial.ctypes.data, _ptr_array(pieces), nodes, len(pieces),
                                     chunk, io_dt, nthreads)
    _check(rc, "rs_phase1")
    return partial


def rs_phase2(inter, out_dt=None, nthreads=1, divisor=0):
    """shard[e] = round_out(sum over n of inter[n][e]), the sum divided by `divisor` first if > 0."""
    inter = [_flat(c) for c in inter]
    io_dt = _dt(inter[0])
    out_dt = io_dt if out_dt is None else out_dt
    chunk = inter[0].size
    shard = np.empty(chunk, dtype=_np_dtype(out_dt))
    rc = lib().pccl_oracle_rs_phase2(shard.ctypes.data, _ptr_array(inter), len(inter), chunk,
                                     io_dt, out_dt, divisor, nthreads)
    _check(rc, "rs_phase2")
    return shard


def reduce_scatter_local(x, my_node=0, inter=None, out_dt=None, nthreads=1, average=False):
    """One GPU's share of a two-level reduce-scatter.

    x: array [gpus][nodes][chunk] (piece g = what node-mate g sent).
    inter: None -> the partial's own rows stand in for what every node sent;
           else a list of `nodes` chunks, entry my_node is ignored and
           partial[my_node] is used in its place.
    average: the shard is the sum over all nodes*gpus ranks divided by that count (one binary32
             division after the last add); the partial stays a plain sum.
    Returns (shard, partial)."""
    gpus, nodes, chunk = x.shape
    partial = rs_phase1([x[g] for g in range(gpus)], nodes, chunk, nthreads)
    if inter is None:
        rows = [partial[n] for n in range(nodes)]
    else:
        rows = [partial[n] if n == my_node else inter[n] for n in range(nodes)]
    shard = rs_phase2(rows, out_dt, nthreads, divisor=gpus * nodes if average else 0)
    return shard, partial


def accumulate(acc, recv, nthreads=1):
    """The literal vector-reduction step: returns round_io(acc + recv) (acc is not modified)."""
    out = np.array(_flat(acc), copy=True)
    recv = _flat(recv)
    io_dt = _dt(out)
    assert recv.size == out.size and _dt(recv) == io_dt
    _check(lib().pccl_oracle_accumulate(out.ctypes.data, recv.ctypes.data, out.size, io_dt, nthreads),
           "accumulate")
    return out.reshape(np.shape(acc))


def ring_chunk_at_step(p, rank, step):
    """Chunk that rank `rank` receives and accumulates at step `step` (0..p-2) of a ring
    reduce-scatter in which every rank sends to rank+1 and rank r ends up owning chunk r."""
    return (rank - 2 - step) % p


def ring_rs_local(msg, recvs, rank, nthreads=1):
    """One rank's reduction work in a ring reduce-scatter over p ranks.
    msg: [p][chunk] local message; recvs[s]: what arrives from rank-1 at step s (p-1 chunks).
    Returns the message buffer after all steps (chunk `rank` is the owned shard)."""
    p = msg.shape[0]
    assert len(recvs) == p - 1
    buf = np.array(msg, copy=True)
    for s in range(p - 1):
        c = ring_chunk_at_step(p, rank, s)
        buf[c] = accumulate(buf[c], recvs[s], nthreads)
    return buf


def halving_kept_range(p, rank, step):
    """(first chunk, number of chunks) rank `rank` keeps and accumulates into at step `step`
    (0..log2(p)-1) of a recursive-halving reduce-scatter: partner = rank xor p/2^(step+1)."""
    if p < 1 or p & (p - 1):
        raise ValueError("recursive halving needs a power-of-two rank count")
    lo, ln = 0, p
    for t in range(step + 1):
        dist = p >> (t + 1)
        ln //= 2
        if rank & dist:
            lo += ln
    return lo, ln


def halving_rs_local(msg, recvs, rank, nthreads=1):
    """One rank's reduction work in a recursive-halving reduce-scatter over p = 2^k ranks.
    msg: [p][chunk]; recvs[t]: the half received at step t ([p/2^(t+1)][chunk]).
    Returns the message buffer after all steps (chunk `rank` is the owned shard)."""
    p = msg.shape[0]
    steps = p.bit_length() - 1
    assert len(recvs) == steps
    buf = np.array(msg, copy=True)
    for t in range(steps):
        lo, ln = halving_kept_range(p, rank, t)
        buf[lo:lo + ln] = accumulate(buf[lo:lo + ln], np.asarray(recvs[t]).reshape(ln, -1), nthreads)
    return buf


def reduce_scatter_local_unpacked(msgs, nodes, gpus, my_gpu, my_node=0, inter=None, out_dt=None,
                                  nthreads=1, average=False):
    """The two-level reduce-scatter share straight from the node-mates' rank-order messages
    (msgs[g2] = [nodes*gpus*chunk], node-mate g2's message): by definition the same as
    pre-shuffling every message and taking piece `my_gpu` of each.  Returns (shard, partial)."""
    assert len(msgs) == gpus
    pieces = []
    for m in msgs:
        packed = hier_pack(np.ascontiguousarray(m).reshape(-1), nodes, gpus)
        pieces.append(packed.reshape(gpus, nodes, -1)[my_gpu])
    return reduce_scatter_local(np.stack(pieces), my_node=my_node, inter=inter, out_dt=out_dt,
                                nthreads=nthreads, average=average)


def _bytes_view(a):
    a = np.ascontiguousarray(a)
    return a.reshape(-1).view(np.uint8)


def hier_pack(src, nodes, gpus):
    """[node][gpu][chunk] -> [gpu][node][chunk]; src is any contiguous array."""
    s = _bytes_view(src)
    assert s.size % (nodes * gpus) == 0
    d = np.empty_like(s)
    _check(lib().pccl_oracle_hier_pack(d.ctypes.data, s.ctypes.data, nodes, gpus,
                                       s.size // (nodes * gpus)), "hier_pack")
    return d.view(src.dtype).reshape(src.shape)


def hier_unpack(src, nodes, gpus):
    """[gpu][node][chunk] -> [node][gpu][chunk]."""
    s = _bytes_view(src)
    assert s.size % (nodes * gpus) == 0
    d = np.empty_like(s)
    _check(lib().pccl_oracle_hier_unpack(d.ctypes.data, s.ctypes.data, nodes, gpus,
                                         s.size // (nodes * gpus)), "hier_unpack")
    return d.view(src.dtype).reshape(src.shape)


def allgather_reassemble(slots, nodes, gpus):
    """slots[g*nodes+n] (one array per hierarchical slot) -> rank-order concatenation."""
    assert len(slots) == nodes * gpus
    views = [_bytes_view(s) for s in slots]
    cb = views[0].size
    assert all(v.size == cb for v in views)
    d = np.empty(cb * len(views), dtype=np.uint8)
    _check(lib().pccl_oracle_allgather_reassemble(d.ctypes.data, _ptr_array(views), nodes, gpus, cb),
           "allgather_reassemble")
    return d.view(slots[0].dtype)


def phase2_reassemble(inter, slots, nodes, gpus, my_node, my_gpu, nthreads=1, divisor=0):
    """The tail of one rank's two-level all-reduce (Section IV-A: all-reduce = two-level
    reduce-scatter, then two-level all-gather), by composition of its two definitions: the
    inter-node phase gives this rank's shard, shard[e] = round_io(sum over n of inter[n][e]);
    the shard is this rank's own contribution to the all-gather, hierarchical slot
    my_gpu*nodes + my_node; the gathered slots are shuffled into rank order.
    slots: one array per hierarchical slot g*nodes+n; the entry at the rank's own slot is
    ignored (None is fine).  Returns the rank-order buffer [nodes*gpus*chunk]."""
    shard = rs_phase2(inter, None, nthreads, divisor)
    filled = list(slots)
    filled[my_gpu * nodes + my_node] = shard
    return allgather_reassemble(filled, nodes, gpus)

