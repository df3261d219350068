"""ctypes binding of libpccl_local.so: same entry points as include/pccl_local.h.

Argument marshalling only -- tensors become device pointers, dtypes become enum codes, the
current torch stream becomes the hipStream_t.  Every step of the path runs in the library's
kernels; there is no fallback: if the library cannot be loaded or built, calls raise.
"""
import ctypes

import torch

from . import build as _build

PCCL_OK, PCCL_ERR_NULL, PCCL_ERR_INVALID, PCCL_ERR_UNSUPPORTED, PCCL_ERR_OVERLAP, PCCL_ERR_HIP, PCCL_ERR_ADDRESS, \
    PCCL_ERR_SCRATCH = range(8)
PCCL_F32, PCCL_BF16, PCCL_F16 = 0, 1, 2
PCCL_SUM, PCCL_AVG = 0, 1
PCCL_MAX_BUCKETS = 512
PCCL_STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = (
    "pccl_local_reduce", "pccl_local_reduce_ptrs", "pccl_local_reduce_ptrs_two_level",
    "pccl_hier_pack", "pccl_hier_unpack", "pccl_reduce_scatter_local",
    "pccl_allgather_reassemble", "pccl_reduce_scatter_local_batched", "pccl_accumulate",
    "pccl_reduce_scatter_local_unpacked", "pccl_ring_reduce_scatter_local",
    "pccl_allgather_reassemble_batched", "pccl_hier_pack_batched", "pccl_halving_reduce_scatter_local", "pccl_model_ring", "pccl_model_rec",
    "pccl_choose_algorithm", "pccl_model_two_level", "pccl_status_string", "pccl_check_device_range",
    "pccl_reduce_scatter_local_unpacked_batched", "pccl_reduce_scatter_local_static", "pccl_diag_reload_env", "pccl_build_id",
    "pccl_phase2_reassemble_local", "pccl_accumulate_batched",
)
PCCL_ALGO_RING, PCCL_ALGO_REC = 0, 1
_NO_STATUS = ("pccl_status_string", "pccl_model_ring", "pccl_model_rec", "pccl_model_two_level",
              "pccl_diag_reload_env", "pccl_build_id")


class pccl_link_model_t(ctypes.Structure):
    _fields_ = [("alpha_ring_s", ctypes.c_double), ("beta_ring_s_per_byte", ctypes.c_double),
                ("alpha_rec_s", ctypes.c_double), ("beta_rec_s_per_byte", ctypes.c_double)]


class pccl_bucket_t(ctypes.Structure):
    _fields_ = [("shard", ctypes.c_void_p), ("partial", ctypes.c_void_p),
                ("intra_base", ctypes.c_void_p), ("intra_stride_bytes", ctypes.c_size_t),
                ("chunk_count", ctypes.c_size_t)]


class pccl_accumulate_pair_t(ctypes.Structure):
    _fields_ = [("acc", ctypes.c_void_p), ("recv", ctypes.c_void_p), ("count", ctypes.c_size_t)]


class pccl_permute_bucket_t(ctypes.Structure):
    _fields_ = [("dst", ctypes.c_void_p), ("src", ctypes.c_void_p), ("chunk_bytes", ctypes.c_size_t)]


class PcclError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s: %s" % (where, status_string(status)))


_lib = None


def lib():
    """The loaded shared library.  A library that is missing, or that was built from other
    sources than the ones on disk, is rebuilt in-tree with hipcc first; there is no fallback."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if _build.is_stale():
            path = _build.build(force=True)
        L = ctypes.CDLL(path)
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.pccl_local_reduce.argtypes = [vp, vp, sz, i, sz, i, i, i, vp]
        L.pccl_local_reduce_ptrs.argtypes = [vp, vp, i, sz, i, i, i, vp]
        L.pccl_local_reduce_ptrs_two_level.argtypes = [vp, vp, i, i, sz, i, i, i, vp]
        L.pccl_hier_pack.argtypes = [vp, vp, i, i, sz, vp]
        L.pccl_hier_unpack.argtypes = [vp, vp, i, i, sz, vp]
        L.pccl_reduce_scatter_local.argtypes = [vp, vp, vp, sz, vp, i, i, i, sz, i, i, vp]
        L.pccl_reduce_scatter_local_static.argtypes = [vp, vp, sz, vp, i, i, i, sz, i, i, vp]
        L.pccl_allgather_reassemble.argtypes = [vp, vp, vp, i, i, sz, vp]
        L.pccl_phase2_reassemble_local.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, sz, i, i, vp]
        L.pccl_reduce_scatter_local_batched.argtypes = [vp, vp, i, i, i, i, i, vp]
        L.pccl_reduce_scatter_local_unpacked_batched.argtypes = [vp, vp, i, i, i, i, i, i, vp]
        L.pccl_accumulate.argtypes = [vp, vp, sz, i, i, vp]
        L.pccl_accumulate_batched.argtypes = [vp, vp, i, i, i, vp]
        L.pccl_allgather_reassemble_batched.argtypes = [vp, vp, i, i, i, vp]
        L.pccl_hier_pack_batched.argtypes = [vp, vp, i, i, i, vp]
        L.pccl_reduce_scatter_local_unpacked.argtypes = [vp, vp, vp, sz, vp, vp, i, i, i, i, sz, i, i, vp]
        L.pccl_ring_reduce_scatter_local.argtypes = [vp, vp, sz, i, i, sz, i, i, vp]
        L.pccl_halving_reduce_scatter_local.argtypes = [vp, vp, i, i, sz, i, i, vp]
        d = ctypes.c_double
        for name in ("pccl_model_ring", "pccl_model_rec"):
            getattr(L, name).argtypes = [i, d, d, d]
            getattr(L, name).restype = d
        L.pccl_choose_algorithm.argtypes = [i, d, vp, vp, vp, vp]
        L.pccl_model_two_level.argtypes = [i, i, d, i, d, d, d, d, d, d]
        L.pccl_model_two_level.restype = d
        for name in EXPORTS:
            if name not in _NO_STATUS:
                getattr(L, name).restype = i
        L.pccl_check_device_range.argtypes = [vp, ctypes.c_size_t]
        L.pccl_build_id.argtypes = []
        L.pccl_build_id.restype = ctypes.c_char_p
        L.pccl_diag_reload_env.argtypes = []
        L.pccl_diag_reload_env.restype = None
        L.pccl_status_string.argtypes = [i]
        L.pccl_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def diag_reload_env():
    """Have the library read its PCCL_* diagnostic switches from the environment again (it reads
    them once, when it is loaded)."""
    lib().pccl_diag_reload_env()


def status_string(status):
    return lib().pccl_status_string(int(status)).decode()


def pccl_check_device_range(ptr, nbytes=None):
    """Status of the library's reachability test for a tensor (its own extent) or for a raw
    address and byte count; launches nothing."""
    if isinstance(ptr, torch.Tensor):
        nbytes = ptr.numel() * ptr.element_size() if nbytes is None else nbytes
        ptr = ptr.data_ptr()
    return lib().pccl_check_device_range(ctypes.c_void_p(ptr), int(nbytes))


def _check(status, where):
    if status != PCCL_OK:
        raise PcclError(status, where)


def dtype_code(dt):
    if dt == torch.float32:
        return PCCL_F32
    if dt == torch.bfloat16:
        return PCCL_BF16
    if dt == torch.float16:
        return PCCL_F16
    raise TypeError("pccl: dtype must be torch.float32, torch.bfloat16 or torch.float16, got %s" % dt)


def _op(average):
    return PCCL_AVG if average else PCCL_SUM


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


# torch reports address 0 for a tensor without elements; the C ABI wants every pointer non-NULL,
# also for an empty range (which it never dereferences), so such a tensor travels as this address
_EMPTY_RANGE = 0x100


def _dev(t, what):
    if not t.is_cuda:
        raise ValueError("pccl: %s must live in GPU memory" % what)
    p = t.data_ptr()
    return _EMPTY_RANGE if p == 0 and t.numel() == 0 else p


def _rows(t, what):
    """(base pointer, row stride in bytes, rows, row elements) of a tensor whose rows are contiguous."""
    if t.dim() < 2:
        raise ValueError("pccl: %s must have a leading source dimension" % what)
    inner = t[0]
    if not inner.is_contiguous():
        raise ValueError("pccl: every source of %s must be contiguous" % what)
    return _dev(t, what), t.stride(0) * t.element_size(), t.shape[0], inner.numel()


def device_pointer_array(tensors, device=None):
    """A device-resident array of the tensors' device pointers (int64 tensor)."""
    ptrs = [_dev(t, "pointer-array entry") for t in tensors]
    device = tensors[0].device if device is None else device
    return torch.tensor(ptrs, dtype=torch.int64).to(device)


# ------------------------------------------------------------------------------- entry points
def pccl_local_reduce(dst, src, stream=None, average=False):
    """dst[e] = sum over rows s of src[s][e], rows in order; src is [nsrc, ...] with contiguous rows."""
    base, stride, nsrc, count = _rows(src, "src")
    if dst.numel() != count or not dst.is_contiguous():
        raise ValueError("pccl_local_reduce: dst must be contiguous with one source's element count")
    _check(lib().pccl_local_reduce(_dev(dst, "dst"), base, stride, nsrc, count, dtype_code(src.dtype),
                                   dtype_code(dst.dtype), _op(average), _stream(stream)),
           "pccl_local_reduce")
    return dst


def pccl_local_reduce_ptrs(dst, d_srcs, count, in_dtype, stream=None, average=False):
    """Flat sum over a device pointer array (int64 tensor) of sources holding `count` elements."""
    _check(lib().pccl_local_reduce_ptrs(_dev(dst, "dst"), _dev(d_srcs, "d_srcs"), d_srcs.numel(), count,
                                        dtype_code(in_dtype), dtype_code(dst.dtype), _op(average),
                                        _stream(stream)), "pccl_local_reduce_ptrs")
    return dst


def pccl_local_reduce_ptrs_two_level(dst, d_srcs, nodes, gpus_per_node, count, in_dtype, stream=None,
                                     average=False):
    """Two-level sum over a node-major device pointer array: d_srcs[n*gpus_per_node + g]."""
    if d_srcs.numel() != nodes * gpus_per_node:
        raise ValueError("pccl_local_reduce_ptrs_two_level: need nodes*gpus_per_node pointers")
    _check(lib().pccl_local_reduce_ptrs_two_level(
        _dev(dst, "dst"), _dev(d_srcs, "d_srcs"), nodes, gpus_per_node, count, dtype_code(in_dtype),
        dtype_code(dst.dtype), _op(average), _stream(stream)), "pccl_local_reduce_ptrs_two_level")
    return dst


def _chunk_bytes(t, nodes, gpus, where):
    total = t.numel() * t.element_size()
    if not t.is_contiguous() or total % (nodes * gpus) != 0:
        raise ValueError("%s: buffer must be contiguous and hold nodes*gpus equal chunks" % where)
    return total // (nodes * gpus)


def pccl_hier_pack(dst, src, nodes, gpus_per_node, stream=None):
    """Rank order [node][gpu][chunk] -> hierarchical order [gpu][node][chunk]."""
    cb = _chunk_bytes(src, nodes, gpus_per_node, "pccl_hier_pack")
    if _chunk_bytes(dst, nodes, gpus_per_node, "pccl_hier_pack") != cb:
        raise ValueError("pccl_hier_pack: dst and src sizes differ")
    _check(lib().pccl_hier_pack(_dev(dst, "dst"), _dev(src, "src"), nodes, gpus_per_node, cb,
                                _stream(stream)), "pccl_hier_pack")
    return dst


def pccl_hier_unpack(dst, src, nodes, gpus_per_node, stream=None):
    """Hierarchical order [gpu][node][chunk] -> rank order [node][gpu][chunk]."""
    cb = _chunk_bytes(src, nodes, gpus_per_node, "pccl_hier_unpack")
    if _chunk_bytes(dst, nodes, gpus_per_node, "pccl_hier_unpack") != cb:
        raise ValueError("pccl_hier_unpack: dst and src sizes differ")
    _check(lib().pccl_hier_unpack(_dev(dst, "dst"), _dev(src, "src"), nodes, gpus_per_node, cb,
                                  _stream(stream)), "pccl_hier_unpack")
    return dst


def pccl_reduce_scatter_local(shard, partial, intra, d_inter=None, my_node=0, stream=None, average=False):
    """One GPU's share of a two-level reduce-scatter.

    intra: [gpus][nodes][chunk] (piece g' = intra[g'], rows may be strided apart);
    partial: [nodes][chunk] scratch/output; shard: [chunk]; d_inter: optional int64 device
    tensor of `nodes` pointers to the chunks received from the other nodes.  shard=None: phase 1 only."""
    if intra.dim() != 3:
        raise ValueError("pccl_reduce_scatter_local: intra must be [gpus][nodes][chunk]")
    base, stride, gpus, _ = _rows(intra, "intra")
    nodes, chunk = intra.shape[1], intra.shape[2]
    if partial.numel() != nodes * chunk or partial.dtype != intra.dtype or not partial.is_contiguous() or \
            (shard is not None and (shard.numel() != chunk or shard.dtype != intra.dtype or
                                    not shard.is_contiguous())):
        raise ValueError("pccl_reduce_scatter_local: partial is [nodes][chunk], shard is [chunk], "
                         "both contiguous and of the message dtype")
    _check(lib().pccl_reduce_scatter_local(
        None if shard is None else _dev(shard, "shard"), _dev(partial, "partial"), base, stride,
        None if d_inter is None else _dev(d_inter, "d_inter"), nodes, gpus, my_node, chunk,
        dtype_code(intra.dtype), _op(average), _stream(stream)), "pccl_reduce_scatter_local")
    return shard


def pccl_reduce_scatter_local_static(shard, intra, d_inter=None, my_node=0, stream=None, average=False):
    """pccl_reduce_scatter_local with the phase-1 result in the library's static workspace (no
    `partial` argument; nodes*chunk*element size at most PCCL_STATIC_SCRATCH_BYTES)."""
    if intra.dim() != 3:
        raise ValueError("pccl_reduce_scatter_local_static: intra must be [gpus][nodes][chunk]")
    base, stride, gpus, _ = _rows(intra, "intra")
    nodes, chunk = intra.shape[1], intra.shape[2]
    if shard.numel() != chunk or shard.dtype != intra.dtype or not shard.is_contiguous():
        raise ValueError("pccl_reduce_scatter_local_static: shard is [chunk], contiguous, of the message dtype")
    _check(lib().pccl_reduce_scatter_local_static(
        _dev(shard, "shard"), base, stride, None if d_inter is None else _dev(d_inter, "d_inter"), nodes, gpus,
        my_node, chunk, dtype_code(intra.dtype), _op(average), _stream(stream)), "pccl_reduce_scatter_local_static")
    return shard


def pccl_allgather_reassemble(dst, src=None, d_slots=None, nodes=1, gpus_per_node=1, stream=None):
    """Hierarchical slots (contiguous src, or int64 device pointer tensor d_slots) -> rank order."""
    cb = _chunk_bytes(dst, nodes, gpus_per_node, "pccl_allgather_reassemble")
    _check(lib().pccl_allgather_reassemble(
        _dev(dst, "dst"), None if src is None else _dev(src, "src"),
        None if d_slots is None else _dev(d_slots, "d_slots"), nodes, gpus_per_node, cb,
        _stream(stream)), "pccl_allgather_reassemble")
    return dst


def pccl_phase2_reassemble_local(dst, partial, d_inter=None, src=None, d_slots=None, nodes=1, gpus_per_node=1,
                                 my_node=0, my_gpu=0, stream=None, average=False):
    """The all-reduce tail in one launch: the inter-node phase into the rank's own chunk of dst, and
    the other chunks from their hierarchical slots (contiguous src, or int64 pointer tensor d_slots)
    into rank order.  partial: [nodes][chunk] phase-1 result; dst: [nodes*gpus*chunk]."""
    if partial.numel() % nodes != 0:
        raise ValueError("pccl_phase2_reassemble_local: partial is [nodes][chunk]")
    chunk = partial.numel() // nodes
    if dst.numel() != nodes * gpus_per_node * chunk or dst.dtype != partial.dtype or not dst.is_contiguous() or \
            not partial.is_contiguous() or (src is not None and (src.numel() != dst.numel() or
                                                                 src.dtype != dst.dtype or not src.is_contiguous())):
        raise ValueError("pccl_phase2_reassemble_local: dst and src are [nodes*gpus*chunk] of partial's dtype")
    _check(lib().pccl_phase2_reassemble_local(
        _dev(dst, "dst"), _dev(partial, "partial"), None if d_inter is None else _dev(d_inter, "d_inter"),
        None if src is None else _dev(src, "src"), None if d_slots is None else _dev(d_slots, "d_slots"),
        nodes, gpus_per_node, my_node, my_gpu, chunk, dtype_code(partial.dtype), _op(average), _stream(stream)),
        "pccl_phase2_reassemble_local")
    return dst


class BucketTable:
    """Descriptor table of a batch: a host array and its device copy, built once and reused."""

    def __init__(self, buckets, nodes=None):
        """buckets: list of (shard, partial, intra) tensors shaped as for pccl_reduce_scatter_local;
        with `nodes` given, the third tensor of a bucket is instead [gpus][nodes*gpus*chunk]: the
        node-mates' rank-order messages (for pccl_reduce_scatter_local_unpacked_batched)."""
        n = len(buckets)
        self.host = (pccl_bucket_t * max(n, 1))()
        self.nbuckets = n
        self.nodes = self.gpus = None
        self.dtype = None
        self.from_messages = nodes is not None
        for k, (shard, partial, intra) in enumerate(buckets):
            base, stride, gpus, row = _rows(intra, "intra")
            if self.from_messages:
                if intra.dim() != 2 or row % (nodes * gpus) != 0:
                    raise ValueError("BucketTable: messages must be [gpus][nodes*gpus*chunk]")
                chunk = row // (nodes * gpus)
            else:
                nodes, chunk = intra.shape[1], intra.shape[2]
            if self.nodes is None:
                self.nodes, self.gpus, self.dtype = nodes, gpus, intra.dtype
            if (nodes, gpus, intra.dtype) != (self.nodes, self.gpus, self.dtype):
                raise ValueError("BucketTable: nodes, gpus and dtype are common to a batch")
            self.host[k] = pccl_bucket_t(_dev(shard, "shard"), _dev(partial, "partial"), base, stride, chunk)
        raw = bytes(self.host)[: n * ctypes.sizeof(pccl_bucket_t)]
        dev = buckets[0][0].device if n else "cuda"
        self.device = torch.frombuffer(bytearray(raw), dtype=torch.uint8).to(dev) if n else None
        self._keep = buckets  # the table holds raw pointers: keep the tensors alive


def pccl_reduce_scatter_local_unpacked_batched(table, my_gpu, stream=None, average=False):
    """All buckets of a BucketTable built from rank-order messages (nodes=...): no pre-shuffle pass."""
    if table.nbuckets == 0:
        return
    if not table.from_messages:
        raise ValueError("pccl_reduce_scatter_local_unpacked_batched: build the table with nodes=...")
    _check(lib().pccl_reduce_scatter_local_unpacked_batched(
        table.device.data_ptr(), ctypes.addressof(table.host), table.nbuckets, table.nodes, table.gpus, my_gpu,
        dtype_code(table.dtype), _op(average), _stream(stream)), "pccl_reduce_scatter_local_unpacked_batched")


def pccl_reduce_scatter_local_batched(table, stream=None, average=False):
    """All buckets of a BucketTable: phase 1 in one launch, phase 2 in one launch."""
    if table.nbuckets == 0:
        return
    if table.from_messages:
        raise ValueError("pccl_reduce_scatter_local_batched: this table holds rank-order messages")
    _check(lib().pccl_reduce_scatter_local_batched(
        table.device.data_ptr(), ctypes.addressof(table.host), table.nbuckets, table.nodes, table.gpus,
        dtype_code(table.dtype), _op(average), _stream(stream)), "pccl_reduce_scatter_local_batched")


def pccl_accumulate(acc, recv, stream=None):
    """acc += recv in place (the literal vector-reduction step); both contiguous, same dtype and size."""
    if acc.dtype != recv.dtype or acc.numel() != recv.numel() or not acc.is_contiguous() or \
            not recv.is_contiguous():
        raise ValueError("pccl_accumulate: acc and recv must be contiguous, of one dtype and size")
    _check(lib().pccl_accumulate(_dev(acc, "acc"), _dev(recv, "recv"), acc.numel(), dtype_code(acc.dtype),
                                 PCCL_SUM, _stream(stream)), "pccl_accumulate")
    return acc


class AccumulateTable:
    """Descriptor table of a batch of acc += recv steps: host array + device copy, built once and reused."""

    def __init__(self, pairs):
        """pairs: list of (acc, recv) contiguous tensors of one dtype, equal sizes within a pair."""
        n = len(pairs)
        self.host = (pccl_accumulate_pair_t * max(n, 1))()
        self.npairs = n
        self.dtype = pairs[0][0].dtype if n else torch.float32
        for k, (acc, recv) in enumerate(pairs):
            if acc.dtype != self.dtype or recv.dtype != self.dtype or acc.numel() != recv.numel() or \
                    not acc.is_contiguous() or not recv.is_contiguous():
                raise ValueError("AccumulateTable: acc and recv must be contiguous, of one dtype, equal in size")
            c = acc.numel()
            self.host[k] = pccl_accumulate_pair_t(_dev(acc, "acc") if c else None, _dev(recv, "recv") if c else None, c)
        raw = bytes(self.host)[: n * ctypes.sizeof(pccl_accumulate_pair_t)]
        dev = pairs[0][0].device if n else "cuda"
        self.device = torch.frombuffer(bytearray(raw), dtype=torch.uint8).to(dev) if n else None
        self._keep = pairs  # the table holds raw pointers: keep the tensors alive


def pccl_accumulate_batched(table, stream=None):
    """Every pair of an AccumulateTable: acc += recv, one launch."""
    if table.npairs == 0:
        return
    _check(lib().pccl_accumulate_batched(table.device.data_ptr(), ctypes.addressof(table.host), table.npairs,
                                         dtype_code(table.dtype), PCCL_SUM, _stream(stream)), "pccl_accumulate_batched")


def pccl_ring_reduce_scatter_local(msg, recv, rank, stream=None):
    """One rank's reduction work of a ring reduce-scatter.  msg: [nranks][chunk], updated in place;
    recv: [nranks-1][chunk] (row s = what arrives at step s; rows may be strided apart)."""
    nranks, chunk = msg.shape
    if not msg.is_contiguous() or msg.dtype != recv.dtype:
        raise ValueError("pccl_ring_reduce_scatter_local: msg must be contiguous, recv of the same dtype")
    if nranks > 1:
        base, stride, rows, count = _rows(recv, "recv")
        if rows != nranks - 1 or count != chunk:
            raise ValueError("pccl_ring_reduce_scatter_local: recv must be [nranks-1][chunk]")
    else:
        base, stride = _dev(recv, "recv"), 0
    _check(lib().pccl_ring_reduce_scatter_local(_dev(msg, "msg"), base, stride, nranks, rank, chunk,
                                                dtype_code(msg.dtype), PCCL_SUM, _stream(stream)),
           "pccl_ring_reduce_scatter_local")
    return msg


def pccl_halving_reduce_scatter_local(msg, recv, rank, stream=None):
    """One rank's reduction work of a recursive-halving reduce-scatter.  msg: [nranks][chunk],
    updated in place; recv: the received halves back to back, (nranks-1)*chunk elements."""
    nranks, chunk = msg.shape
    if not msg.is_contiguous() or not recv.is_contiguous() or msg.dtype != recv.dtype or \
            recv.numel() != max(nranks - 1, 0) * chunk and nranks > 1:
        raise ValueError("pccl_halving_reduce_scatter_local: recv must hold (nranks-1)*chunk elements "
                         "of msg's dtype, both contiguous")
    _check(lib().pccl_halving_reduce_scatter_local(_dev(msg, "msg"), _dev(recv, "recv"), nranks, rank, chunk,
                                                   dtype_code(msg.dtype), PCCL_SUM, _stream(stream)),
           "pccl_halving_reduce_scatter_local")
    return msg


def pccl_reduce_scatter_local_unpacked(shard, partial, msgs=None, d_msgs=None, d_inter=None, nodes=1,
                                       gpus_per_node=1, my_node=0, my_gpu=0, stream=None, average=False):
    """The two-level reduce-scatter share straight from the node-mates' rank-order messages.

    msgs: [gpus][nodes*gpus*chunk] tensor (row g' = node-mate g's message, rows may be strided
    apart), or d_msgs: int64 device tensor of `gpus` pointers to such messages.
    shard=None: phase 1 only (the chunk size then follows from partial)."""
    only_phase1 = shard is None
    if only_phase1:
        if partial.numel() % nodes != 0:
            raise ValueError("pccl_reduce_scatter_local_unpacked: partial is [nodes][chunk]")
        shard = partial[: partial.numel() // nodes]              # stands in for the dtype and chunk size only
    chunk = shard.numel()
    if partial.numel() != nodes * chunk or partial.dtype != shard.dtype or \
            not partial.is_contiguous() or not shard.is_contiguous():
        raise ValueError("pccl_reduce_scatter_local_unpacked: partial is [nodes][chunk], shard is [chunk]")
    if d_msgs is None:
        base, stride, rows, count = _rows(msgs, "msgs")
        if rows != gpus_per_node or count != nodes * gpus_per_node * chunk or msgs.dtype != shard.dtype:
            raise ValueError("pccl_reduce_scatter_local_unpacked: msgs must be [gpus][nodes*gpus*chunk]")
    else:
        base, stride = None, 0
        if d_msgs.numel() != gpus_per_node:
            raise ValueError("pccl_reduce_scatter_local_unpacked: need gpus_per_node message pointers")
    _check(lib().pccl_reduce_scatter_local_unpacked(
        None if only_phase1 else _dev(shard, "shard"), _dev(partial, "partial"), base, stride,
        None if d_msgs is None else _dev(d_msgs, "d_msgs"),
        None if d_inter is None else _dev(d_inter, "d_inter"), nodes, gpus_per_node, my_node, my_gpu, chunk,
        dtype_code(shard.dtype), _op(average), _stream(stream)), "pccl_reduce_scatter_local_unpacked")
    return None if only_phase1 else shard


def pccl_choose_algorithm(p, m_bytes, alpha_ring, beta_ring, alpha_rec, beta_rec):
    """(PCCL_ALGO_RING or PCCL_ALGO_REC, modelled ring seconds, modelled recursive seconds)."""
    model = pccl_link_model_t(alpha_ring, beta_ring, alpha_rec, beta_rec)
    algo, tr, tc = ctypes.c_int(-1), ctypes.c_double(), ctypes.c_double()
    _check(lib().pccl_choose_algorithm(p, m_bytes, ctypes.byref(model), ctypes.byref(algo), ctypes.byref(tr),
                                       ctypes.byref(tc)), "pccl_choose_algorithm")
    return algo.value, tr.value, tc.value


class PermuteTable:
    """Descriptor table of a batched shuffle: host array + device copy, built once and reused."""

    def __init__(self, pairs, nodes, gpus_per_node):
        """pairs: list of (dst, src) contiguous tensors, each holding nodes*gpus_per_node equal chunks."""
        n = len(pairs)
        self.host = (pccl_permute_bucket_t * max(n, 1))()
        self.nbuckets, self.nodes, self.gpus = n, nodes, gpus_per_node
        for k, (dst, src) in enumerate(pairs):
            cb = _chunk_bytes(src, nodes, gpus_per_node, "PermuteTable")
            if _chunk_bytes(dst, nodes, gpus_per_node, "PermuteTable") != cb:
                raise ValueError("PermuteTable: dst and src sizes differ")
            self.host[k] = pccl_permute_bucket_t(_dev(dst, "dst") if cb else None, _dev(src, "src") if cb else None, cb)
        raw = bytes(self.host)[: n * ctypes.sizeof(pccl_permute_bucket_t)]
        dev = pairs[0][0].device if n else "cuda"
        self.device = torch.frombuffer(bytearray(raw), dtype=torch.uint8).to(dev) if n else None
        self._keep = pairs  # the table holds raw pointers: keep the tensors alive


def _permute_batched(name, table, stream):
    if table.nbuckets == 0:
        return
    _check(getattr(lib(), name)(table.device.data_ptr(), ctypes.addressof(table.host), table.nbuckets, table.nodes,
                                table.gpus, _stream(stream)), name)


def pccl_allgather_reassemble_batched(table, stream=None):
    """Every bucket of a PermuteTable: hierarchical order -> rank order, one launch."""
    _permute_batched("pccl_allgather_reassemble_batched", table, stream)


def pccl_hier_pack_batched(table, stream=None):
    """Every bucket of a PermuteTable: rank order -> hierarchical order, one launch."""
    _permute_batched("pccl_hier_pack_batched", table, stream)
