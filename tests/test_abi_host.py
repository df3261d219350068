"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re

import pytest

import paper_2504_18658_amd as pccl
from paper_2504_18658_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = 1 << 20  # a fake, 16-byte aligned "device address"; never dereferenced on these paths


@pytest.fixture(autouse=True)
def _only_without_a_gpu():
    """Every call below must be turned away before any launch.  Should an expectation ever be
    wrong, the call would launch on a made-up address: harmless where no GPU exists (the launch
    fails), not on a GPU machine -- so there these checks do not run."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("host argument checks run on machines without a GPU")


def _header_symbols():
    text = open(os.path.join(ROOT, "include", "pccl_local.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pccl_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = pccl.lib()
    names = _header_symbols()
    assert len(names) >= 9
    for n in names:
        assert hasattr(L, n), "missing export %s" % n
    assert set(names) == set(binding.EXPORTS)


def test_loaded_library_was_built_from_the_sources_on_disk(tmp_path):
    from paper_2504_18658_amd import build
    assert build.source_id() == build.built_id() == pccl.lib().pccl_build_id().decode()
    assert not build.is_stale()
    # a file that is not a build of these sources is recognised as such
    other = tmp_path / "lib.so"
    other.write_bytes(b"\x7fELF" + b"pccl-build-id:0123456789abcdef" + b"\0" * 8)
    assert build.built_id(str(other)) == "0123456789abcdef" != build.source_id()
    other.write_bytes(b"\x7fELF no marker")
    assert build.built_id(str(other)) is None and build.built_id(str(tmp_path / "absent.so")) is None


def test_header_and_binding_constants_agree():
    text = open(os.path.join(ROOT, "include", "pccl_local.h")).read()
    assert int(re.search(r"#define PCCL_MAX_BUCKETS (\d+)", text).group(1)) == pccl.PCCL_MAX_BUCKETS
    for name in ("PCCL_OK", "PCCL_ERR_NULL", "PCCL_ERR_INVALID", "PCCL_ERR_UNSUPPORTED",
                 "PCCL_ERR_OVERLAP", "PCCL_ERR_HIP", "PCCL_F32", "PCCL_BF16", "PCCL_F16", "PCCL_SUM",
                 "PCCL_AVG"):
        m = re.search(r"\b%s = (\d+)" % name, text)
        assert m and int(m.group(1)) == getattr(pccl, name), name
    assert ctypes.sizeof(pccl.pccl_bucket_t) == 40


def test_status_strings():
    for s in range(8):
        assert pccl.status_string(s).startswith("PCCL_")
    assert "unknown" in pccl.status_string(99)


def test_local_reduce_rejects_bad_arguments():
    f = pccl.lib().pccl_local_reduce
    ok = dict(dst=A, src=8 * A, stride=4096, nsrc=4, count=1024, i=0, o=0, op=0)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["dst"], a["src"], a["stride"], a["nsrc"], a["count"], a["i"], a["o"], a["op"], None)

    assert call(dst=None) == pccl.PCCL_ERR_NULL
    assert call(src=None) == pccl.PCCL_ERR_NULL
    assert call(nsrc=0) == pccl.PCCL_ERR_INVALID
    assert call(nsrc=-3) == pccl.PCCL_ERR_INVALID
    assert call(i=3) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(o=7) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(i=1, o=2) == pccl.PCCL_ERR_UNSUPPORTED         # bf16 in, fp16 out: no such pair
    assert call(i=2, o=1) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(op=2) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(op=1, nsrc=(1 << 24) + 1, stride=1 << 12) == pccl.PCCL_ERR_INVALID  # average: count not exact in fp32
    assert call(stride=4092) == pccl.PCCL_ERR_INVALID          # sources would overlap
    assert call(stride=4098, i=0) == pccl.PCCL_ERR_INVALID     # not a multiple of the element size
    assert call(count=(1 << 63)) == pccl.PCCL_ERR_INVALID      # byte size overflows
    assert call(stride=(1 << 63), count=8) == pccl.PCCL_ERR_INVALID  # span overflows
    assert call(dst=A + 2) == pccl.PCCL_ERR_INVALID            # fp32 dst not 4-byte aligned
    assert call(src=8 * A + 1, i=1) == pccl.PCCL_ERR_INVALID   # bf16 src not 2-byte aligned
    assert call(dst=8 * A + 4096) == pccl.PCCL_ERR_OVERLAP     # dst inside source 1
    assert call(dst=8 * A - 4092) == pccl.PCCL_ERR_OVERLAP     # dst tail reaches source 0
    assert call(count=0) == pccl.PCCL_OK                       # empty: nothing launched
    assert call(count=0, dst=None) == pccl.PCCL_ERR_NULL


def test_ptr_reduce_rejects_bad_arguments():
    L = pccl.lib()
    assert L.pccl_local_reduce_ptrs(None, A, 4, 16, 0, 0, 0, None) == pccl.PCCL_ERR_NULL
    assert L.pccl_local_reduce_ptrs(A, None, 4, 16, 0, 0, 0, None) == pccl.PCCL_ERR_NULL
    assert L.pccl_local_reduce_ptrs(A, 2 * A, 0, 16, 0, 0, 0, None) == pccl.PCCL_ERR_INVALID
    assert L.pccl_local_reduce_ptrs(A, 2 * A, 4, 16, 5, 0, 0, None) == pccl.PCCL_ERR_UNSUPPORTED
    assert L.pccl_local_reduce_ptrs(A, 2 * A, 4, 0, 0, 0, 0, None) == pccl.PCCL_OK
    f = L.pccl_local_reduce_ptrs_two_level
    assert f(None, A, 2, 2, 16, 0, 0, 0, None) == pccl.PCCL_ERR_NULL
    assert f(A, 2 * A, 0, 2, 16, 0, 0, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(A, 2 * A, 2, -1, 16, 0, 0, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(A, 2 * A, 1 << 30, 1 << 30, 16, 0, 0, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(A, 2 * A, 2, 2, 16, 0, 0, 3, None) == pccl.PCCL_ERR_UNSUPPORTED
    assert f(A, 2 * A, 2, 2, 0, 0, 0, 0, None) == pccl.PCCL_OK


@pytest.mark.parametrize("name", ["pccl_hier_pack", "pccl_hier_unpack"])
def test_permute_rejects_bad_arguments(name):
    f = getattr(pccl.lib(), name)
    assert f(None, A, 4, 8, 64, None) == pccl.PCCL_ERR_NULL
    assert f(A, None, 4, 8, 64, None) == pccl.PCCL_ERR_NULL
    assert f(A, 8 * A, 0, 8, 64, None) == pccl.PCCL_ERR_INVALID
    assert f(A, 8 * A, 4, -8, 64, None) == pccl.PCCL_ERR_INVALID
    assert f(A, 8 * A, 1 << 20, 1 << 20, 64, None) == pccl.PCCL_ERR_INVALID
    assert f(A, 8 * A, 4, 8, 1 << 62, None) == pccl.PCCL_ERR_INVALID
    assert f(A, A + 64, 4, 8, 64, None) == pccl.PCCL_ERR_OVERLAP
    assert f(A, A, 4, 8, 64, None) == pccl.PCCL_ERR_OVERLAP       # in place is not supported
    assert f(A, 8 * A, 4, 8, 0, None) == pccl.PCCL_OK


def test_reassemble_rejects_bad_arguments():
    f = pccl.lib().pccl_allgather_reassemble
    assert f(None, A, None, 4, 8, 64, None) == pccl.PCCL_ERR_NULL
    assert f(A, None, None, 4, 8, 64, None) == pccl.PCCL_ERR_NULL
    assert f(A, None, 2 * A, 4, 0, 64, None) == pccl.PCCL_ERR_INVALID
    assert f(A, None, 2 * A, 4, 8, 0, None) == pccl.PCCL_OK


def test_reduce_scatter_local_rejects_bad_arguments():
    f = pccl.lib().pccl_reduce_scatter_local
    ok = dict(shard=A, partial=2 * A, intra=8 * A, stride=1 << 16, inter=None, nodes=4, gpus=8, my=0,
              chunk=1024, dt=1, op=0)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["shard"], a["partial"], a["intra"], a["stride"], a["inter"], a["nodes"], a["gpus"],
                 a["my"], a["chunk"], a["dt"], a["op"], None)

    assert call(shard=None, chunk=0) == pccl.PCCL_OK          # no shard: phase 1 only
    assert call(shard=None, partial=None) == pccl.PCCL_ERR_NULL
    assert call(partial=None) == pccl.PCCL_ERR_NULL
    assert call(intra=None) == pccl.PCCL_ERR_NULL
    assert call(nodes=0) == pccl.PCCL_ERR_INVALID
    assert call(gpus=0) == pccl.PCCL_ERR_INVALID
    assert call(my=4) == pccl.PCCL_ERR_INVALID
    assert call(my=-1) == pccl.PCCL_ERR_INVALID
    assert call(dt=9) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(op=2) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(stride=8190) == pccl.PCCL_ERR_INVALID     # piece is 4*1024*2 = 8192 bytes
    assert call(chunk=1 << 62) == pccl.PCCL_ERR_INVALID
    assert call(partial=8 * A + 100) == pccl.PCCL_ERR_OVERLAP
    assert call(shard=8 * A + (7 << 16)) == pccl.PCCL_ERR_OVERLAP
    assert call(shard=2 * A + 4096) == pccl.PCCL_ERR_OVERLAP   # shard inside partial
    assert call(chunk=0) == pccl.PCCL_OK


def test_static_reduce_scatter_local_rejects_bad_arguments():
    f = pccl.lib().pccl_reduce_scatter_local_static
    ok = dict(shard=A, intra=8 * A, stride=1 << 16, inter=None, nodes=4, gpus=8, my=0, chunk=1024, dt=1, op=0)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["shard"], a["intra"], a["stride"], a["inter"], a["nodes"], a["gpus"], a["my"], a["chunk"],
                 a["dt"], a["op"], None)

    assert call(shard=None) == pccl.PCCL_ERR_NULL
    assert call(intra=None) == pccl.PCCL_ERR_NULL
    assert call(nodes=0) == pccl.PCCL_ERR_INVALID
    assert call(my=4) == pccl.PCCL_ERR_INVALID
    assert call(dt=9) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(stride=8190) == pccl.PCCL_ERR_INVALID
    assert call(chunk=1 << 62) == pccl.PCCL_ERR_INVALID
    assert call(shard=8 * A + (7 << 16)) == pccl.PCCL_ERR_OVERLAP
    assert call(chunk=0) == pccl.PCCL_OK
    # the workspace holds 32 MiB of partial: nodes * chunk * element size
    limit = pccl.PCCL_STATIC_SCRATCH_BYTES
    text = open(os.path.join(ROOT, "include", "pccl_local.h")).read()
    assert "#define PCCL_STATIC_SCRATCH_BYTES ((size_t)32 << 20)" in text and limit == 32 << 20
    assert call(nodes=16, chunk=limit // 32 + 1, stride=1 << 40) == pccl.PCCL_ERR_SCRATCH
    assert call(nodes=16, chunk=limit // 64 + 1, dt=0, stride=1 << 40) == pccl.PCCL_ERR_SCRATCH
    assert "SCRATCH" in pccl.status_string(pccl.PCCL_ERR_SCRATCH)


def test_batched_rejects_bad_arguments():
    f = pccl.lib().pccl_reduce_scatter_local_batched
    good = (pccl.pccl_bucket_t * 2)(pccl.pccl_bucket_t(A, 2 * A, 8 * A, 1 << 16, 1024),
                                    pccl.pccl_bucket_t(3 * A, 4 * A, 16 * A, 1 << 16, 512))
    h = ctypes.addressof(good)
    assert f(None, h, 2, 4, 8, 1, 0, None) == pccl.PCCL_ERR_NULL
    assert f(A, None, 2, 4, 8, 1, 0, None) == pccl.PCCL_ERR_NULL
    assert f(A, h, -1, 4, 8, 1, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, pccl.PCCL_MAX_BUCKETS + 1, 4, 8, 1, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, 2, 0, 8, 1, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, 2, 4, 8, 3, 0, None) == pccl.PCCL_ERR_UNSUPPORTED
    assert f(None, None, 0, 4, 8, 1, 0, None) == pccl.PCCL_OK
    bad = (pccl.pccl_bucket_t * 1)(pccl.pccl_bucket_t(A, None, 8 * A, 1 << 16, 1024))
    assert f(A, ctypes.addressof(bad), 1, 4, 8, 1, 0, None) == pccl.PCCL_ERR_NULL
    bad = (pccl.pccl_bucket_t * 1)(pccl.pccl_bucket_t(A, 2 * A, 8 * A, 100, 1024))
    assert f(A, ctypes.addressof(bad), 1, 4, 8, 1, 0, None) == pccl.PCCL_ERR_INVALID
    bad = (pccl.pccl_bucket_t * 1)(pccl.pccl_bucket_t(A, 8 * A, 8 * A, 1 << 16, 1024))
    assert f(A, ctypes.addressof(bad), 1, 4, 8, 1, 0, None) == pccl.PCCL_ERR_OVERLAP
    empty = (pccl.pccl_bucket_t * 1)(pccl.pccl_bucket_t(A, 2 * A, 8 * A, 1 << 16, 0))
    assert f(A, ctypes.addressof(empty), 1, 4, 8, 1, 0, None) == pccl.PCCL_OK


def test_workload_generators_are_seeded_and_shaped():
    from paper_2504_18658_amd import workloads as W
    a, b = W.two_level_input(W.cfg3(chunk=64)), W.two_level_input(W.cfg3(chunk=64))
    assert a.shape == (8, 16, 64) and a.dtype.is_floating_point and bool((a.view(-1).view(dtype=a.dtype) == b.view(-1)).all())
    sizes = W.bucket_sizes_bytes()
    assert len(sizes) == 40 and all(16 * W.MB <= s < 512 * W.MB and s % 1024 == 0 for s in sizes)
    assert sizes == W.bucket_sizes_bytes()
    bits = W.random_bits16(1 << 16, 1)
    assert bits.dtype.itemsize == 2


def test_accumulate_rejects_bad_arguments():
    f = pccl.lib().pccl_accumulate
    assert f(None, A, 8, 0, 0, None) == pccl.PCCL_ERR_NULL
    assert f(A, None, 8, 0, 0, None) == pccl.PCCL_ERR_NULL
    assert f(A, 2 * A, 8, 5, 0, None) == pccl.PCCL_ERR_UNSUPPORTED
    assert f(A, 2 * A, 8, 0, 3, None) == pccl.PCCL_ERR_UNSUPPORTED
    assert f(A, 2 * A, 8, 0, 1, None) == pccl.PCCL_ERR_UNSUPPORTED         # average is not a step op
    assert f(A, 2 * A, 1 << 63, 0, 0, None) == pccl.PCCL_ERR_INVALID       # byte size overflows
    assert f(A + 2, 2 * A, 8, 0, 0, None) == pccl.PCCL_ERR_INVALID         # fp32 not 4-byte aligned
    assert f(A, 2 * A + 1, 8, 1, 0, None) == pccl.PCCL_ERR_INVALID         # bf16 not 2-byte aligned
    assert f(A, A + 16, 8, 0, 0, None) == pccl.PCCL_ERR_OVERLAP            # 32-byte ranges 16 apart
    assert f(A, A, 8, 1, 0, None) == pccl.PCCL_ERR_OVERLAP
    assert f(A, 2 * A, 0, 0, 0, None) == pccl.PCCL_OK                      # empty: nothing launched


def test_ring_local_rejects_bad_arguments():
    f = pccl.lib().pccl_ring_reduce_scatter_local
    ok = dict(msg=A, recv=8 * A, stride=4096, p=8, r=3, c=1024, dt=0, op=0)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["msg"], a["recv"], a["stride"], a["p"], a["r"], a["c"], a["dt"], a["op"], None)

    assert call(msg=None) == pccl.PCCL_ERR_NULL
    assert call(recv=None) == pccl.PCCL_ERR_NULL
    assert call(p=0) == pccl.PCCL_ERR_INVALID
    assert call(r=-1) == pccl.PCCL_ERR_INVALID
    assert call(r=8) == pccl.PCCL_ERR_INVALID
    assert call(dt=9) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(op=2) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(op=1) == pccl.PCCL_ERR_UNSUPPORTED             # a step only adds
    assert call(stride=4092) == pccl.PCCL_ERR_INVALID          # received chunks would overlap
    assert call(stride=4098) == pccl.PCCL_ERR_INVALID          # not a multiple of the element size
    assert call(c=1 << 62) == pccl.PCCL_ERR_INVALID
    assert call(stride=1 << 62, c=4) == pccl.PCCL_ERR_INVALID  # span overflows
    assert call(recv=A + 4096) == pccl.PCCL_ERR_OVERLAP        # recv inside the message
    assert call(msg=8 * A + 6 * 4096) == pccl.PCCL_ERR_OVERLAP # message starts inside the last recv chunk
    assert call(c=0) == pccl.PCCL_OK
    assert call(p=1, r=0, c=0, recv=A) == pccl.PCCL_OK         # one rank: no step, nothing can overlap
    assert call(p=2, r=1, stride=0, c=0) == pccl.PCCL_OK       # a single received chunk: stride unused


def test_halving_local_rejects_bad_arguments():
    f = pccl.lib().pccl_halving_reduce_scatter_local
    ok = dict(msg=A, recv=8 * A, p=8, r=5, c=1024, dt=1, op=0)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["msg"], a["recv"], a["p"], a["r"], a["c"], a["dt"], a["op"], None)

    assert call(msg=None) == pccl.PCCL_ERR_NULL
    assert call(recv=None) == pccl.PCCL_ERR_NULL
    for p in (0, -4, 3, 6, 12):
        assert call(p=p, r=0) == pccl.PCCL_ERR_INVALID         # recursive halving: powers of two only
    assert call(r=8) == pccl.PCCL_ERR_INVALID
    assert call(r=-1) == pccl.PCCL_ERR_INVALID
    assert call(dt=3) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(op=1) == pccl.PCCL_ERR_UNSUPPORTED             # a step only adds
    assert call(c=1 << 62) == pccl.PCCL_ERR_INVALID
    assert call(msg=A + 1) == pccl.PCCL_ERR_INVALID
    assert call(recv=A + 2048) == pccl.PCCL_ERR_OVERLAP
    assert call(msg=8 * A + 7 * 2048 - 2) == pccl.PCCL_ERR_OVERLAP  # last received byte pair
    assert call(c=0) == pccl.PCCL_OK


def test_unpacked_reduce_scatter_rejects_bad_arguments():
    f = pccl.lib().pccl_reduce_scatter_local_unpacked
    # 4 nodes x 2 gpus, 256-element fp32 chunks: a message is 8 KiB, a piece 4 KiB
    ok = dict(shard=A, partial=2 * A, msgs=8 * A, stride=8192, d_msgs=None, d_inter=None, n=4, m=2, my_n=1,
              my_g=1, c=256, dt=0, op=0)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["shard"], a["partial"], a["msgs"], a["stride"], a["d_msgs"], a["d_inter"], a["n"], a["m"],
                 a["my_n"], a["my_g"], a["c"], a["dt"], a["op"], None)

    assert call(shard=None, c=0) == pccl.PCCL_OK               # no shard: phase 1 only
    assert call(partial=None) == pccl.PCCL_ERR_NULL
    assert call(msgs=None) == pccl.PCCL_ERR_NULL               # neither a base nor a pointer array
    assert call(my_g=2) == pccl.PCCL_ERR_INVALID
    assert call(my_g=-1) == pccl.PCCL_ERR_INVALID
    assert call(my_n=4) == pccl.PCCL_ERR_INVALID
    assert call(n=0) == pccl.PCCL_ERR_INVALID
    assert call(n=70000, my_n=0) == pccl.PCCL_ERR_INVALID      # rows of the launch grid
    assert call(stride=8188) == pccl.PCCL_ERR_INVALID          # messages would overlap
    assert call(c=1 << 61) == pccl.PCCL_ERR_INVALID
    assert call(dt=4) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(op=2) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(partial=8 * A + 100 * 4) == pccl.PCCL_ERR_OVERLAP   # partial inside message 0
    assert call(shard=8 * A + 16380) == pccl.PCCL_ERR_OVERLAP       # shard reaches the last message word
    assert call(shard=2 * A + 4092) == pccl.PCCL_ERR_OVERLAP        # shard reaches into the partial
    assert call(c=0) == pccl.PCCL_OK


@pytest.mark.parametrize("name", ["pccl_allgather_reassemble_batched", "pccl_hier_pack_batched"])
def test_batched_permute_rejects_bad_arguments(name):
    f = getattr(pccl.lib(), name)
    good = (pccl.pccl_permute_bucket_t * 2)(pccl.pccl_permute_bucket_t(A, 8 * A, 4096),
                                            pccl.pccl_permute_bucket_t(2 * A, 16 * A, 100))
    h = ctypes.addressof(good)
    assert f(None, h, 2, 4, 8, None) == pccl.PCCL_ERR_NULL
    assert f(A, None, 2, 4, 8, None) == pccl.PCCL_ERR_NULL
    assert f(A, h, -1, 4, 8, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, pccl.PCCL_MAX_BUCKETS + 1, 4, 8, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, 2, 0, 8, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, 2, 4, -2, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, 2, 1 << 20, 1 << 20, None) == pccl.PCCL_ERR_INVALID     # rank count out of range
    assert f(None, None, 0, 4, 8, None) == pccl.PCCL_OK                    # empty batch
    null_dst = (pccl.pccl_permute_bucket_t * 1)(pccl.pccl_permute_bucket_t(None, 8 * A, 64))
    assert f(A, ctypes.addressof(null_dst), 1, 4, 8, None) == pccl.PCCL_ERR_NULL
    over = (pccl.pccl_permute_bucket_t * 1)(pccl.pccl_permute_bucket_t(8 * A + 64, 8 * A, 64))
    assert f(A, ctypes.addressof(over), 1, 4, 8, None) == pccl.PCCL_ERR_OVERLAP
    huge = (pccl.pccl_permute_bucket_t * 1)(pccl.pccl_permute_bucket_t(A, 8 * A, 1 << 62))
    assert f(A, ctypes.addressof(huge), 1, 4, 8, None) == pccl.PCCL_ERR_INVALID  # byte size overflows
    empty = (pccl.pccl_permute_bucket_t * 2)(pccl.pccl_permute_bucket_t(None, None, 0),
                                             pccl.pccl_permute_bucket_t(None, None, 0))
    assert f(A, ctypes.addressof(empty), 2, 4, 8, None) == pccl.PCCL_OK    # only empty buckets: no launch


def test_checked_mode_refuses_addresses_no_kernel_can_reach(monkeypatch):
    """With PCCL_CHECK_POINTERS set, made-up addresses are refused before any launch."""
    L = binding.lib()
    assert L.pccl_check_device_range(None, 0) == pccl.PCCL_OK
    assert L.pccl_check_device_range(None, 16) == pccl.PCCL_ERR_NULL
    assert L.pccl_check_device_range(0x10000, 16) == pccl.PCCL_ERR_ADDRESS
    monkeypatch.setenv("PCCL_CHECK_POINTERS", "1")
    pccl.diag_reload_env()
    a, b = 0x10000000, 0x20000000
    assert L.pccl_local_reduce(a, b, 4096, 2, 1024, pccl.PCCL_F32, pccl.PCCL_F32, pccl.PCCL_SUM, None) == pccl.PCCL_ERR_ADDRESS
    assert L.pccl_accumulate(a, b, 1024, pccl.PCCL_BF16, pccl.PCCL_SUM, None) == pccl.PCCL_ERR_ADDRESS
    assert L.pccl_hier_pack(a, b, 4, 2, 256, None) == pccl.PCCL_ERR_ADDRESS
    assert L.pccl_local_reduce_ptrs(a, b, 4, 1024, pccl.PCCL_F32, pccl.PCCL_F32, pccl.PCCL_SUM, None) == pccl.PCCL_ERR_ADDRESS
    # argument errors still come first, and empty problems still succeed
    assert L.pccl_local_reduce(a, b, 4096, 0, 1024, pccl.PCCL_F32, pccl.PCCL_F32, pccl.PCCL_SUM, None) == pccl.PCCL_ERR_INVALID
    assert L.pccl_local_reduce(a, b, 4096, 2, 0, pccl.PCCL_F32, pccl.PCCL_F32, pccl.PCCL_SUM, None) == pccl.PCCL_OK
    assert "ADDRESS" in pccl.status_string(pccl.PCCL_ERR_ADDRESS)


def test_unpacked_batched_rejects_bad_arguments():
    f = pccl.lib().pccl_reduce_scatter_local_unpacked_batched
    # 4 nodes x 8 GPUs, bf16, chunk 1024 elements: a message is 4*8*1024*2 = 65536 bytes
    good = (pccl.pccl_bucket_t * 1)(pccl.pccl_bucket_t(A, 2 * A, 8 * A, 1 << 16, 1024))
    h = ctypes.addressof(good)
    assert f(None, h, 1, 4, 8, 3, 1, 0, None) == pccl.PCCL_ERR_NULL
    assert f(A, None, 1, 4, 8, 3, 1, 0, None) == pccl.PCCL_ERR_NULL
    assert f(A, h, 1, 4, 8, -1, 1, 0, None) == pccl.PCCL_ERR_INVALID            # my_gpu out of range
    assert f(A, h, 1, 4, 8, 8, 1, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, 1, 0, 8, 3, 1, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, 1, 4, 8, 3, 7, 0, None) == pccl.PCCL_ERR_UNSUPPORTED
    assert f(A, h, pccl.PCCL_MAX_BUCKETS + 1, 4, 8, 3, 1, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(None, None, 0, 4, 8, 3, 1, 0, None) == pccl.PCCL_OK
    # a stride that fits a pre-shuffled piece (4*1024*2 bytes) but not a whole message
    bad = (pccl.pccl_bucket_t * 1)(pccl.pccl_bucket_t(A, 2 * A, 8 * A, 1 << 13, 1024))
    assert f(A, ctypes.addressof(bad), 1, 4, 8, 3, 1, 0, None) == pccl.PCCL_ERR_INVALID
    # the partial inside the span of the eight messages
    bad = (pccl.pccl_bucket_t * 1)(pccl.pccl_bucket_t(A, 8 * A + (5 << 16), 8 * A, 1 << 16, 1024))
    assert f(A, ctypes.addressof(bad), 1, 4, 8, 3, 1, 0, None) == pccl.PCCL_ERR_OVERLAP
    bad = (pccl.pccl_bucket_t * 1)(pccl.pccl_bucket_t(None, 2 * A, 8 * A, 1 << 16, 1024))
    assert f(A, ctypes.addressof(bad), 1, 4, 8, 3, 1, 0, None) == pccl.PCCL_ERR_NULL
    empty = (pccl.pccl_bucket_t * 1)(pccl.pccl_bucket_t(None, None, None, 0, 0))
    assert f(A, ctypes.addressof(empty), 1, 4, 8, 3, 1, 0, None) == pccl.PCCL_OK


def test_phase2_reassemble_rejects_bad_arguments():
    f = pccl.lib().pccl_phase2_reassemble_local
    # 4 nodes x 2 gpus, 256-element fp32 chunks: the result is 8 KiB, the partial 4 KiB
    ok = dict(dst=A, partial=2 * A, inter=None, src=8 * A, slots=None, n=4, m=2, my_n=1, my_g=1, c=256, dt=0, op=0)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["dst"], a["partial"], a["inter"], a["src"], a["slots"], a["n"], a["m"], a["my_n"], a["my_g"],
                 a["c"], a["dt"], a["op"], None)

    assert call(dst=None) == pccl.PCCL_ERR_NULL
    assert call(partial=None) == pccl.PCCL_ERR_NULL
    assert call(src=None) == pccl.PCCL_ERR_NULL                # neither contiguous slots nor a pointer array
    assert call(n=0) == pccl.PCCL_ERR_INVALID
    assert call(m=0) == pccl.PCCL_ERR_INVALID
    assert call(my_n=4) == pccl.PCCL_ERR_INVALID
    assert call(my_g=2) == pccl.PCCL_ERR_INVALID
    assert call(my_g=-1) == pccl.PCCL_ERR_INVALID
    assert call(c=1 << 61) == pccl.PCCL_ERR_INVALID
    assert call(n=1 << 20, m=1 << 12, my_n=0) == pccl.PCCL_ERR_INVALID     # 2^32 ranks
    assert call(dt=5) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(op=3) == pccl.PCCL_ERR_UNSUPPORTED
    assert call(dst=A + 2) == pccl.PCCL_ERR_INVALID            # fp32 result not 4-byte aligned
    assert call(partial=A + 8188) == pccl.PCCL_ERR_OVERLAP     # partial starts in the last word of the result
    assert call(src=A + 4096) == pccl.PCCL_ERR_OVERLAP
    assert call(dst=8 * A + 8188) == pccl.PCCL_ERR_OVERLAP
    assert call(c=0) == pccl.PCCL_OK
    assert call(op=1, n=1 << 13, m=1 << 12, my_n=0, c=0) == pccl.PCCL_ERR_INVALID   # average: 2^25 ranks


def test_accumulate_batched_rejects_bad_arguments():
    f = pccl.lib().pccl_accumulate_batched
    T = pccl.pccl_accumulate_pair_t
    good = (T * 3)(T(A, 8 * A, 1024), T(2 * A, 16 * A, 100), T(None, None, 0))
    h = ctypes.addressof(good)
    assert f(None, h, 3, 0, 0, None) == pccl.PCCL_ERR_NULL
    assert f(A, None, 3, 0, 0, None) == pccl.PCCL_ERR_NULL
    assert f(A, h, -1, 0, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, pccl.PCCL_MAX_BUCKETS + 1, 0, 0, None) == pccl.PCCL_ERR_INVALID
    assert f(A, h, 3, 7, 0, None) == pccl.PCCL_ERR_UNSUPPORTED
    assert f(A, h, 3, 0, 1, None) == pccl.PCCL_ERR_UNSUPPORTED            # a step adds; no average
    assert f(None, None, 0, 0, 0, None) == pccl.PCCL_OK
    empty = (T * 2)(T(None, None, 0), T(A, None, 0))
    assert f(A, ctypes.addressof(empty), 2, 0, 0, None) == pccl.PCCL_OK    # only empty pairs: nothing to launch
    for bad, want in ((T(None, 8 * A, 4), pccl.PCCL_ERR_NULL), (T(A, None, 4), pccl.PCCL_ERR_NULL),
                      (T(A + 2, 8 * A, 4), pccl.PCCL_ERR_INVALID), (T(A, 8 * A, 1 << 62), pccl.PCCL_ERR_INVALID),
                      (T(A, A + 8, 4), pccl.PCCL_ERR_OVERLAP)):
        one = (T * 1)(bad)
        assert f(A, ctypes.addressof(one), 1, 0, 0, None) == want
    # two pairs that update the same elements, or one that reads what another updates
    two = (T * 2)(T(A, 8 * A, 1024), T(A + 4092, 16 * A, 8))
    assert f(A, ctypes.addressof(two), 2, 0, 0, None) == pccl.PCCL_ERR_OVERLAP
    two = (T * 2)(T(A, 8 * A, 1024), T(2 * A, A + 100, 8))
    assert f(A, ctypes.addressof(two), 2, 0, 0, None) == pccl.PCCL_ERR_OVERLAP
    assert ctypes.sizeof(T) == 24

