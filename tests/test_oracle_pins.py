"""Pins for the CPU oracle: every check here compares the oracle with something other
than itself -- hand-worked IEEE cases (tests/golden), closed forms, brute force in pure
Python, numpy/torch library routines that coincide with a special case, and a literal
copy-by-copy simulation of the paper's three all-gather steps (Section IV-A)."""
import functools
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import world


# ----------------------------------------------------------------------------- helpers
def _parse_float(tok):
    return float.fromhex(tok) if "0x" in tok.lower() else float(tok)


def _read_cases(path):
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line


def _torch_bf16_bits(x32):
    """Independent bf16 rounding: torch's CPU cast (library routine)."""
    t = torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def _bf16_bits_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _brute_two_level(srcs32, nodes, gpus, round_partial_bf16, round_out_bf16):
    """Pure-Python double loop with numpy float32 scalars; bf16 rounding through torch."""
    count = len(srcs32[0])
    out = np.empty(count, dtype=np.float32)
    for e in range(count):
        acc = None
        for n in range(nodes):
            t = np.float32(srcs32[n * gpus][e])
            for g in range(1, gpus):
                t = np.float32(t + np.float32(srcs32[n * gpus + g][e]))
            if round_partial_bf16:
                t = _bf16_bits_to_f32(_torch_bf16_bits(np.array([t])))[0]
            acc = t if acc is None else np.float32(acc + t)
        out[e] = acc
    if round_out_bf16:
        return _torch_bf16_bits(out)
    return out


def _same_bits(a, b):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    return a.dtype == b.dtype and a.shape == b.shape and a.tobytes() == b.tobytes()


# ----------------------------------------------------------------------------- bf16 rounding
def test_bf16_rne_hand_cases(golden_dir):
    n = 0
    for line in _read_cases(os.path.join(golden_dir, "bf16_rne_cases.txt")):
        f32_hex, bf16_hex = line.split()[:2]
        got = oracle.lib().pccl_oracle_f32_to_bf16(int(f32_hex, 16))
        assert got == int(bf16_hex, 16), line
        n += 1
    assert n >= 15


def test_bf16_rne_textbook_definition_stratified():
    """Nearest representable, ties to even kept mantissa, computed exactly in float64 for all
    2^16 upper halves x the lower halves around every decision point."""
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    rng = np.random.default_rng(123)
    lows = np.concatenate([np.array([0, 1, 2, 0x7FFE, 0x7FFF, 0x8000, 0x8001, 0x8002, 0xFFFE, 0xFFFF],
                                    dtype=np.uint32), rng.integers(0, 1 << 16, 22).astype(np.uint32)])
    for low in lows:
        u = hi | low
        mag = u & np.uint32(0x7FFFFFFF)
        finite = mag < np.uint32(0x7F800000)
        u, mag = u[finite], mag[finite]
        lo_bits = mag & np.uint32(0xFFFF0000)
        hi_bits = lo_bits + np.uint32(0x10000)
        x = mag.view(np.float32).astype(np.float64)
        lo_v = lo_bits.view(np.float32).astype(np.float64)
        hi_v = np.where(hi_bits == np.uint32(0x7F800000), 2.0 ** 128,
                        hi_bits.view(np.float32).astype(np.float64))
        d_lo, d_hi = x - lo_v, hi_v - x
        kept_odd = ((lo_bits >> 16) & 1).astype(bool)
        up = (d_hi < d_lo) | ((d_hi == d_lo) & kept_odd)
        want_mag = np.where(up, hi_bits, lo_bits) >> 16
        want = (want_mag | ((u >> 31) << 15)).astype(np.uint16)
        got = oracle.f32_to_bf16(u.view(np.float32))
        assert np.array_equal(got, want), hex(int(low))


def test_bf16_rne_exhaustive_against_torch_cast():
    """All 2^32 binary32 patterns against torch's CPU float32->bfloat16 cast; NaNs by NaN-ness."""
    step = 1 << 22  # small enough to stay cache- and page-friendly
    base = np.arange(step, dtype=np.uint32)
    for start in range(0, 1 << 32, step):
        u = base + np.uint32(start)
        x = u.view(np.float32)
        got = oracle.f32_to_bf16(x)
        want = _torch_bf16_bits(x)
        if start >> 23 & 0xFF != 0xFF:  # no NaN in this block
            assert np.array_equal(got, want), hex(start)
            continue
        nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
        assert np.array_equal(got[~nan], want[~nan]), hex(start)
        g = got[nan]
        assert np.all((g & 0x7FFF) > 0x7F80), "NaN must stay NaN"
        assert np.array_equal(g >> 15, (u[nan] >> 31).astype(np.uint16)), "NaN keeps its sign"


def test_bf16_widening_is_exact():
    bits = np.arange(1 << 16, dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    got = oracle.bf16_to_f32(bits)
    assert _same_bits(got.view(np.uint32), want.view(np.uint32))


# ----------------------------------------------------------------------------- flat reduce
def test_order_cases_by_hand(golden_dir):
    n = 0
    for line in _read_cases(os.path.join(golden_dir, "fp32_order_cases.txt")):
        shape, terms, expected = [p.strip() for p in line.split("|")]
        nodes, gpus = map(int, shape.split())
        vals = [np.array([_parse_float(t)], dtype=np.float32) for t in terms.split()]
        assert len(vals) == nodes * gpus, line
        want = np.array([_parse_float(expected)], dtype=np.float32)
        got2 = oracle.two_level_reduce(vals, nodes, gpus)
        assert _same_bits(got2, want), (line, got2)
        if nodes == 1:
            got1 = oracle.flat_reduce(vals)
            assert _same_bits(got1, want), (line, got1)
        n += 1
    assert n >= 10


def test_bf16_partial_rounding_by_hand(golden_dir):
    for line in _read_cases(os.path.join(golden_dir, "bf16_partial_rounding_cases.txt")):
        shape, terms, expected, unrounded = [p.strip() for p in line.split("|")]
        nodes, gpus = map(int, shape.split())
        vals32 = [np.array([_parse_float(t)], dtype=np.float32) for t in terms.split()]
        vals = [_torch_bf16_bits(v) for v in vals32]
        for v, v32 in zip(vals, vals32):  # the terms themselves are bf16 values
            assert _bf16_bits_to_f32(v)[0] == v32[0]
        got = oracle.two_level_reduce(vals, nodes, gpus)
        assert _bf16_bits_to_f32(got)[0] == np.float32(_parse_float(expected)), line
        # the same terms summed flat never round in between and give the other value
        flat = oracle.flat_reduce(vals)
        assert _bf16_bits_to_f32(flat)[0] == np.float32(_parse_float(unrounded)), line
        # fp32 output of the two-level sum still sees bf16-rounded partials
        got32 = oracle.two_level_reduce(vals, nodes, gpus, out_dt=oracle.F32)
        assert got32.dtype == np.float32


@pytest.mark.parametrize("S", [1, 2, 3, 8, 16])
def test_flat_equals_sequential_numpy_add(S):
    rng = np.random.default_rng(S)
    srcs = [rng.uniform(-1, 1, 257).astype(np.float32) for _ in range(S)]
    want = functools.reduce(np.add, srcs)  # strictly left-to-right binary32 adds
    got = oracle.flat_reduce(srcs)
    assert _same_bits(got, np.asarray(want, dtype=np.float32))


@pytest.mark.parametrize("S,count", [(1, 5), (2, 7), (5, 64), (16, 33)])
@pytest.mark.parametrize("io", ["f32", "bf16", "bf16_f32"])
def test_flat_brute_force(S, count, io):
    rng = np.random.default_rng(100 * S + count)
    src32 = [rng.normal(0, 1, count).astype(np.float32) for _ in range(S)]
    if io == "f32":
        got = oracle.flat_reduce(src32)
        want = _brute_two_level(src32, 1, S, False, False)
    else:
        bits = [_torch_bf16_bits(s) for s in src32]
        src32 = [_bf16_bits_to_f32(b) for b in bits]
        out_bf16 = io == "bf16"
        got = oracle.flat_reduce(bits, out_dt=oracle.BF16 if out_bf16 else oracle.F32)
        want = _brute_two_level(src32, 1, S, False, out_bf16)
    assert _same_bits(got, want)


def test_flat_integer_closed_form():
    # x_s[e] = (s+1) * 2^k(e): exact in fp32 and bf16, sum = S(S+1)/2 * 2^k for every order
    for S in (1, 2, 8, 15):
        k = np.arange(-6, 7)
        scale = (2.0 ** k).astype(np.float32)
        srcs = [np.float32(s + 1) * scale for s in range(S)]
        want = np.float32(S * (S + 1) / 2) * scale
        assert _same_bits(oracle.flat_reduce(srcs), want)
        bits = [_torch_bf16_bits(s) for s in srcs]
        assert _same_bits(oracle.bf16_to_f32(oracle.flat_reduce(bits)), want)
        assert _same_bits(oracle.flat_reduce(bits, out_dt=oracle.F32), want)


def test_single_source_is_exact_copy():
    x = np.array([-0.0, 0.0, 1e-45, -3.5, np.inf, 1.17549435e-38], dtype=np.float32)
    assert _same_bits(oracle.flat_reduce([x]), x)
    assert _same_bits(oracle.two_level_reduce([x], 1, 1), x)
    b = np.arange(0, 1 << 16, 7, dtype=np.uint16)
    b = b[((b & 0x7FFF) <= 0x7F80)]  # NaN payloads are not pinned
    assert _same_bits(oracle.flat_reduce([b]), b)


def test_accuracy_bound_against_float64():
    rng = np.random.default_rng(7)
    for S in (8, 64, 300):
        srcs = [rng.normal(0, 1, 500).astype(np.float32) for _ in range(S)]
        got = oracle.flat_reduce(srcs).astype(np.float64)
        ref = np.sum(np.stack(srcs).astype(np.float64), axis=0)
        bound = (S - 1) * 2.0 ** -24 * np.sum(np.abs(np.stack(srcs)).astype(np.float64), axis=0)
        assert np.all(np.abs(got - ref) <= bound * (1 + 1e-6))
        # and the sum is not trivially wrong by a dropped term
        assert np.all(np.abs(got - ref) < 0.01 * np.max(np.abs(np.stack(srcs)), axis=0) + 1e-3)


# ----------------------------------------------------------------------------- two-level reduce
@pytest.mark.parametrize("nodes,gpus,count", [(2, 2, 9), (3, 4, 17), (4, 1, 8), (1, 5, 8), (5, 3, 64)])
@pytest.mark.parametrize("io", ["f32", "bf16", "bf16_f32"])
def test_two_level_brute_force(nodes, gpus, count, io):
    rng = np.random.default_rng(nodes * 1000 + gpus * 10 + count)
    src32 = [rng.uniform(-1, 1, count).astype(np.float32) for _ in range(nodes * gpus)]
    if io == "f32":
        got, parts = oracle.two_level_reduce(src32, nodes, gpus, want_partials=True)
        want = _brute_two_level(src32, nodes, gpus, False, False)
        for n in range(nodes):
            assert _same_bits(parts[n], _brute_two_level(src32[n * gpus:(n + 1) * gpus], 1, gpus, False, False))
    else:
        bits = [_torch_bf16_bits(s) for s in src32]
        src32 = [_bf16_bits_to_f32(b) for b in bits]
        out_bf16 = io == "bf16"
        got, parts = oracle.two_level_reduce(bits, nodes, gpus, want_partials=True,
                                             out_dt=oracle.BF16 if out_bf16 else oracle.F32)
        want = _brute_two_level(src32, nodes, gpus, True, out_bf16)
        for n in range(nodes):
            assert _same_bits(parts[n], _brute_two_level(src32[n * gpus:(n + 1) * gpus], 1, gpus, False, True))
    assert _same_bits(got, want)


def test_two_level_degenerate_shapes_equal_flat():
    rng = np.random.default_rng(11)
    srcs = [rng.normal(0, 1, 100).astype(np.float32) for _ in range(6)]
    flat = oracle.flat_reduce(srcs)
    assert _same_bits(oracle.two_level_reduce(srcs, 1, 6), flat)
    assert _same_bits(oracle.two_level_reduce(srcs, 6, 1), flat)
    bits = [_torch_bf16_bits(s) for s in srcs]
    flatb = oracle.flat_reduce(bits)
    assert _same_bits(oracle.two_level_reduce(bits, 1, 6), flatb)
    assert _same_bits(oracle.two_level_reduce(bits, 6, 1), flatb)
    # but a genuinely two-level shape differs from flat somewhere (the order is not ignored)
    assert not _same_bits(oracle.two_level_reduce(srcs, 3, 2), flat) or \
        not _same_bits(oracle.two_level_reduce(srcs, 2, 3), flat)


def test_two_level_integer_inputs_any_order():
    rng = np.random.default_rng(5)
    nodes, gpus, count = 4, 3, 50
    ints = [rng.integers(-8, 9, count) for _ in range(nodes * gpus)]
    want = np.sum(np.stack(ints), axis=0).astype(np.float32)
    srcs = [i.astype(np.float32) for i in ints]
    assert _same_bits(oracle.two_level_reduce(srcs, nodes, gpus), want)
    bits = [_torch_bf16_bits(s) for s in srcs]
    assert _same_bits(oracle.bf16_to_f32(oracle.two_level_reduce(bits, nodes, gpus)), want)


def test_phases_compose_to_two_level():
    """reduce_scatter_local on x[g][n][c] == two-level sum with source (n,g) = x[g][n]."""
    rng = np.random.default_rng(21)
    gpus, nodes, chunk = 3, 4, 37
    x32 = rng.uniform(-1, 1, (gpus, nodes, chunk)).astype(np.float32)
    for as_bf16 in (False, True):
        x = _torch_bf16_bits(x32.reshape(-1)).reshape(x32.shape) if as_bf16 else x32
        shard, partial = oracle.reduce_scatter_local(x)
        srcs = [x[g][n] for n in range(nodes) for g in range(gpus)]
        want, want_parts = oracle.two_level_reduce(srcs, nodes, gpus, want_partials=True)
        assert _same_bits(shard, want)
        assert _same_bits(partial, want_parts)
        xs = oracle.bf16_to_f32(x) if as_bf16 else x
        brute = _brute_two_level([xs[g][n] for n in range(nodes) for g in range(gpus)], nodes, gpus,
                                 as_bf16, as_bf16)
        assert _same_bits(shard, brute)


def test_external_inter_chunks_replace_all_but_own_node():
    rng = np.random.default_rng(22)
    gpus, nodes, chunk, my = 2, 3, 10, 1
    x = rng.integers(-4, 5, (gpus, nodes, chunk)).astype(np.float32)
    inter = [rng.integers(-4, 5, chunk).astype(np.float32) for _ in range(nodes)]
    shard, partial = oracle.reduce_scatter_local(x, my_node=my, inter=inter)
    want = x[:, my, :].sum(axis=0) + inter[0] + inter[2]
    assert _same_bits(shard, want.astype(np.float32))
    assert _same_bits(partial, x.sum(axis=0).astype(np.float32))


# ----------------------------------------------------------------------------- permutations
def test_worked_example_n2_m3(golden_dir):
    rows = {}
    for line in _read_cases(os.path.join(golden_dir, "hier_slots_n2_m3.txt")):
        k, v = line.split(":")
        rows[k.strip()] = np.array(v.split(), dtype=np.float32)
    assert _same_bits(oracle.hier_unpack(rows["hierarchical"], 2, 3), rows["rank_order"])
    assert _same_bits(oracle.hier_pack(rows["rank_order"], 2, 3), rows["hierarchical"])


def _literal_hier_gather(X, nodes, gpus):
    """Steps 1 and 2 of Section IV-A as plain list copies, no index formula."""
    step1 = {}
    for g in range(gpus):  # one inter-node group per local id
        members = [(n, g) for n in range(nodes)]
        gathered = [X[n * gpus + g] for (n, g) in members]
        for m in members:
            step1[m] = list(gathered)
    step2 = {}
    for n in range(nodes):  # one intra-node group per node
        members = [(n, g) for g in range(gpus)]
        gathered = []
        for m in members:
            gathered.extend(step1[m])
        for m in members:
            step2[m] = list(gathered)
    return step2


@pytest.mark.parametrize("nodes,gpus,chunk", [(2, 3, 1), (4, 8, 5), (3, 2, 16), (1, 4, 3), (5, 1, 2), (7, 5, 3)])
def test_unpack_against_literal_gather(nodes, gpus, chunk):
    P = nodes * gpus
    rng = np.random.default_rng(P)
    X = [rng.integers(0, 1 << 16, chunk).astype(np.uint16) for _ in range(P)]
    want = np.concatenate(X)  # definition of all-gather: rank-order concatenation
    step2 = _literal_hier_gather(X, nodes, gpus)
    for key, chunks in step2.items():
        H = np.concatenate(chunks)
        assert _same_bits(oracle.hier_unpack(H, nodes, gpus), want), key
        assert _same_bits(oracle.allgather_reassemble(chunks, nodes, gpus), want), key
        assert _same_bits(oracle.hier_pack(want, nodes, gpus), H), key


@pytest.mark.parametrize("nodes,gpus,chunk_bytes", [(4, 8, 6), (16, 8, 2), (3, 5, 1), (256, 8, 4)])
def test_permutation_invariants(nodes, gpus, chunk_bytes):
    P = nodes * gpus
    rng = np.random.default_rng(P + chunk_bytes)
    src = rng.integers(0, 256, P * chunk_bytes).astype(np.uint8)
    # numpy transpose is the textbook special case
    want_unpack = src.reshape(gpus, nodes, chunk_bytes).transpose(1, 0, 2).reshape(-1)
    want_pack = src.reshape(nodes, gpus, chunk_bytes).transpose(1, 0, 2).reshape(-1)
    assert _same_bits(oracle.hier_unpack(src, nodes, gpus), want_unpack)
    assert _same_bits(oracle.hier_pack(src, nodes, gpus), want_pack)
    # round trips
    assert _same_bits(oracle.hier_pack(oracle.hier_unpack(src, nodes, gpus), nodes, gpus), src)
    assert _same_bits(oracle.hier_unpack(oracle.hier_pack(src, nodes, gpus), nodes, gpus), src)
    # rank stamps: every chunk lands exactly once, in rank order
    stamps = np.repeat(np.array([n * gpus + g for g in range(gpus) for n in range(nodes)],
                                dtype=np.uint16), 3)
    out = oracle.hier_unpack(stamps, nodes, gpus)
    assert np.array_equal(out, np.repeat(np.arange(P, dtype=np.uint16), 3))


def test_degenerate_permutations_are_identity():
    src = np.arange(40, dtype=np.float32)
    assert _same_bits(oracle.hier_unpack(src, 1, 8), src)
    assert _same_bits(oracle.hier_unpack(src, 8, 1), src)
    assert _same_bits(oracle.hier_pack(src, 1, 5), src)
    assert _same_bits(oracle.hier_pack(src, 5, 1), src)


# ----------------------------------------------------------------------------- whole world
@pytest.mark.parametrize("nodes,gpus", [(2, 3), (4, 2), (3, 4)])
def test_world_allgather_is_concatenation(nodes, gpus):
    P = nodes * gpus
    rng = np.random.default_rng(P)
    X = [rng.normal(0, 1, 5).astype(np.float32) for _ in range(P)]
    want = np.concatenate(X)
    for out in world.hier_allgather(X, nodes, gpus):
        assert _same_bits(out, want)
    for out in world.hier_allgather_slots(X, nodes, gpus):
        assert _same_bits(out, want)


@pytest.mark.parametrize("nodes,gpus", [(2, 3), (4, 2), (3, 4)])
def test_world_reduce_scatter_definition(nodes, gpus):
    P, chunk = nodes * gpus, 6
    rng = np.random.default_rng(P + 1)
    # integer data: the definition (sum over ranks of chunk d) holds in every order
    Y = [rng.integers(-8, 9, (P, chunk)).astype(np.float32) for _ in range(P)]
    shards, _ = world.hier_reduce_scatter(Y, nodes, gpus)
    total = np.sum(np.stack(Y), axis=0)
    for d in range(P):
        assert _same_bits(shards[d], total[d].astype(np.float32)), d
    # real data: brute force in the two-level order, source (n', g') = rank n'*gpus + g'
    Y = [rng.normal(0, 1, (P, chunk)).astype(np.float32) for _ in range(P)]
    shards, _ = world.hier_reduce_scatter(Y, nodes, gpus)
    for d in range(P):
        srcs = [Y[n2 * gpus + g2][d] for n2 in range(nodes) for g2 in range(gpus)]
        assert _same_bits(shards[d], _brute_two_level(srcs, nodes, gpus, False, False)), d


@pytest.mark.parametrize("nodes,gpus", [(2, 2), (2, 4)])
def test_world_allreduce_is_reduce_scatter_then_allgather(nodes, gpus):
    P, chunk = nodes * gpus, 4
    rng = np.random.default_rng(P + 2)
    Y = [rng.integers(-8, 9, (P, chunk)).astype(np.float32) for _ in range(P)]
    want = np.sum(np.stack(Y), axis=0).astype(np.float32).reshape(-1)
    for out in world.hier_allreduce(Y, nodes, gpus):
        assert _same_bits(out, want)
    # bf16 world, integer data
    Yb = [_torch_bf16_bits(y.reshape(-1)).reshape(P, chunk) for y in Y]
    for out in world.hier_allreduce(Yb, nodes, gpus):
        assert _same_bits(oracle.bf16_to_f32(out), want)


@pytest.mark.parametrize("nodes,gpus", [(2, 3), (4, 2)])
def test_unpacked_share_equals_the_world(nodes, gpus):
    """Reading the node-mates' rank-order messages directly gives every rank the partial and the
    shard of the whole-world two-level reduce-scatter (which pre-shuffles every message)."""
    P, chunk = nodes * gpus, 5
    rng = np.random.default_rng(77 + P)
    Y = [rng.standard_normal((P, chunk)).astype(np.float32) for _ in range(P)]
    shards, partial = world.hier_reduce_scatter(Y, nodes, gpus)
    for n in range(nodes):
        for g in range(gpus):
            msgs = [Y[n * gpus + g2].reshape(-1) for g2 in range(gpus)]
            inter = [partial[n2 * gpus + g][n] for n2 in range(nodes)]
            shard, part = oracle.reduce_scatter_local_unpacked(msgs, nodes, gpus, g, my_node=n, inter=inter)
            assert _same_bits(part, partial[n * gpus + g])
            assert _same_bits(shard, shards[n * gpus + g])
    # integers: the shard is the plain sum over all ranks of the chunk bound for this rank
    Yi = [rng.integers(-30, 31, (P, chunk)).astype(np.float32) for _ in range(P)]
    shards, partial = world.hier_reduce_scatter(Yi, nodes, gpus)
    total = np.sum(np.stack(Yi), axis=0).astype(np.float32)
    n, g = nodes - 1, gpus - 1
    shard, _ = oracle.reduce_scatter_local_unpacked(
        [Yi[n * gpus + g2].reshape(-1) for g2 in range(gpus)], nodes, gpus, g, my_node=n,
        inter=[partial[n2 * gpus + g][n] for n2 in range(nodes)])
    assert _same_bits(shard, total[n * gpus + g])


@pytest.mark.parametrize("nodes,gpus", [(2, 3), (4, 2), (1, 4), (3, 1)])
def test_phase2_reassemble_equals_the_world(nodes, gpus):
    """The all-reduce tail (inter-node phase, then the all-gather shuffle with the rank's own shard
    in its own slot) gives every rank exactly the buffer the whole-world two-level all-reduce of
    Section IV-A gives it -- reals in the fixed order, and on integers the plain sum of all messages."""
    P, chunk = nodes * gpus, 7
    rng = np.random.default_rng(91 + P)
    for kind in ("real", "int", "bf16"):
        if kind == "real":
            Y = [rng.standard_normal((P, chunk)).astype(np.float32) for _ in range(P)]
        else:
            Y = [rng.integers(-20, 21, (P, chunk)).astype(np.float32) for _ in range(P)]
        if kind == "bf16":
            Y = [_torch_bf16_bits(y.reshape(-1)).reshape(P, chunk) for y in Y]
        shards, partial = world.hier_reduce_scatter(Y, nodes, gpus)
        final = world.hier_allreduce(Y, nodes, gpus)
        for n in range(nodes):
            for g in range(gpus):
                inter = [partial[n2 * gpus + g][n] for n2 in range(nodes)]
                # what the all-gather delivered: every OTHER rank's shard; the own slot holds junk
                slots = [shards[n2 * gpus + g2] for g2 in range(gpus) for n2 in range(nodes)]
                slots[g * nodes + n] = np.full_like(shards[0], 77)
                out = oracle.phase2_reassemble(inter, slots, nodes, gpus, n, g)
                assert _same_bits(out, final[n * gpus + g]), (kind, n, g)
                if kind == "int":
                    want = np.sum(np.stack(Y), axis=0).astype(np.float32).reshape(-1)
                    assert _same_bits(out, want)
                # rank stamp: chunk (n', g') of the result is rank (n', g')'s shard, the own one included
                for r in range(P):
                    assert _same_bits(out.reshape(P, chunk)[r], shards[r])


def test_phase2_reassemble_average_and_ignored_slot():
    """op = average divides the rank's own shard only (the gathered chunks arrive finished), and the
    entry at the rank's own slot is never read (None is accepted)."""
    nodes, gpus, chunk = 2, 2, 3
    inter = [np.array([1, 2, 3], np.float32), np.array([3, 2, 1], np.float32)]
    slots = [np.full(chunk, 10 * k, np.float32) for k in range(4)]
    slots[1 * nodes + 0] = None                                  # rank (node 0, gpu 1): slot g*N + n = 2
    out = oracle.phase2_reassemble(inter, slots, nodes, gpus, 0, 1, divisor=4).reshape(4, chunk)
    assert out[0 * gpus + 1].tolist() == [1.0, 1.0, 1.0]          # (1+3)/4, (2+2)/4, (3+1)/4
    assert out[0].tolist() == [0.0] * 3 and out[2].tolist() == [10.0] * 3 and out[3].tolist() == [30.0] * 3
