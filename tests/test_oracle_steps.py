"""Pins for the oracle's step-wise reductions: the literal vector-reduction step
(acc += recv, Sections III-B / IV-B) and the ring / recursive-halving orders it is used in.
Each check compares with something other than the oracle: hand-worked IEEE cases, numpy and
torch adds (library routines that coincide with one step), the summation trees written out
as pure-Python formulas, the definition of the collectives on integer inputs."""
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import world


def _parse_float(tok):
    return float.fromhex(tok) if "0x" in tok.lower() else float(tok)


def _read_cases(path):
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line


def _torch_bf16_bits(x32):
    t = torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def _bf16_bits_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _same_bits(a, b):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    return a.dtype == b.dtype and a.shape == b.shape and a.tobytes() == b.tobytes()


def _rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------- one step
def test_accumulate_hand_cases(golden_dir):
    n = 0
    for line in _read_cases(os.path.join(golden_dir, "accumulate_cases.txt")):
        dt, a, r, want = [p.strip() for p in line.split("|")]
        a32 = np.array([_parse_float(a)], dtype=np.float32)
        r32 = np.array([_parse_float(r)], dtype=np.float32)
        w32 = np.array([_parse_float(want)], dtype=np.float32)
        if dt == "f32":
            got = oracle.accumulate(a32, r32)
            assert _same_bits(got, w32), (line, got)
        else:
            ab, rb, wb = _torch_bf16_bits(a32), _torch_bf16_bits(r32), _torch_bf16_bits(w32)
            for bits, v in ((ab, a32), (rb, r32), (wb, w32)):  # the operands are bf16 values
                assert _same_bits(_bf16_bits_to_f32(bits), v), line
            got = oracle.accumulate(ab, rb)
            assert _same_bits(got, wb), (line, got)
        n += 1
    assert n >= 15


def test_accumulate_equals_library_adds():
    rng = _rng(11)
    a = rng.standard_normal(5000).astype(np.float32)
    r = (rng.standard_normal(5000) * 1e-3).astype(np.float32)
    assert _same_bits(oracle.accumulate(a, r), np.add(a, r))          # one binary32 add
    ab, rb = _torch_bf16_bits(a), _torch_bf16_bits(r)
    ta = torch.from_numpy(ab.view(np.int16)).view(torch.bfloat16)
    tr = torch.from_numpy(rb.view(np.int16)).view(torch.bfloat16)
    want = (ta + tr).view(torch.int16).numpy().view(np.uint16)           # torch's bf16 add
    assert _same_bits(oracle.accumulate(ab, rb), want)
    # the inputs are untouched and an empty buffer is fine
    assert _same_bits(a, a.copy())
    assert oracle.accumulate(a[:0], r[:0]).size == 0


def test_accumulate_is_two_source_flat_reduce_and_commutes():
    rng = _rng(12)
    a = rng.uniform(-1, 1, 777).astype(np.float32)
    r = rng.uniform(-1, 1, 777).astype(np.float32)
    assert _same_bits(oracle.accumulate(a, r), oracle.flat_reduce([a, r]))
    assert _same_bits(oracle.accumulate(a, r), oracle.accumulate(r, a))
    ab, rb = _torch_bf16_bits(a), _torch_bf16_bits(r)
    assert _same_bits(oracle.accumulate(ab, rb), oracle.flat_reduce([ab, rb]))


# ----------------------------------------------------------------------------- schedules
@pytest.mark.parametrize("p", [2, 3, 4, 7, 8, 16])
def test_ring_schedule_visits_every_other_chunk_once_and_ends_at_own(p):
    for rank in range(p):
        seq = [oracle.ring_chunk_at_step(p, rank, s) for s in range(p - 1)]
        assert sorted(seq) == sorted(set(range(p)) - {(rank - 1) % p})
        assert seq[-1] == rank


@pytest.mark.parametrize("p", [1, 2, 4, 8, 32, 256])
def test_halving_schedule_nests_and_ends_at_own(p):
    steps = p.bit_length() - 1
    for rank in range(0, p, max(1, p // 16)):
        lo, ln = 0, p
        for t in range(steps):
            lo2, ln2 = oracle.halving_kept_range(p, rank, t)
            assert ln2 * 2 == ln and lo2 in (lo, lo + ln2) and lo2 <= rank < lo2 + ln2
            # the partner keeps the other half of the same range
            plo, pln = oracle.halving_kept_range(p, rank ^ (p >> (t + 1)), t)
            assert pln == ln2 and {plo, lo2} == {lo, lo + ln2}
            lo, ln = lo2, ln2
        assert (lo, ln) == (rank, 1)
    with pytest.raises(ValueError):
        oracle.halving_kept_range(6, 0, 0)


# ----------------------------------------------------------------------------- orders
def _one_element_world(p, chunk, xs):
    Y = []
    for r in range(p):
        y = np.zeros((p, 1), dtype=np.float32)
        y[chunk, 0] = np.float32(xs[r])
        Y.append(y)
    return Y


def test_step_order_cases_by_hand(golden_dir):
    seen = set()
    for line in _read_cases(os.path.join(golden_dir, "step_order_cases.txt")):
        head, terms, expected = [p.strip() for p in line.split("|")]
        order, p, chunk = head.split()
        p, chunk = int(p), int(chunk)
        xs = [_parse_float(t) for t in terms.split()]
        assert len(xs) == p, line
        want = np.array([_parse_float(expected)], dtype=np.float32)
        if order == "flat":
            got = oracle.flat_reduce([np.array([x], dtype=np.float32) for x in xs])
        elif order == "ring":
            got = world.ring_reduce_scatter(_one_element_world(p, chunk, xs))[chunk]
        else:
            got = world.recursive_halving_reduce_scatter(_one_element_world(p, chunk, xs))[chunk]
        assert _same_bits(got, want), (line, got)
        seen.add(order)
    assert seen == {"flat", "ring", "halving"}


def _ring_formula(vals, c, bf16):
    """((x[c+1] + x[c+2]) + ...) + x[c], each partial stored in the message dtype."""
    p = len(vals)
    acc = np.float32(vals[(c + 1) % p])
    for k in range(2, p + 1):
        acc = np.float32(acc + np.float32(vals[(c + k) % p]))
        if bf16:
            acc = _bf16_bits_to_f32(_torch_bf16_bits(np.array([acc])))[0]
    return acc


def _halving_formula(vals, c, bf16):
    """f0(i) = x[i]; f_{t+1}(i) = f_t(i) + f_t(i xor dist_t), dist = p/2, p/4, ..., 1; owner c."""
    p = len(vals)
    f = [np.float32(v) for v in vals]
    dist = p // 2
    while dist >= 1:
        g = list(f)
        for i in range(p):
            s = np.float32(f[i] + f[i ^ dist])
            if bf16:
                s = _bf16_bits_to_f32(_torch_bf16_bits(np.array([s])))[0]
            g[i] = s
        f = g
        dist //= 2
    return f[c]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("p", [2, 3, 5, 8])
def test_ring_world_follows_the_ring_formula(p, bf16):
    rng = _rng(100 + p)
    chunk = 6
    Y32 = [rng.standard_normal((p, chunk)).astype(np.float32) for _ in range(p)]
    Y = [_torch_bf16_bits(y.reshape(-1)).reshape(p, chunk) for y in Y32] if bf16 else Y32
    vals = [_bf16_bits_to_f32(y) for y in Y] if bf16 else Y32
    shards = world.ring_reduce_scatter(Y)
    for c in range(p):
        want = np.array([_ring_formula([vals[r][c, e] for r in range(p)], c, bf16) for e in range(chunk)],
                        dtype=np.float32)
        got = _bf16_bits_to_f32(shards[c]) if bf16 else shards[c]
        assert _same_bits(got, want), (c, got, want)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("p", [1, 2, 4, 8, 16])
def test_halving_world_follows_the_tree_formula(p, bf16):
    rng = _rng(200 + p)
    chunk = 5
    Y32 = [rng.standard_normal((p, chunk)).astype(np.float32) for _ in range(p)]
    Y = [_torch_bf16_bits(y.reshape(-1)).reshape(p, chunk) for y in Y32] if bf16 else Y32
    vals = [_bf16_bits_to_f32(y) for y in Y] if bf16 else Y32
    shards = world.recursive_halving_reduce_scatter(Y)
    for c in range(p):
        want = np.array([_halving_formula([vals[r][c, e] for r in range(p)], c, bf16)
                         for e in range(chunk)], dtype=np.float32)
        got = _bf16_bits_to_f32(shards[c]) if bf16 else shards[c]
        assert _same_bits(got, want), (c, got, want)


# ----------------------------------------------------------------------------- definitions
@pytest.mark.parametrize("p", [2, 4, 8])
def test_step_algorithms_meet_the_definitions_on_integers(p):
    """Integers are exact in every order: reduce-scatter = per-chunk sum over ranks,
    all-gather = concatenation, all-reduce = the full sum on every rank."""
    rng = _rng(300 + p)
    chunk = 4
    Y = [rng.integers(-50, 51, (p, chunk)).astype(np.float32) for _ in range(p)]
    total = np.sum(np.stack(Y), axis=0, dtype=np.float64).astype(np.float32)
    for fn in (world.ring_reduce_scatter, world.recursive_halving_reduce_scatter):
        shards = fn(Y)
        for r in range(p):
            assert _same_bits(shards[r], total[r])
    X = [rng.integers(0, 1000, 7).astype(np.float32) for _ in range(p)]
    for fn in (world.ring_allgather, world.recursive_doubling_allgather):
        for out in fn(X):
            assert _same_bits(out, np.concatenate(X))
    for fn in (world.ring_allreduce, world.rec_allreduce):
        for out in fn(Y):
            assert _same_bits(out, total.reshape(-1))


def test_ring_works_for_any_rank_count_and_halving_rejects_non_powers_of_two():
    rng = _rng(7)
    Y = [rng.integers(-9, 10, (6, 3)).astype(np.float32) for _ in range(6)]
    total = np.sum(np.stack(Y), axis=0)
    for r, s in enumerate(world.ring_reduce_scatter(Y)):
        assert _same_bits(s, total[r].astype(np.float32))
    with pytest.raises(ValueError):
        world.recursive_halving_reduce_scatter(Y)


# ----------------------------------------------------------------------------- one rank's share
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("p", [2, 5, 8])
def test_ring_local_replay_equals_the_world(p, bf16):
    rng = _rng(400 + p)
    chunk = 9
    Y = [rng.standard_normal((p, chunk)).astype(np.float32) for _ in range(p)]
    if bf16:
        Y = [_torch_bf16_bits(y.reshape(-1)).reshape(p, chunk) for y in Y]
    received = [[] for _ in range(p)]
    shards = world.ring_reduce_scatter(Y, received)
    for r in range(p):
        buf = oracle.ring_rs_local(Y[r], received[r], r)
        assert _same_bits(buf[r], shards[r])
        # the one chunk this rank never receives (it forwards it first) stays as it was
        assert _same_bits(buf[(r - 1) % p], Y[r][(r - 1) % p])


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("p", [1, 2, 8, 16])
def test_halving_local_replay_equals_the_world(p, bf16):
    rng = _rng(500 + p)
    chunk = 7
    Y = [rng.standard_normal((p, chunk)).astype(np.float32) for _ in range(p)]
    if bf16:
        Y = [_torch_bf16_bits(y.reshape(-1)).reshape(p, chunk) for y in Y]
    received = [[] for _ in range(p)]
    shards = world.recursive_halving_reduce_scatter(Y, received)
    for r in range(p):
        buf = oracle.halving_rs_local(Y[r], received[r], r)
        assert _same_bits(buf[r], shards[r])


def test_two_level_with_ring_inter_node_phase_on_integers():
    """Hierarchical reduce-scatter with the paper's own inter-node algorithm: intra-node
    phase from the two-level world, inter-node phase by ring over each inter-node group."""
    nodes, gpus, chunk = 4, 2, 3
    P = nodes * gpus
    rng = _rng(9)
    Y = [rng.integers(-20, 21, (P, chunk)).astype(np.float32) for _ in range(P)]
    total = np.sum(np.stack(Y), axis=0)
    _, partial = world.hier_reduce_scatter(Y, nodes, gpus)
    for g in range(gpus):
        group = [partial[n * gpus + g] for n in range(nodes)]      # [nodes][chunk] each
        for fn in (world.ring_reduce_scatter, world.recursive_halving_reduce_scatter):
            shards = fn(group)
            for n in range(nodes):
                assert _same_bits(shards[n], total[n * gpus + g].astype(np.float32))
