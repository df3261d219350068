"""Randomised property checks of the oracle (hypothesis): invariants that hold for any shape,
compared with numpy's own reshape/transpose/sum (library routines) or with exact integers."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from oracle import world

small = settings(max_examples=60, deadline=None)


def _same_bits(a, b):
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    return a.dtype == b.dtype and a.size == b.size and a.tobytes() == b.tobytes()


@small
@given(nodes=st.integers(1, 9), gpus=st.integers(1, 9), chunk=st.integers(0, 40), seed=st.integers(0, 2 ** 31))
def test_permutations_any_shape(nodes, gpus, chunk, seed):
    rng = np.random.default_rng(seed)
    msg = rng.integers(0, 256, nodes * gpus * chunk, dtype=np.uint8)
    packed = oracle.hier_pack(msg, nodes, gpus)
    assert _same_bits(packed, msg.reshape(nodes, gpus, chunk).transpose(1, 0, 2))        # numpy's transpose
    assert _same_bits(oracle.hier_unpack(packed, nodes, gpus), msg)                          # round trip
    assert _same_bits(oracle.hier_unpack(msg, nodes, gpus), msg.reshape(gpus, nodes, chunk).transpose(1, 0, 2))
    if chunk:
        slots = [packed.reshape(gpus * nodes, chunk)[k].copy() for k in range(gpus * nodes)]
        assert _same_bits(oracle.allgather_reassemble(slots, nodes, gpus), msg)
        # every source chunk lands exactly once: stamps 0..P-1 come out in rank order
        stamps = np.repeat(np.arange(nodes * gpus, dtype=np.uint8), chunk)
        hier = stamps.reshape(nodes, gpus, chunk).transpose(1, 0, 2).reshape(-1)
        assert _same_bits(oracle.hier_unpack(hier, nodes, gpus), stamps)


@small
@given(nodes=st.integers(1, 6), gpus=st.integers(1, 6), count=st.integers(1, 50), seed=st.integers(0, 2 ** 31),
       average=st.booleans())
def test_integer_sums_any_shape_any_dtype(nodes, gpus, count, seed, average):
    """Small integers are exact in fp32, bf16 and fp16 and in every summation order: the result
    is numpy's integer sum (divided by the rank count when averaging, a power of two or not)."""
    rng = np.random.default_rng(seed)
    S = nodes * gpus
    ints = rng.integers(-3, 4, (S, count))
    total = ints.sum(axis=0)
    want32 = (total.astype(np.float32) / np.float32(S)) if average else total.astype(np.float32)
    srcs32 = [ints[s].astype(np.float32) for s in range(S)]
    assert _same_bits(oracle.two_level_reduce(srcs32, nodes, gpus, average=average), want32)
    assert _same_bits(oracle.flat_reduce(srcs32, average=average), want32)
    srcs16 = [ints[s].astype(np.float16) for s in range(S)]
    assert _same_bits(oracle.two_level_reduce(srcs16, nodes, gpus, oracle.F32, average=average), want32)
    srcsb = [oracle.f32_to_bf16(x) for x in srcs32]
    assert _same_bits(oracle.two_level_reduce(srcsb, nodes, gpus, oracle.F32, average=average), want32)
    # the reduce-scatter share sees the same numbers through its two phases
    x = np.stack([np.stack([srcs32[n * gpus + g] for n in range(nodes)]) for g in range(gpus)])
    shard, partial = oracle.reduce_scatter_local(x, average=average)
    assert _same_bits(shard, want32)
    assert _same_bits(partial, ints.reshape(nodes, gpus, count).sum(axis=1).astype(np.float32))


@small
@given(S=st.integers(1, 12), count=st.integers(1, 40), seed=st.integers(0, 2 ** 31))
def test_fp32_flat_sum_is_the_accumulate_chain_and_within_the_error_bound(S, count, seed):
    rng = np.random.default_rng(seed)
    srcs = [rng.standard_normal(count).astype(np.float32) * np.float32(10.0 ** rng.integers(-3, 4)) for _ in range(S)]
    got = oracle.flat_reduce(srcs)
    acc = srcs[0]
    for s in range(1, S):
        acc = oracle.accumulate(acc, srcs[s])              # one step at a time: the same left-to-right chain
    assert _same_bits(got, acc)
    ref = np.sum(np.stack(srcs).astype(np.float64), axis=0)
    bound = (S - 1) * 2.0 ** -24 * np.sum(np.abs(np.stack(srcs).astype(np.float64)), axis=0) * 1.0001 + 1e-45
    assert np.all(np.abs(got.astype(np.float64) - ref) <= bound)


@small
@given(logp=st.integers(0, 4), chunk=st.integers(1, 6), seed=st.integers(0, 2 ** 31))
def test_step_algorithms_on_integers_any_power_of_two(logp, chunk, seed):
    p = 1 << logp
    rng = np.random.default_rng(seed)
    Y = [rng.integers(-9, 10, (p, chunk)).astype(np.float32) for _ in range(p)]
    total = np.sum(np.stack(Y), axis=0).astype(np.float32)
    for fn in (world.ring_reduce_scatter, world.recursive_halving_reduce_scatter):
        for r, shard in enumerate(fn(Y)):
            assert _same_bits(shard, total[r])
    for out in world.rec_allreduce(Y):
        assert _same_bits(out, total.reshape(-1))
