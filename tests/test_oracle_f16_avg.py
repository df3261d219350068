"""Pins for the oracle's fp16 conversions and op = average: hand-worked cases, numpy's own
float16 casts and float32 division (library routines that coincide with one step), exact
rational arithmetic, pure-Python brute force."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle


def _parse_float(tok):
    return float.fromhex(tok) if "0x" in tok.lower() else float(tok)


def _read_cases(path):
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line


def _same_bits(a, b):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    return a.dtype == b.dtype and a.shape == b.shape and a.tobytes() == b.tobytes()


# ----------------------------------------------------------------------------- fp16 rounding
def test_f16_rne_hand_cases(golden_dir):
    n = 0
    for line in _read_cases(os.path.join(golden_dir, "f16_rne_cases.txt")):
        f32_hex, f16_hex = line.split()[:2]
        got = oracle.lib().pccl_oracle_f32_to_f16(int(f32_hex, 16))
        assert got == int(f16_hex, 16), (line, hex(got))
        n += 1
    assert n >= 25


def _check_block(start, base, cast):
    u = base + np.uint32(start)
    x = u.view(np.float32)
    got = oracle.f32_to_f16(x).view(np.uint16)
    want = cast(x)
    if start >> 23 & 0xFF != 0xFF:
        assert np.array_equal(got, want), hex(start)
        return
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    assert np.array_equal(got[~nan], want[~nan]), hex(start)
    g = got[nan]
    assert np.all((g & 0x7FFF) > 0x7C00), "NaN must stay NaN"
    assert np.array_equal(g >> 15, (u[nan] >> 31).astype(np.uint16)), "NaN keeps its sign"


def test_f16_rne_exhaustive_against_torch_cast():
    """All 2^32 binary32 patterns against torch's CPU float32 -> float16 cast; NaNs by NaN-ness and sign."""
    step = 1 << 22
    base = np.arange(step, dtype=np.uint32)
    cast = lambda x: torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    for start in range(0, 1 << 32, step):
        _check_block(start, base, cast)


def test_f16_rne_against_numpy_cast_over_the_half_range():
    """numpy's float32 -> float16 cast (slow outside the half range, so: every block that holds
    values a half can represent or that sit next to its limits, both signs, plus a few far ones)."""
    step = 1 << 22
    base = np.arange(step, dtype=np.uint32)
    cast = lambda x: x.astype(np.float16).view(np.uint16)
    lo, hi = 0x32000000, 0x48000000          # 2^-27 .. 2^17 covers 2^-25 (rounds to 0) .. 65520 (rounds to inf)
    starts = list(range(lo, hi, step)) + [s | 0x80000000 for s in range(lo, hi, step * 8)]
    starts += [0, 0x7F800000 - step, 0x7FC00000, 0xFF800000 - step]
    with np.errstate(over="ignore", under="ignore", invalid="ignore"):
        for start in starts:
            _check_block(start, base, cast)


def test_f16_widening_is_exact():
    bits = np.arange(1 << 16, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = oracle.f16_to_f32(bits)
    nan = np.isnan(want)
    assert _same_bits(got[~nan].view(np.uint32), want[~nan].view(np.uint32))
    assert np.all(np.isnan(got[nan]))
    # every finite half survives the round trip
    back = oracle.f32_to_f16(got[~nan]).view(np.uint16)
    assert np.array_equal(back, bits[~nan])


def test_f16_rounding_is_nearest_by_exact_arithmetic():
    """For sampled inputs the result is a nearest half (exact rationals), ties go to the even one."""
    rng = np.random.default_rng(5)
    xs = np.concatenate([rng.standard_normal(400).astype(np.float32) * np.float32(s)
                         for s in (1e-7, 1e-4, 1.0, 300.0, 6e4)])
    halves = np.arange(0x7C00, dtype=np.uint16).view(np.float16)          # all non-negative finite halves
    hv = [Fraction(float(h)) for h in halves]
    for x in xs:
        got = oracle.f32_to_f16(np.array([x]))[0]
        fx = abs(Fraction(float(x)))
        if fx >= Fraction(65520):
            assert np.isinf(got)
            continue
        i = int(np.searchsorted(halves.astype(np.float64), float(fx)))
        cands = [k for k in (i - 1, i, i + 1) if 0 <= k < len(hv)]
        best = min(abs(hv[k] - fx) for k in cands)
        g = abs(Fraction(float(got)))
        assert abs(g - fx) == best, (x, got)
        ties = [k for k in cands if abs(hv[k] - fx) == best]
        if len(ties) == 2:
            assert int(np.float16(abs(got)).view(np.uint16)) % 2 == 0, (x, got)


# ----------------------------------------------------------------------------- fp16 reductions
def _brute_two_level_f16(srcs, nodes, gpus, out_f16):
    count = len(srcs[0])
    out = np.empty(count, dtype=np.float32)
    for e in range(count):
        acc = None
        for n in range(nodes):
            t = np.float32(srcs[n * gpus][e])
            for g in range(1, gpus):
                t = np.float32(t + np.float32(srcs[n * gpus + g][e]))
            t = np.float32(np.float16(t))                      # the partial travels as fp16
            acc = t if acc is None else np.float32(acc + t)
        out[e] = acc
    with np.errstate(over="ignore"):
        return out.astype(np.float16) if out_f16 else out


@pytest.mark.parametrize("nodes,gpus,count", [(1, 1, 5), (1, 7, 33), (3, 4, 17), (5, 2, 64)])
@pytest.mark.parametrize("out_f16", [True, False])
def test_f16_reductions_brute_force(nodes, gpus, count, out_f16):
    rng = np.random.default_rng(nodes * 100 + gpus)
    srcs = [(rng.standard_normal(count) * 4).astype(np.float16) for _ in range(nodes * gpus)]
    out_dt = oracle.F16 if out_f16 else oracle.F32
    got = oracle.two_level_reduce(srcs, nodes, gpus, out_dt)
    assert _same_bits(got, _brute_two_level_f16(srcs, nodes, gpus, out_f16))
    if nodes == 1 and out_f16:
        assert _same_bits(oracle.flat_reduce(srcs, out_dt), got)
    # phases compose the same way as for bf16
    x = np.stack([np.stack([srcs[n * gpus + g] for n in range(nodes)]) for g in range(gpus)])
    shard, partial = oracle.reduce_scatter_local(x, out_dt=out_dt)
    assert _same_bits(shard, got)


def test_f16_accumulate_equals_numpy_half_add():
    rng = np.random.default_rng(3)
    a = rng.standard_normal(4000).astype(np.float16)
    r = (rng.standard_normal(4000) * 100).astype(np.float16)
    want = (a.astype(np.float32) + r.astype(np.float32)).astype(np.float16)
    assert _same_bits(oracle.accumulate(a, r), want)
    assert _same_bits(oracle.accumulate(a, r), np.add(a, r))       # numpy's half add: same definition


def test_f16_overflow_and_subnormal_sums():
    big = np.array([60000.0], dtype=np.float16)
    assert np.isinf(oracle.flat_reduce([big, big])[0])                        # 120000 > 65504 -> inf
    assert oracle.flat_reduce([big, big], oracle.F32)[0] == np.float32(120000.0)
    tiny = np.array([2.0 ** -24], dtype=np.float16)
    assert oracle.flat_reduce([tiny, tiny])[0] == np.float16(2.0 ** -23)       # subnormals add exactly


# ----------------------------------------------------------------------------- average
def test_average_hand_cases(golden_dir):
    n = 0
    for line in _read_cases(os.path.join(golden_dir, "avg_cases.txt")):
        shape, terms, expected = [p.strip() for p in line.split("|")]
        nodes, gpus = map(int, shape.split())
        vals = [np.array([_parse_float(t)], dtype=np.float32) for t in terms.split()]
        assert len(vals) == nodes * gpus, line
        want = np.array([_parse_float(expected)], dtype=np.float32)
        got = oracle.two_level_reduce(vals, nodes, gpus, average=True)
        assert _same_bits(got, want), (line, got)
        if nodes == 1:
            assert _same_bits(oracle.flat_reduce(vals, average=True), want), line
        n += 1
    assert n >= 12


def _nearest_f32(fr):
    """The binary32 nearest to the rational fr (ties to even), by exact comparison of neighbours."""
    c = np.float32(float(fr))          # float(fr) is correctly rounded to binary64; c is a close guess
    cands = {c, np.nextafter(c, np.float32(np.inf)), np.nextafter(c, np.float32(-np.inf))}
    best = min(abs(Fraction(float(k)) - fr) for k in cands)
    win = [k for k in cands if abs(Fraction(float(k)) - fr) == best]
    if len(win) == 1:
        return win[0]
    return [k for k in win if int(np.float32(k).view(np.uint32)) % 2 == 0][0]


@pytest.mark.parametrize("S", [2, 3, 7, 8, 24])
def test_average_is_one_exact_division_of_the_sum(S):
    rng = np.random.default_rng(40 + S)
    srcs = [rng.standard_normal(300).astype(np.float32) for _ in range(S)]
    s = oracle.flat_reduce(srcs)
    got = oracle.flat_reduce(srcs, average=True)
    assert _same_bits(got, np.divide(s, np.float32(S)))                        # numpy's binary32 division
    for e in range(0, 300, 7):
        assert got[e] == _nearest_f32(Fraction(float(s[e])) / S), e              # exact rationals
    # power-of-two counts only change the exponent
    if S & (S - 1) == 0:
        assert _same_bits(got, s * np.float32(1.0 / S))


def test_average_in_two_level_shapes_and_output_rounding():
    rng = np.random.default_rng(8)
    nodes, gpus, count = 3, 4, 50
    srcs32 = [rng.standard_normal(count).astype(np.float32) for _ in range(nodes * gpus)]
    s = oracle.two_level_reduce(srcs32, nodes, gpus)
    assert _same_bits(oracle.two_level_reduce(srcs32, nodes, gpus, average=True), np.divide(s, np.float32(12)))
    # bf16 messages: partials stay plain (rounded) sums; the division happens once, in fp32, before
    # the output rounding
    srcs = [oracle.f32_to_bf16(x) for x in srcs32]
    out, partials = oracle.two_level_reduce(srcs, nodes, gpus, want_partials=True, average=True)
    out_sum, partials_sum = oracle.two_level_reduce(srcs, nodes, gpus, want_partials=True)
    assert _same_bits(partials, partials_sum)
    s32 = oracle.two_level_reduce(srcs, nodes, gpus, out_dt=oracle.F32)
    assert _same_bits(out, oracle.f32_to_bf16(np.divide(s32, np.float32(12))))
    # the reduce-scatter share divides by the full rank count in phase 2
    x = np.stack([np.stack([srcs[n * gpus + g] for n in range(nodes)]) for g in range(gpus)])
    shard, partial = oracle.reduce_scatter_local(x, average=True)
    assert _same_bits(shard, out) and _same_bits(partial, partials)
    # integers: the plain definition of the mean
    ints = [rng.integers(-40, 41, count).astype(np.float32) for _ in range(nodes * gpus)]
    mean = np.sum(np.stack(ints), axis=0).astype(np.float32) / np.float32(12)
    assert _same_bits(oracle.two_level_reduce(ints, nodes, gpus, average=True), mean)
