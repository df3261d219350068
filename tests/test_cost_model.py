"""The closed-form cost model (host arithmetic): the oracle against the paper's two equations
evaluated by hand, closed forms and limits; the library against the oracle."""
import ctypes
import math

import pytest

import paper_2504_18658_amd as pccl
from oracle import cost_model as cm

# double arithmetic on both sides, at most a handful of operations that may be ordered
# differently: a few ulps
RTOL = 1e-14


def _lib():
    return pccl.lib()


# ----------------------------------------------------------------------------- oracle pins
def test_oracle_hand_values():
    # p = 8, m = 64 MiB, alpha = 10 us, beta = 1/(25 GB/s) = 4e-11 s/B
    m = 64 * 2 ** 20
    # ring: 7 * 1e-5 + 4e-11 * (7/8) * 67108864 = 7e-5 + 2.34881024e-3
    assert cm.t_ring(8, m, 1e-5, 4e-11) == pytest.approx(2.41881024e-3, rel=1e-12)
    # recursive: 3 * 1e-5 + the same bandwidth term
    assert cm.t_rec(8, m, 1e-5, 4e-11) == pytest.approx(2.37881024e-3, rel=1e-12)
    # one process: nothing to send
    assert cm.t_ring(1, m, 1e-5, 4e-11) == 0.0 and cm.t_rec(1, m, 1e-5, 4e-11) == 0.0


def test_oracle_closed_forms_and_limits():
    a, b = 3e-6, 2e-11
    for p in (2, 4, 64, 2048):
        for m in (0.0, 1e6, 1e9):
            # same bandwidth term, latency terms p-1 and log2 p
            assert cm.t_ring(p, m, a, b) - cm.t_rec(p, m, a, b) == pytest.approx(a * (p - 1 - math.log2(p)), rel=1e-9, abs=1e-18)
    assert cm.t_ring(2, 5e7, a, b) == cm.t_rec(2, 5e7, a, b)            # log2 2 = 2 - 1
    assert cm.t_ring(256, 0.0, a, b) / cm.t_rec(256, 0.0, a, b) == pytest.approx(255 / 8)
    assert cm.t_ring(256, 1e15, a, b) / cm.t_rec(256, 1e15, a, b) == pytest.approx(1.0, rel=1e-6)
    assert cm.t_rec(6, 1e6, a, b) == math.inf and cm.t_rec(12, 1e6, a, b) == math.inf
    # with one shared (alpha, beta) the recursive algorithm never loses
    for p in (2, 8, 128):
        assert cm.choose(p, 1e8, a, b, a, b)[0] == (cm.RING if p == 2 else cm.REC)
    # with its own, larger effective beta it loses beyond m* = alpha*(p-1-log2 p) / ((b2-b)*(p-1)/p)
    p, b2 = 16, 2.5e-11
    m_star = a * (p - 1 - 4) / ((b2 - b) * (p - 1) / p)
    assert cm.choose(p, 0.9 * m_star, a, b, a, b2)[0] == cm.REC
    assert cm.choose(p, 1.1 * m_star, a, b, a, b2)[0] == cm.RING
    assert cm.choose(6, 1e3, a, b, a, b)[0] == cm.RING                 # not a power of two


def test_oracle_two_level_hand_values(golden_dir):
    import os
    n = 0
    for line in open(os.path.join(golden_dir, "two_level_cost_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        args, want = line.split("|")
        nodes, gpus, m, algo, ai, bi, aa, ba, local, rate = args.split()
        got = cm.t_two_level(int(nodes), int(gpus), float(m), cm.RING if algo == "ring" else cm.REC, float(ai),
                             float(bi), float(aa), float(ba), float(local), float(rate))
        assert got == pytest.approx(float(want), rel=1e-12), line
        n += 1
    assert n == 4


def test_oracle_two_level_is_the_sum_of_its_parts():
    n, g, m = 16, 8, 256 * 2 ** 20
    t = cm.t_two_level(n, g, m, cm.REC, 1e-5, 4e-11, 2e-6, 1e-11, 1.4e9, 6.4e12)
    assert t == pytest.approx(cm.t_rec(n, m / g, 1e-5, 4e-11) + cm.t_ring(g, m, 2e-6, 1e-11) + 1.4e9 / 6.4e12)
    # a single node has no inter-node phase
    assert cm.t_two_level(1, 8, m, cm.RING, 1e-5, 4e-11, 2e-6, 1e-11, 0.0, 1.0) == cm.t_ring(8, m, 2e-6, 1e-11)


# ----------------------------------------------------------------------------- library vs oracle
@pytest.mark.parametrize("p", [1, 2, 3, 8, 12, 256, 2048])
@pytest.mark.parametrize("m", [0.0, 1.0, 16 * 2 ** 20, 2.0 ** 30])
def test_library_matches_oracle(p, m):
    L = _lib()
    for a, b in ((1e-5, 4e-11), (0.0, 1e-10), (2.5e-6, 0.0)):
        assert L.pccl_model_ring(p, m, a, b) == pytest.approx(cm.t_ring(p, m, a, b), rel=RTOL, abs=0.0)
        want = cm.t_rec(p, m, a, b)
        got = L.pccl_model_rec(p, m, a, b)
        assert got == want if math.isinf(want) else got == pytest.approx(want, rel=RTOL, abs=0.0)
        algo, tr, tc = pccl.pccl_choose_algorithm(p, m, a, b, 1.5 * a, 1.25 * b)
        walgo, wr, wc = cm.choose(p, m, a, b, 1.5 * a, 1.25 * b)
        assert algo == walgo and tr == pytest.approx(wr, rel=RTOL) and (tc == wc or tc == pytest.approx(wc, rel=RTOL))
    for algo in (cm.RING, cm.REC):
        got = L.pccl_model_two_level(p, 8, m, algo, 1e-5, 4e-11, 2e-6, 1e-11, 3e8, 6.4e12)
        want = cm.t_two_level(p, 8, m, algo, 1e-5, 4e-11, 2e-6, 1e-11, 3e8, 6.4e12)
        assert got == want if math.isinf(want) else got == pytest.approx(want, rel=RTOL)


def test_library_rejects_bad_arguments():
    L = _lib()
    nan = float("nan")
    for f in (L.pccl_model_ring, L.pccl_model_rec):
        assert math.isnan(f(0, 1e6, 1e-5, 1e-10))
        assert math.isnan(f(4, -1.0, 1e-5, 1e-10))
        assert math.isnan(f(4, 1e6, -1e-5, 1e-10))
        assert math.isnan(f(4, 1e6, 1e-5, nan))
        assert math.isnan(f(4, float("inf"), 1e-5, 1e-10))
    model = pccl.pccl_link_model_t(1e-5, 4e-11, 1e-5, 4e-11)
    algo = ctypes.c_int(-1)
    assert L.pccl_choose_algorithm(8, 1e6, None, ctypes.byref(algo), None, None) == pccl.PCCL_ERR_NULL
    assert L.pccl_choose_algorithm(8, 1e6, ctypes.byref(model), None, None, None) == pccl.PCCL_ERR_NULL
    assert L.pccl_choose_algorithm(0, 1e6, ctypes.byref(model), ctypes.byref(algo), None, None) == pccl.PCCL_ERR_INVALID
    assert L.pccl_choose_algorithm(8, 1e6, ctypes.byref(model), ctypes.byref(algo), None, None) == pccl.PCCL_OK
    assert algo.value == pccl.PCCL_ALGO_REC
    assert math.isnan(L.pccl_model_two_level(0, 8, 1e6, 0, 1e-5, 1e-10, 1e-6, 1e-11, 0.0, 1e12))
    assert math.isnan(L.pccl_model_two_level(4, 8, 1e6, 7, 1e-5, 1e-10, 1e-6, 1e-11, 0.0, 1e12))
    assert math.isnan(L.pccl_model_two_level(4, 8, 1e6, 0, 1e-5, 1e-10, 1e-6, 1e-11, 0.0, 0.0))
