"""Oracle for the closed-form cost model (test infrastructure only, plain Python floats).

The paper models a ring collective over p processes on an m-byte buffer as
    T_ring = alpha*(p-1) + beta*((p-1)/p)*m            (Section II-B, Eq. 1)
and the recursive doubling / halving collective as
    T_rec  = alpha*log2(p) + beta*((p-1)/p)*m          (Section II-B, Eq. 2)
with alpha the start-up latency per message and beta the inverse point-to-point bandwidth.
The two-level design (Section IV-A) runs an intra-node ring over the M GPUs of a node on the
whole m-byte buffer and an inter-node collective over the N nodes on m/M bytes, plus the
device-local kernels (transposes, reductions) whose cost is bytes moved / HBM rate.
"""
import math

RING, REC = 0, 1


def t_ring(p, m, alpha, beta):
    return alpha * (p - 1) + beta * ((p - 1) / p) * m


def t_rec(p, m, alpha, beta):
    if p < 1 or p & (p - 1):
        return math.inf                      # recursive doubling / halving: powers of two only
    return alpha * math.log2(p) + beta * ((p - 1) / p) * m


def choose(p, m, alpha_ring, beta_ring, alpha_rec, beta_rec):
    """(algorithm, t_ring, t_rec): the cheaper one, the ring on a tie."""
    a, b = t_ring(p, m, alpha_ring, beta_ring), t_rec(p, m, alpha_rec, beta_rec)
    return (REC if b < a else RING), a, b


def t_two_level(nodes, gpus, m, algo, alpha_inter, beta_inter, alpha_intra, beta_intra, local_bytes, hbm_rate):
    inter = t_ring(nodes, m / gpus, alpha_inter, beta_inter) if algo == RING else \
        t_rec(nodes, m / gpus, alpha_inter, beta_inter)
    return inter + t_ring(gpus, m, alpha_intra, beta_intra) + local_bytes / hbm_rate
