"""Whole-world CPU simulation of the paper's two-level collectives (test infrastructure).

Plays all P = nodes*gpus ranks in one address space, taking the steps of
Section IV-A ("Hierarchical Collective Algorithms") in the paper's order and
using the oracle's local operations for the on-GPU work.  Message passing is
simulated by handing arrays from one rank's state to another's.

Rank numbering: rank r = n*gpus + g (node n, local id g).
"""
import numpy as np

from . import (accumulate, allgather_reassemble, halving_kept_range, hier_pack, hier_unpack,
               ring_chunk_at_step, rs_phase1, rs_phase2)


def hier_allgather(X, nodes, gpus):
    """X[r] = chunk owned by rank r.  Returns out[r] = rank r's final buffer.

    Step 1: all-gather inside every inter-node group (same local id g, ordered by node).
    Step 2: all-gather inside every node (ordered by local id) of the step-1 results.
    Step 3: device-local shuffle of the gathered buffer into rank order."""
    P = nodes * gpus
    assert len(X) == P
    after_inter = [None] * P
    for n in range(nodes):
        for g in range(gpus):
            after_inter[n * gpus + g] = np.concatenate([X[n2 * gpus + g] for n2 in range(nodes)])
    after_intra = [None] * P
    for n in range(nodes):
        for g in range(gpus):
            after_intra[n * gpus + g] = np.concatenate(
                [after_inter[n * gpus + g2] for g2 in range(gpus)])
    return [hier_unpack(after_intra[r], nodes, gpus) for r in range(P)]


def hier_allgather_slots(X, nodes, gpus):
    """As hier_allgather, but the gathered chunks stay separate allocations
    (slot g*nodes + n holds rank (n,g)'s chunk) and step 3 reads them by pointer."""
    slots = [X[n * gpus + g] for g in range(gpus) for n in range(nodes)]
    return [allgather_reassemble(slots, nodes, gpus) for _ in range(nodes * gpus)]


def hier_reduce_scatter(Y, nodes, gpus, out_dt=None):
    """Y[r] = rank r's message: P chunks in destination-rank order, shape [P][chunk].
    Returns (shards, partials): shards[r] = what rank r owns afterwards.

    Pre-shuffle every message so the chunks bound for one local id are contiguous,
    run the intra-node phase (each GPU sums what its node-mates hold for its local
    id), then the inter-node phase (each GPU sums what its counterparts on the
    other nodes hold for its node)."""
    P = nodes * gpus
    assert len(Y) == P
    chunk = Y[0].shape[1]
    packed = [hier_pack(Y[r], nodes, gpus).reshape(gpus, nodes, chunk) for r in range(P)]
    partial = [None] * P
    for n in range(nodes):
        for g in range(gpus):
            pieces = [packed[n * gpus + g2][g] for g2 in range(gpus)]
            partial[n * gpus + g] = rs_phase1(pieces, nodes, chunk)
    shards = [None] * P
    for n in range(nodes):
        for g in range(gpus):
            inter = [partial[n2 * gpus + g][n] for n2 in range(nodes)]
            shards[n * gpus + g] = rs_phase2(inter, out_dt)
    return shards, partial


def hier_allreduce(Y, nodes, gpus):
    """All-reduce = two-level reduce-scatter followed by two-level all-gather."""
    shards, _ = hier_reduce_scatter(Y, nodes, gpus)
    return hier_allgather(shards, nodes, gpus)


# ---- the inter-node algorithms of Section IV-B, played by all p ranks -------------------
# Every step first collects what each rank sends (a snapshot), then lets each rank receive
# and reduce, exactly as simultaneous point-to-point messages would.

def ring_reduce_scatter(Y, received=None):
    """PCCL_ring reduce-scatter (Sections II-B, IV-B).  Y[r]: rank r's message [p][chunk].
    If `received` is a list of p empty lists, received[r] collects what rank r got at each step.
    Every rank sends to rank+1 and receives from rank-1; p-1 steps; the received chunk is
    added into the local copy of the same chunk (the GPU vector reduction), which is what the
    next step sends.  Rank r ends up owning chunk r.  Returns shards[r]."""
    p = len(Y)
    buf = [np.array(y, copy=True) for y in Y]
    for s in range(p - 1):
        sent = []
        for i in range(p):
            c = (i - 1 - s) % p                      # the chunk rank i forwards at step s
            sent.append((c, buf[i][c].copy()))
        for i in range(p):
            c, data = sent[(i - 1) % p]
            assert c == ring_chunk_at_step(p, i, s)
            if received is not None:
                received[i].append(data)
            buf[i][c] = accumulate(buf[i][c], data)
    return [buf[i][i] for i in range(p)]


def recursive_halving_reduce_scatter(Y, received=None):
    """PCCL_rec reduce-scatter (Sections II-B, IV-B): log2 p steps; at each step a rank
    exchanges with the partner at half the previous distance, sends the half of its active
    range the partner's side owns, and adds the half it receives into the half it keeps."""
    p = len(Y)
    buf = [np.array(y, copy=True) for y in Y]
    steps = p.bit_length() - 1
    for t in range(steps):
        dist = p >> (t + 1)
        sent = []
        for i in range(p):
            lo, ln = halving_kept_range(p, i ^ dist, t)   # what the partner keeps is what i sends
            sent.append(buf[i][lo:lo + ln].copy())
        for i in range(p):
            lo, ln = halving_kept_range(p, i, t)
            if received is not None:
                received[i].append(sent[i ^ dist])
            buf[i][lo:lo + ln] = accumulate(buf[i][lo:lo + ln], sent[i ^ dist])
    return [buf[i][i] for i in range(p)]


def ring_allgather(X):
    """Ring all-gather: p-1 steps, rank i forwards to rank+1 the chunk it received last."""
    p = len(X)
    out = [[None] * p for _ in range(p)]
    for i in range(p):
        out[i][i] = X[i]
    for s in range(p - 1):
        sent = [((i - s) % p, out[i][(i - s) % p]) for i in range(p)]
        for i in range(p):
            c, data = sent[(i - 1) % p]
            out[i][c] = data
    return [np.concatenate(out[i]) for i in range(p)]


def recursive_doubling_allgather(X):
    """Recursive-doubling all-gather: log2 p steps, partner distance 1, 2, 4, ...; the two
    partners swap everything they hold so far."""
    p = len(X)
    if p & (p - 1):
        raise ValueError("recursive doubling needs a power-of-two rank count")
    held = [{i: X[i]} for i in range(p)]
    dist = 1
    while dist < p:
        sent = [dict(h) for h in held]
        for i in range(p):
            held[i].update(sent[i ^ dist])
        dist *= 2
    return [np.concatenate([held[i][c] for c in range(p)]) for i in range(p)]


def rec_allreduce(Y):
    """PCCL_rec all-reduce: recursive halving followed by recursive doubling (Section IV-B)."""
    return recursive_doubling_allgather(recursive_halving_reduce_scatter(Y))


def ring_allreduce(Y):
    """PCCL_ring all-reduce: ring reduce-scatter followed by ring all-gather."""
    return ring_allgather(ring_reduce_scatter(Y))
