"""Whole-world CPU simulation of the paper's two-level collectives (test infrastructure).

Plays all P = nodes*gpus ranks in one address space, taking the steps of
Section IV-A ("Hierarchical Collective Algorithms") in the paper's order and
using the oracle's local operations for the on-GPU work.  Message passing is
simulated by handing arrays from one rank's state to another's.

Rank numbering: rank r = n*gpus + g (node n, local id g).
"""
import numpy as np

from . import allgather_reassemble, hier_pack, hier_unpack, rs_phase1, rs_phase2


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
