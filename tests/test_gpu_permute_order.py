"""The shuffle kernel sweeps the chunk matrix in one of two block orders (destination-
contiguous or source-contiguous), picked from the chunk size and the shape.  Either order is
the same permutation: every shape below is checked byte for byte against the oracle with the
order forced each way and with the library's own choice, on chunk sizes on both sides of the
thresholds of that choice."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_18658_amd as pccl
from util import same_bits, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda"
KB = 1 << 10

SHAPES = [(12, 3), (3, 12), (5, 5), (1, 7), (7, 1)]
CHUNKS = [1000, 48 * KB + 16, 64 * KB, 200 * KB + 2, 512 * KB, 640 * KB + 48]


@pytest.mark.parametrize("skew", [None, "0", "7", "131"])
@pytest.mark.parametrize("order", ["dst", "src", None])
@pytest.mark.parametrize("nodes,gpus", SHAPES)
def test_pack_unpack_reassemble_in_either_block_order(monkeypatch, order, skew, nodes, gpus):
    """`skew` rotates the tiles of chunk (r, c) by (r + c) * skew: None leaves the library's own
    choice (on from 512 KB chunks), a number forces it for every chunk size below."""
    if order is None:
        monkeypatch.delenv("PCCL_PERMUTE_ORDER", raising=False)
        pccl.diag_reload_env()
    else:
        monkeypatch.setenv("PCCL_PERMUTE_ORDER", order)
        pccl.diag_reload_env()
    if skew is None:
        monkeypatch.delenv("PCCL_PERMUTE_SKEW", raising=False)
        pccl.diag_reload_env()
    else:
        monkeypatch.setenv("PCCL_PERMUTE_SKEW", skew)
        pccl.diag_reload_env()
    gen = torch.Generator()
    gen.manual_seed(nodes * 100 + gpus)
    P = nodes * gpus
    for cb in CHUNKS:
        host = torch.randint(0, 256, (P * cb,), generator=gen, dtype=torch.uint8)
        src = host.to(DEV)
        packed, back, via = torch.empty_like(src), torch.empty_like(src), torch.empty_like(src)
        pccl.pccl_hier_pack(packed, src, nodes, gpus)
        pccl.pccl_hier_unpack(back, packed, nodes, gpus)
        slots = pccl.device_pointer_array([packed.view(P, cb)[k] for k in range(P)])
        pccl.pccl_allgather_reassemble(via, d_slots=slots, nodes=nodes, gpus_per_node=gpus)
        torch.cuda.synchronize()
        assert same_bits(to_np(packed), oracle.hier_pack(host.numpy(), nodes, gpus)), (cb, "pack")
        assert same_bits(to_np(back), oracle.hier_unpack(to_np(packed), nodes, gpus)), (cb, "unpack")
        assert torch.equal(back, src) and torch.equal(via, src), cb
