"""MI355X-native local kernels of PCCL's hierarchical collectives (HIP, gfx950).

The product is libpccl_local.so (csrc/, C ABI in include/pccl_local.h); this package is
its thin ctypes binding plus the seeded workload generators.  Nothing is loaded at import.
"""
from .binding import (  # noqa: F401
    PCCL_ALGO_REC, PCCL_ALGO_RING, PCCL_AVG, PCCL_BF16, PCCL_ERR_ADDRESS, PCCL_ERR_HIP, PCCL_ERR_INVALID, PCCL_ERR_NULL,
    PCCL_ERR_OVERLAP, PCCL_ERR_SCRATCH, PCCL_ERR_UNSUPPORTED, PCCL_F16, PCCL_F32, PCCL_MAX_BUCKETS, PCCL_OK, PCCL_STATIC_SCRATCH_BYTES, PCCL_SUM,
    AccumulateTable, BucketTable, PcclError, PermuteTable, device_pointer_array, diag_reload_env, lib, pccl_accumulate, pccl_accumulate_batched, pccl_accumulate_pair_t, pccl_allgather_reassemble,
    pccl_allgather_reassemble_batched, pccl_hier_pack_batched, pccl_permute_bucket_t,
    pccl_bucket_t, pccl_check_device_range, pccl_choose_algorithm, pccl_halving_reduce_scatter_local, pccl_hier_pack,
    pccl_hier_unpack, pccl_link_model_t, pccl_local_reduce, pccl_local_reduce_ptrs,
    pccl_local_reduce_ptrs_two_level, pccl_phase2_reassemble_local, pccl_reduce_scatter_local, pccl_reduce_scatter_local_batched, pccl_reduce_scatter_local_static,
    pccl_reduce_scatter_local_unpacked, pccl_reduce_scatter_local_unpacked_batched,
    pccl_ring_reduce_scatter_local, status_string,
)
