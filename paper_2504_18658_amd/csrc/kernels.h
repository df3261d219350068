// Host-side view of the gfx950 kernels: parameter blocks and launchers.
// The C ABI (pccl_api.hip) validates arguments and calls these; nothing here allocates.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/pccl_local.h"

namespace pccl {

// One two-level (or flat) reduction problem.  Source (n, g), n < nodes, g < gpus, is
//   ptrs != nullptr : ptrs[n*gpus + g]   (slot override_index reads override_ptr instead)
//   else            : base + n*stride_n + g*stride_g
// and holds `count` elements.  For every element e:
//   t_n = x[n][0][e] + ... + x[n][gpus-1][e];  p_n = round_partial ? through in_dt : t_n
//   partial[n*count + e] = p_n (if partial != nullptr, in in_dt);  dst[e] = p_0 + ... + p_{nodes-1},
//   divided by `divisor` (one IEEE division) when divisor != 0: op = average
// `rows` > 1 repeats the problem for rows r = 0 .. rows-1 (the streaming kernel's grid.y):
// row r reads every source at +r*row_stride_src bytes and writes dst at +r*row_stride_dst
// bytes (partial must be nullptr then).  src_offset is added to pointer-array entries.
struct ReduceProblem {
  void* dst;
  void* partial;
  const char* base;
  const void* const* ptrs;
  const void* override_ptr;
  size_t stride_n;
  size_t stride_g;
  size_t count;
  size_t src_offset;
  size_t row_stride_src;
  size_t row_stride_dst;
  int nodes;
  int gpus;
  int override_index;  // -1: none
  int round_partial;
  int rows;
  int row_pad;  // rows > 1: one more tile per row, so that a row's tile grid can be shifted onto cache lines
  int keep_cached;  // streaming kernel: store dst non-temporally instead of through (the batched phase 1, whose output phase 2 reads at once)
  float divisor;
};

// Chunk-granular transpose: dst chunk (c*rows + r) = src chunk (r*cols + c); src chunk k is
// slots[k] when slots != nullptr, else src + k*chunk_bytes.
struct PermuteProblem {
  char* dst;
  const char* src;
  const void* const* slots;
  size_t chunk_bytes;
  int rows;
  int cols;
};

// Launch shape of the kernel that runs a flat sum and a chunk transpose in one grid (blockIdx =
// (tile, source row, plane)): the first reduce_planes planes hold LDS-staged reduction slices
// (linear index over z, y, x; reduce_tiles of them do work; 0 planes for up to 16 sources), the
// others copy tiles of source chunk (blockIdx.y, blockIdx.z - reduce_planes) -- except in chunk
// (own_r, own_c), whose blocks compute its destination instead (tiles below reduce_tiles, when
// there are no planes).
struct FusedShape {
  uint32_t tiles_per_chunk;
  uint32_t skew;
  uint32_t reduce_planes;
  uint32_t reduce_tiles;
  int own_r;
  int own_c;
};

// One two-level reduce-scatter share with received inter-node chunks, for the one-launch form:
// pieces g at intra_base + g*intra_stride, each [nodes][chunk_count] of the message dtype;
// partial [nodes][chunk_count]; inter[n] for n != my_node from the device pointer array.
// own_src (the rows form only): source 0's chunk of the own node, the other sources intra_stride
// apart; in the contiguous form it is intra_base + my_node * chunk bytes.
struct ShareProblem {
  void* shard;
  void* partial;
  const char* intra_base;
  const char* own_src;
  const void* const* d_inter;
  size_t intra_stride;
  size_t chunk_count;
  int nodes;
  int gpus;
  int my_node;
  float divisor;
};

constexpr int kMaxBuckets = PCCL_MAX_BUCKETS;

// Prefix of tiles over the buckets of a batch, passed by value to the batched kernels.
struct BatchTiles {
  uint32_t first_tile[kMaxBuckets + 1];
};

// in_dt / out_dt are pccl_dtype_t values; unsupported pairs return hipErrorInvalidValue.
hipError_t launch_reduce(const ReduceProblem& p, int in_dt, int out_dt, hipStream_t st);
hipError_t launch_reduce_two_level_lds(const ReduceProblem& p, int in_dt, int out_dt,
                                       hipStream_t st);
// Both phases of a share in ONE launch (a per-node source count with an unrolled body; the blocks
// of the own row add the received chunks kShareFusedMaxNodes at a time): hipErrorNotSupported when
// the shape has no such form, or (unless any_shape) is one where a launch per phase measured faster
// (the caller then launches phase by phase), other errors as above.
constexpr int kShareFusedMaxNodes = 16;
hipError_t launch_share_fused(const ShareProblem& s, int dt, bool any_shape, hipStream_t st);
// The same for a share read straight from rank-order messages: `rows` is the phase-1 problem as
// launch_reduce takes it (rows = nodes, strided sources only; s.own_src = row my_node's source 0).
hipError_t launch_share_rows_fused(const ShareProblem& s, const ReduceProblem& rows, int dt, bool any_shape,
                                   hipStream_t st);
// True when the LDS-staged kernel is the better choice for this shape.
bool prefer_lds_two_level(const ReduceProblem& p, int in_dt);
// True when a flat sum of many short sources (p.gpus == 1, p.nodes sources) is better sent through
// the two-level LDS kernel than through the flat LDS kernel.
bool prefer_two_level_for_flat(const ReduceProblem& p, int in_dt);
// A flat sum written as p.nodes sources (p.gpus == 1, one row, no partial kept) through the
// LDS-staged flat kernel: every load of an element slice in flight at once.
hipError_t launch_reduce_flat_lds(const ReduceProblem& p, int in_dt, int out_dt, hipStream_t st);
// True when that kernel is the better choice for a flat sum of p.nodes sources.
bool prefer_flat_lds(const ReduceProblem& p, int in_dt);

// nbuckets chunk transposes (dst chunk c*rows + r = src chunk r*cols + c in every bucket) in
// one launch; h_buckets is the host copy used to size the grid.
hipError_t launch_permute_batched(const pccl_permute_bucket_t* d_buckets,
                                  const pccl_permute_bucket_t* h_buckets, int nbuckets, int rows, int cols,
                                  hipStream_t st);

// x and z extents for `blocks` thread blocks of `threads` threads each, keeping blocks*threads
// of the x dimension below 2^32 work-items (kernels index with linear_block_xz()).  False when
// even 65535 z-slices do not hold them.  PCCL_GRID_X_LIMIT (work-items, for tests) lowers the
// x limit so that small problems exercise the split.
bool split_grid_xz(size_t blocks, unsigned threads, unsigned* gx, unsigned* gz);

hipError_t launch_permute(const PermuteProblem& p, hipStream_t st);

// One launch for a flat sum (p: one node of p.gpus sources of dtype dt, result into p.dst, no
// partial kept, one row) and the chunk transpose q without its source chunk (own_r, own_c);
// p.dst is expected to be that chunk's place in q.dst.
hipError_t launch_phase2_reassemble(const ReduceProblem& p, const PermuteProblem& q, int own_r, int own_c, int dt,
                                    hipStream_t st);

// acc[e] = round_io(acc[e] + recv[e]) for e < count, in place (the two ranges are disjoint).
hipError_t launch_accumulate(void* acc, const void* recv, size_t count, int dt, hipStream_t st);

// Every step of one rank's ring / recursive-halving reduce-scatter in one launch (the layouts
// of pccl_ring_reduce_scatter_local / pccl_halving_reduce_scatter_local): hipErrorInvalidValue
// when the steps (ring) or half the ranks (halving) exceed 65535, the caller then launches step
// by step.
hipError_t launch_ring_steps(void* msg, const void* recv_base, size_t recv_stride, size_t count, int nranks, int rank,
                             int dt, hipStream_t st);
hipError_t launch_halving_steps(void* msg, const void* recv, size_t count, int nranks, int rank, int dt,
                                hipStream_t st);
// npairs independent acc += recv steps in one launch; h_pairs is the host copy used to size the grid.
hipError_t launch_accumulate_batched(const pccl_accumulate_pair_t* d_pairs, const pccl_accumulate_pair_t* h_pairs,
                                     int npairs, int dt, hipStream_t st);

// Batched two-level reduce-scatter share; h_buckets is the host copy used to size the grid.
// Phase 2 divides by `divisor` when it is not 0 (op = average).  my_gpu < 0: a bucket's
// intra_base holds pre-shuffled pieces; my_gpu >= 0: it holds `gpus` rank-order messages
// intra_stride_bytes apart and phase 1 reads chunk (n, my_gpu) of each.
hipError_t launch_rs_batched(const pccl_bucket_t* d_buckets, const pccl_bucket_t* h_buckets,
                             int nbuckets, int nodes, int gpus, int dt, float divisor,
                             hipStream_t st, int my_gpu = -1);

}  // namespace pccl
