// Chunk-granular transpose for gfx950: the device-local shuffle between hierarchical order
// [gpu][node][chunk] and rank order [node][gpu][chunk] (Section IV-A, step 3 of the two-level
// all-gather, and its inverse ahead of the two-level reduce-scatter).
//
// Every chunk is contiguous on both sides, so the transpose is P independent streaming
// copies; nothing is staged in LDS.  A block is ONE wavefront copying one 1 KB tile of one
// chunk with a single 128-bit load and store per lane, and the grid is three-dimensional
// (tile, source row, source column) so that no index division is needed: measured on MI355X
// this moves 6.7 TB/s, against 6.3 TB/s with 256-thread blocks and 5.2 TB/s with four
// vectors in flight per lane.  HBM-bound: 2 bytes moved per byte of message.
#include "device_utils.h"
#include "kernels.h"
#include "knobs.h"
#include "permute_device.h"

namespace pccl {

namespace {

// GRID3: blockIdx = (tile, r, c), or (tile, c, r) with CFAST; otherwise a flat grid,
// chunk-major in destination order.  Blocks start in x, y, z order, so without CFAST the
// resident blocks walk the destination contiguously and read from as many places as they span
// source rows; with CFAST they walk the source contiguously and write to `cols` places.
template <bool GRID3, bool CFAST>
__global__ __launch_bounds__(kPermBlock) void k_permute(PermuteProblem p, uint32_t tiles_per_chunk, uint32_t skew) {
  uint32_t tile, r, c;
  if (GRID3) {
    tile = blockIdx.x;
    r = CFAST ? blockIdx.z : blockIdx.y;
    c = CFAST ? blockIdx.y : blockIdx.z;
    if (skew) tile = (uint32_t)(((uint64_t)tile + (uint64_t)(r + c) * skew) % tiles_per_chunk);
  } else {
    const uint32_t chunk = blockIdx.x / tiles_per_chunk;  // dst chunk = c*rows + r
    tile = blockIdx.x - chunk * tiles_per_chunk;
    c = chunk / (uint32_t)p.rows;
    r = chunk - c * (uint32_t)p.rows;
  }
  const size_t sidx = (size_t)r * p.cols + c;
  const char* sp = p.slots != nullptr ? ld_pointer(p.slots, (int)sidx) : p.src + sidx * p.chunk_bytes;
  char* dp = p.dst + ((size_t)c * p.rows + r) * p.chunk_bytes;
  copy_chunk_tile(sp, dp, p.chunk_bytes, tile);
}

// Many independent chunk transposes (one per bucket, common rows x cols) in one launch: a flat
// tile space over all buckets, chunk-major inside a bucket; the tile prefix travels as a kernel
// argument and a block bisects it.
__global__ __launch_bounds__(kPermBlock) void k_permute_batched(
    const pccl_permute_bucket_t* __restrict__ buckets, BatchTiles tiles, int nbuckets, int rows, int cols) {
  const size_t block = linear_block_xz();
  if (block >= tiles.first_tile[nbuckets]) return;  // the x*z rectangle is rounded up
  int lo = 0, hi = nbuckets;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tiles.first_tile[mid] <= block)
      lo = mid;
    else
      hi = mid;
  }
  const pccl_permute_bucket_t b = buckets[lo];
  const uint32_t t = (uint32_t)(block - tiles.first_tile[lo]);
  // tiles in this bucket = chunks * tiles_per_chunk, so the latter follows from the prefix
  const uint32_t tiles_per_chunk = (tiles.first_tile[lo + 1] - tiles.first_tile[lo]) / (uint32_t)(rows * cols);
  // chunks in destination order (k = c*rows + r) or, by the rule above, in source order
  // (k = r*cols + c)
  const uint32_t k = t / tiles_per_chunk;
  const uint32_t tile = t - k * tiles_per_chunk;
  uint32_t r, c;
  if (column_fast_order(b.chunk_bytes, rows, cols)) {
    r = k / (uint32_t)cols;
    c = k - r * (uint32_t)cols;
  } else {
    c = k / (uint32_t)rows;
    r = k - c * (uint32_t)rows;
  }
  const char* sp = reinterpret_cast<const char*>(b.src) + ((size_t)r * cols + c) * b.chunk_bytes;
  char* dp = reinterpret_cast<char*>(b.dst) + ((size_t)c * rows + r) * b.chunk_bytes;
  copy_chunk_tile(sp, dp, b.chunk_bytes, tile);
}

}  // namespace

bool split_grid_xz(size_t blocks, unsigned threads, unsigned* gx, unsigned* gz) {
  size_t limit = (size_t)1 << 31;  // work-items in x; the hardware packet holds 32 bits
  const size_t t = knobs().grid_x_limit;  // tests lower it so that small problems take the split
  if (t >= threads && t < limit) limit = t;
  const size_t max_x = limit / threads;
  if (blocks <= max_x) {
    *gx = (unsigned)(blocks == 0 ? 1 : blocks);
    *gz = 1;
    return true;
  }
  const size_t z = (blocks + max_x - 1) / max_x;
  if (z > 65535) return false;
  *gx = (unsigned)max_x;
  *gz = (unsigned)z;
  return true;
}

hipError_t launch_permute(const PermuteProblem& p, hipStream_t st) {
  const size_t tiles_per_chunk = tiles_per_chunk_for(p.dst, p.chunk_bytes);
  const size_t chunks = (size_t)p.rows * (size_t)p.cols;
  if (tiles_per_chunk == 0 || chunks == 0) return hipSuccess;
  if (tiles_per_chunk > kPermMaxTilesX || chunks > 0x7FFFFFFFull) return hipErrorInvalidValue;
  if (p.rows <= 65535 && p.cols <= 65535) {
    bool cfast = column_fast_order(p.chunk_bytes, p.rows, p.cols);
    if (knobs().permute_order != 0) cfast = knobs().permute_order == 2;  // forced, for A/B runs
    // Chunk (r, c) starts (r + c) * skew tiles into itself, modulo its tile count: the resident
    // blocks otherwise sit at the same offset of several chunks a power of two apart.  Measured
    // with 131 tiles: 1-7 % faster for chunks of 512 KB-1 MB (256 MB as 64x8: 85.8 -> 79.5 us,
    // 128 MB as 32x8: 43.7 -> 40.9 us), no change from 2 MB up; see skew_pays() for the rest.
    uint32_t skew = skew_pays(p.chunk_bytes) ? kSkewTiles : 0u;
    if (knobs().permute_skew >= 0) skew = (uint32_t)knobs().permute_skew;
    if (cfast)
      hipLaunchKernelGGL((k_permute<true, true>), dim3((unsigned)tiles_per_chunk, (unsigned)p.cols, (unsigned)p.rows),
                         dim3(kPermBlock), 0, st, p, (uint32_t)tiles_per_chunk, skew);
    else
      hipLaunchKernelGGL((k_permute<true, false>), dim3((unsigned)tiles_per_chunk, (unsigned)p.rows, (unsigned)p.cols),
                         dim3(kPermBlock), 0, st, p, (uint32_t)tiles_per_chunk, skew);
  } else {
    if (tiles_per_chunk * chunks > kPermMaxTilesX) return hipErrorInvalidValue;
    hipLaunchKernelGGL((k_permute<false, false>), dim3((unsigned)(tiles_per_chunk * chunks)), dim3(kPermBlock), 0,
                       st, p, (uint32_t)tiles_per_chunk, 0u);
  }
  return hipGetLastError();
}

hipError_t launch_permute_batched(const pccl_permute_bucket_t* d_buckets,
                                  const pccl_permute_bucket_t* h_buckets, int nbuckets, int rows, int cols,
                                  hipStream_t st) {
  BatchTiles tiles;
  size_t total = 0;
  const size_t chunks = (size_t)rows * (size_t)cols;
  for (int b = 0; b < nbuckets; ++b) {
    tiles.first_tile[b] = (uint32_t)total;
    const size_t tpc = tiles_per_chunk_for(h_buckets[b].dst, h_buckets[b].chunk_bytes);
    if (tpc > 0xFFFFFFFFull / chunks) return hipErrorInvalidValue;
    total += tpc * chunks;
    if (total > 0xFFFFFFFFull) return hipErrorInvalidValue;  // the prefix holds 32-bit tile indices
  }
  for (int b = nbuckets; b <= kMaxBuckets; ++b) tiles.first_tile[b] = (uint32_t)total;
  if (total == 0) return hipSuccess;
  unsigned gx, gz;
  if (!split_grid_xz(total, kPermBlock, &gx, &gz)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_permute_batched, dim3(gx, 1, gz), dim3(kPermBlock), 0, st, d_buckets, tiles, nbuckets,
                     rows, cols);
  return hipGetLastError();
}

}  // namespace pccl
