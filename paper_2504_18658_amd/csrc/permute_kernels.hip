// Chunk-granular transpose for gfx950: the device-local shuffle between hierarchical order
// [gpu][node][chunk] and rank order [node][gpu][chunk] (Section IV-A, step 3 of the two-level
// all-gather, and its inverse ahead of the two-level reduce-scatter).
//
// Every chunk is contiguous on both sides, so the transpose is P independent streaming
// copies; nothing is staged in LDS.  A block copies one 4 KB tile of one chunk, one 128-bit
// load and store per lane: measured on MI355X, more bytes in flight per lane at full
// occupancy lowers the achieved HBM bandwidth.  HBM-bound: 2 bytes moved per byte.
#include "device_utils.h"
#include "kernels.h"

namespace pccl {

namespace {

constexpr int kPermU = 1;                                // 16-byte vectors per thread
constexpr size_t kPermTile = (size_t)kBlock * 16 * kPermU;  // bytes per block

__global__ __launch_bounds__(kBlock) void k_permute(PermuteProblem p, uint32_t tiles_per_chunk) {
  // blocks are numbered in destination order: chunk-major, then tile within the chunk
  const uint32_t chunk = blockIdx.x / tiles_per_chunk;
  const uint32_t tile = blockIdx.x - chunk * tiles_per_chunk;
  const uint32_t c = chunk / (uint32_t)p.rows;  // dst chunk = c*rows + r
  const uint32_t r = chunk - c * (uint32_t)p.rows;
  const size_t sidx = (size_t)r * p.cols + c;
  const char* sp = p.slots != nullptr ? ld_pointer_lane(p.slots, sidx)
                                      : p.src + sidx * p.chunk_bytes;
  char* dp = p.dst + (size_t)chunk * p.chunk_bytes;
  const size_t off = (size_t)tile * kPermTile;
  const size_t left = p.chunk_bytes - off;
  const size_t len = left < kPermTile ? left : kPermTile;
  sp += off;
  dp += off;

  if (aligned_to(sp, 16) && aligned_to(dp, 16)) {
    const size_t nv = len / 16;
    u32x4 v[kPermU];
#pragma unroll
    for (int u = 0; u < kPermU; ++u) {
      const size_t i = (size_t)u * kBlock + threadIdx.x;
      if (i < nv) v[u] = ld_stream<u32x4>(sp + i * 16);
    }
#pragma unroll
    for (int u = 0; u < kPermU; ++u) {
      const size_t i = (size_t)u * kBlock + threadIdx.x;
      if (i < nv) st_stream<u32x4>(dp + i * 16, v[u]);
    }
    const size_t b = nv * 16 + threadIdx.x;  // fewer than 16 bytes can be left
    if (b < len) st_stream<uint8_t>(dp + b, ld_stream<uint8_t>(sp + b));
  } else if (aligned_to(sp, 4) && aligned_to(dp, 4)) {
    const size_t nw = len / 4;
    for (size_t i = threadIdx.x; i < nw; i += kBlock)
      st_stream<uint32_t>(dp + i * 4, ld_stream<uint32_t>(sp + i * 4));
    const size_t b = nw * 4 + threadIdx.x;
    if (b < len) st_stream<uint8_t>(dp + b, ld_stream<uint8_t>(sp + b));
  } else {
    for (size_t i = threadIdx.x; i < len; i += kBlock)
      st_stream<uint8_t>(dp + i, ld_stream<uint8_t>(sp + i));
  }
}

}  // namespace

hipError_t launch_permute(const PermuteProblem& p, hipStream_t st) {
  const size_t tiles_per_chunk = (p.chunk_bytes + kPermTile - 1) / kPermTile;
  const size_t chunks = (size_t)p.rows * (size_t)p.cols;
  if (tiles_per_chunk == 0 || chunks == 0) return hipSuccess;
  if (tiles_per_chunk > 0x7FFFFFFFull || chunks > 0x7FFFFFFFull ||
      tiles_per_chunk * chunks > 0x7FFFFFFFull)
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_permute, dim3((unsigned)(tiles_per_chunk * chunks)), dim3(kBlock), 0, st, p,
                     (uint32_t)tiles_per_chunk);
  return hipGetLastError();
}

}  // namespace pccl
