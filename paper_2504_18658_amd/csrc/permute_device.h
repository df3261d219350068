// Device-side body of the chunk shuffle for gfx950 (one wavefront copies one 1 KB tile), shared
// by the shuffle kernels (permute_kernels.hip) and by the kernel that runs the shuffle next to
// the inter-node phase of the reduction (fused_kernels.hip).
#pragma once
#include "device_utils.h"
#include "kernels.h"

namespace pccl {

namespace {

constexpr int kPermBlock = 64;                        // one wavefront
constexpr size_t kPermTile = (size_t)kPermBlock * 16;  // bytes per block
// Chunk (r, c) starts (r + c) * kSkewTiles tiles into itself when chunks are a multiple of
// kSkewRound (the rotation undoes a resonance between chunks a round number of bytes apart;
// with chunk sizes that are multiples of 16 bytes only -- the 40-bucket batch -- it costs 5 %)
// and of a size where it was measured to pay: from 512 KB up (1-7 %), and at 64 KB-128 KB
// (the 2048 x 64 KB reassembly: 46.1 -> 43.0 us), not at 128-256 KB and not below 64 KB
// (up to 18 % slower).  How strong the resonance is depends on the physical placement the
// process got, so these are averages over runs from two different host programs.
constexpr uint32_t kSkewTiles = 131;
constexpr size_t kSkewRound = (size_t)64 << 10;
inline bool skew_pays(size_t chunk_bytes) {
  if (chunk_bytes % kSkewRound != 0) return false;
  return chunk_bytes >= ((size_t)512 << 10) || chunk_bytes < ((size_t)128 << 10);
}

// A 16-byte vector at an address that is only 4-byte aligned.
typedef u32x4 u32x4_align4 __attribute__((aligned(4)));

// `len` <= kPermTile bytes by one wavefront.  Both sides 16-byte aligned: a 128-bit load and
// store per lane.  Otherwise the stores are still 128-bit and 16-byte aligned (after a head of
// fewer than 16 single bytes), and the source is read as 4-byte-aligned 128-bit vectors and
// put right in registers: with the source `r` bytes past a 32-bit boundary, output word k is
// bytes r.. of (word k, word k+1), and a lane's fifth word is the next lane's first (the last
// lane fetches it itself).  Every 32-bit word read holds at least one byte of the tile.
// Chunk sizes that are odd multiples of 1, 2, 4 or 8 bytes (an odd number of 16-bit elements
// per rank-chunk, say) put nearly every tile on this path.  Measured, 256 MB as 16 x 8 chunks
// of 2 MB + 1 / 2 / 4 / 8 bytes: 5.4 / 6.0 / 6.2 / 6.2 TB/s, where copies in single bytes
// and 32-bit words (what the narrowest common alignment allows) reached 1.9 / 2.5 / 4.9 / 5.5.
__device__ __forceinline__ void copy_tile(const char* sp, char* dp, uint32_t len) {
  const uint32_t lane = threadIdx.x & 63;  // blocks of several wavefronts copy one tile per wavefront
  if (aligned_to(sp, 16) && aligned_to(dp, 16)) {
    const uint32_t lo = lane * 16;
    if (lo + 16 <= len) {
      const u32x4 v = ld_stream<u32x4>(sp + lo);
      const uint32_t w[4] = {v[0], v[1], v[2], v[3]};
      st_through<4>(wave_uniform(dp), lo, len, w);
    }
    const uint32_t b = (len & ~15u) + lane;  // fewer than 16 bytes can be left
    if (b < len) st_stream<uint8_t>(dp + b, ld_stream<uint8_t>(sp + b));
    return;
  }
  uint32_t head = (uint32_t)((16 - (reinterpret_cast<uintptr_t>(dp) & 15)) & 15);
  if (head > len) head = len;
  if (lane < head) st_stream<uint8_t>(dp + lane, ld_stream<uint8_t>(sp + lane));
  const uint32_t nvec = (len - head) >> 4;  // whole destination vectors, at most 64; wave-uniform
  if (nvec > 0) {
    const char* s = sp + head;
    const uint32_t r = (uint32_t)(reinterpret_cast<uintptr_t>(s) & 3);  // wave-uniform
    const char* sa = s - r;                                              // 4-byte aligned
    u32x4 v = {0u, 0u, 0u, 0u};
    if (lane < nvec) v = __builtin_nontemporal_load((const PCCL_GLOBAL u32x4_align4*)(sa + 16 * lane));
    if (r != 0) {
      uint32_t up = __shfl_down(v[0], 1);  // every lane takes part; lanes past nvec hold zeros
      if (lane == nvec - 1) up = ld_stream<uint32_t>(sa + 16 * nvec);
      v[0] = __builtin_amdgcn_alignbyte(v[1], v[0], r);
      v[1] = __builtin_amdgcn_alignbyte(v[2], v[1], r);
      v[2] = __builtin_amdgcn_alignbyte(v[3], v[2], r);
      v[3] = __builtin_amdgcn_alignbyte(up, v[3], r);
    }
    if (lane < nvec) {
      const uint32_t w[4] = {v[0], v[1], v[2], v[3]};
      st_through<4>(wave_uniform(dp + head), 16 * lane, 16 * nvec, w);
    }
  }
  const uint32_t b = head + 16 * nvec + lane;  // fewer than 16 bytes can be left
  if (b < len) st_stream<uint8_t>(dp + b, ld_stream<uint8_t>(sp + b));
}

// Tile `t` of one chunk (source sp0, destination dp0, chunk_bytes long).  Tiles are cut at
// kPermTile boundaries of the DESTINATION ADDRESS, not of the offset inside the chunk: a chunk
// whose size is not a multiple of the cache line would otherwise start every store of every
// later chunk in mid-line, and partial-line stores are what costs most (measured with 64 MB
// chunks: both sides aligned 6.65 TB/s, source 16 bytes off 6.27, destination 16 bytes off
// 5.68, chunk size = 16 mod 128 with tiles cut by offset 5.41).  Tile 0 is the short head up
// to the first boundary; a tile past the end of the chunk does nothing.
__device__ __forceinline__ void copy_chunk_tile(const char* sp0, char* dp0, size_t chunk_bytes, size_t t) {
  const size_t m = reinterpret_cast<uintptr_t>(dp0) & (kPermTile - 1);
  const size_t lo = t == 0 ? 0 : t * kPermTile - m;
  size_t hi = (t + 1) * kPermTile - m;
  if (hi > chunk_bytes) hi = chunk_bytes;
  if (lo < hi) copy_tile(sp0 + lo, dp0 + lo, (uint32_t)(hi - lo));
}

// Tiles a chunk of `chunk_bytes` can need when chunk k of a buffer starts at dst + k*chunk_bytes.
inline size_t tiles_per_chunk_for(const void* dst, size_t chunk_bytes) {
  if (chunk_bytes == 0) return 0;
  // every chunk has the misalignment of the buffer when the chunk size keeps it, else assume the worst
  const size_t m = chunk_bytes % kPermTile == 0 ? (reinterpret_cast<uintptr_t>(dst) & (kPermTile - 1))
                                                : kPermTile - 1;
  return (m + chunk_bytes + kPermTile - 1) / kPermTile;
}

// Largest launch: a grid dimension holds fewer than 2^32 work-items, so a chunk has at most
// 2^26 - 1 one-wavefront tiles (just under 64 GiB) in the 3-D form, and the whole message that
// many in the flat form (used only when a side of the chunk matrix exceeds 65535).
constexpr size_t kPermMaxTilesX = ((size_t)1 << 32) / kPermBlock - 1;

// Which chunk index the resident blocks sweep first.  Measured on MI355X for N x 8 and 8 x N
// chunk matrices of 32-256 MB (both orders within 0.3 % run to run): with chunks of 64-256 KB
// the order whose fast index is the SHORT side of the matrix is 2-10 % faster (the resident
// blocks then touch one contiguous span on one side and only `short side` spans on the
// other, instead of one span per chunk); below 64 KB the long side first is 4-5 % faster;
// from 512 KB up the two are within 2 % and the destination-contiguous order is kept.
__host__ __device__ inline bool column_fast_order(size_t chunk_bytes, int rows, int cols) {
  if (chunk_bytes >= ((size_t)512 << 10)) return false;
  if (chunk_bytes >= ((size_t)64 << 10)) return cols < rows;
  return cols > rows;
}

}  // namespace

}  // namespace pccl
