// The paper's GPU vector-reduction kernel in its literal, step-wise form for gfx950
// (Section III-B: reduce-scatter from point-to-point messages plus a GPU vector reduction;
// Section IV-B: PCCL_ring and PCCL_rec run their local reduction on the GPU): the buffer a
// step has just received is added into the local data in place, and the sum -- stored in the
// message dtype -- is what the next step forwards.
//
// HBM-bound: two loads and one store per element, one add.  A thread owns one 128-bit vector
// of each operand (measured on MI355X for two sources: 16 bytes per lane and operand moves
// 6.3 TB/s, 4 bytes 4.3 TB/s -- with only two streams the lane needs the wide access to keep
// enough bytes in flight).
//
// Kernels:
//   k_accumulate          one step: acc += recv.
//   k_ring_steps          every step of one rank's ring reduce-scatter in one launch: step s
//                         adds into chunk (rank-2-s) mod p, so the p-1 steps touch p-1 DIFFERENT
//                         chunks and are independent of one another (grid.y = step).
//   k_halving_steps       every step of one rank's recursive-halving reduce-scatter in one
//                         launch: the kept ranges are nested, so a chunk that takes part in m
//                         steps is read once, takes its m additions in registers (each sum
//                         rounded through the message dtype, as the stored step result is)
//                         and is written once (grid.y = chunk of the first kept half).
//   k_accumulate_batched  many independent steps of different sizes in one launch.
#include "device_utils.h"
#include "kernels.h"

namespace pccl {

namespace {

constexpr int kW = 4;  // 32-bit words per lane and operand

template <int DT>
__device__ __forceinline__ void add_words(uint32_t* a, const uint32_t* r) {
#pragma unroll
  for (int k = 0; k < kW; ++k) {
    if (narrow(DT))
      a[k] = pack16<DT>(lo16<DT>(a[k]) + lo16<DT>(r[k]), hi16<DT>(a[k]) + hi16<DT>(r[k]));
    else
      a[k] = __float_as_uint(__uint_as_float(a[k]) + __uint_as_float(r[k]));
  }
}

// Block `block` of acc[e] = round_io(acc[e] + recv[e]), e < count: BLOCK vectors, and the
// ragged tail (fewer than 8 elements) with the last block that holds vectors.
template <int DT, bool FAST, int BLOCK>
__device__ __forceinline__ void accumulate_tile(char* acc, const char* recv, size_t count, size_t block) {
  constexpr int VE = narrow(DT) ? 2 * kW : kW;
  constexpr int ES = narrow(DT) ? 2 : 4;
  const size_t nvec = count / VE;
  const size_t v = block * BLOCK + threadIdx.x;
  if (v < nvec) {
    const size_t tile = block * BLOCK * (4 * kW);  // wave-uniform byte offset of the block's vectors
    const uint32_t lane_off = threadIdx.x * (4 * kW);
    uint32_t a[kW], r[kW];
    ld_words<kW, ES, FAST>(acc, tile + lane_off, a);
    ld_words<kW, ES, FAST>(recv, tile + lane_off, r);
    add_words<DT>(a, r);
    st_tile_words<kW, ES, FAST>(acc + tile, lane_off, a);
  }
  if (block == (nvec == 0 ? 0 : (nvec - 1) / BLOCK)) {
    const size_t e = nvec * VE + threadIdx.x;
    if (e < count) st_elem<DT>(acc, e, ld_elem<DT>(acc, e) + ld_elem<DT>(recv, e));
  }
}

template <int DT, bool FAST, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_accumulate(char* acc, const char* recv, size_t count) {
  accumulate_tile<DT, FAST, BLOCK>(acc, recv, count, linear_block_xz());
}

__host__ __device__ inline size_t blocks_for(size_t count, bool is_narrow, int block) {
  const size_t nvec = count / (is_narrow ? 2 * kW : kW);
  const size_t b = (nvec + block - 1) / block;
  return b == 0 ? 1 : b;  // a lone ragged tail still needs one block
}

// Rows (steps, chunks) are a round number of bytes apart, and the blocks resident at one time
// span several rows at the same offsets; as in the row form of the streaming reduce, every row
// starts its blocks this many further along (modulo the blocks of a row).
constexpr size_t kStepRowSkew = 131;

// Ring: row s = step s; what arrives at step s is chunk (rank - 2 - s) mod nranks.
template <int DT, bool FAST, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_ring_steps(char* msg, const char* recv_base, size_t recv_stride,
                                                      size_t count, int nranks, int rank) {
  constexpr size_t ES = narrow(DT) ? 2 : 4;
  const size_t nblocks = blocks_for(count, narrow(DT), BLOCK);
  size_t block = linear_block_xz();
  if (block >= nblocks) return;  // the x*z rectangle is rounded up
  const int s = (int)blockIdx.y;
  block = (block + (size_t)s * kStepRowSkew) % nblocks;
  const int c = ((rank - 2 - s) % nranks + nranks) % nranks;
  accumulate_tile<DT, FAST, BLOCK>(msg + (size_t)c * count * ES, recv_base + (size_t)s * recv_stride, count, block);
}

// Recursive halving over nranks = 2^levels ranks: row j = chunk j of the first kept half.  Step t
// keeps the chunks that share their top t+1 index bits with `rank`; chunk c therefore takes part
// in the first m steps, m = number of leading index bits it shares with rank.  Step t's received
// half starts (nranks - (nranks >> t)) chunks into recv and holds the kept range in order.
template <int DT, bool FAST, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_halving_steps(char* msg, const char* recv, size_t count, int levels,
                                                         int rank) {
  constexpr int VE = narrow(DT) ? 2 * kW : kW;
  constexpr size_t ES = narrow(DT) ? 2 : 4;
  const size_t nblocks = blocks_for(count, narrow(DT), BLOCK);
  size_t block = linear_block_xz();
  if (block >= nblocks) return;  // the x*z rectangle is rounded up
  const int nranks = 1 << levels;
  const int half = nranks >> 1;
  const int lo0 = rank & half;  // first chunk of the half that holds `rank`
  const int c = lo0 + (int)blockIdx.y;
  block = (block + (size_t)blockIdx.y * kStepRowSkew) % nblocks;
  const int diff = c ^ rank;                                   // < half
  const int m = diff == 0 ? levels : levels - (32 - __builtin_clz(diff));  // steps this chunk takes part in, >= 1
  const size_t chunk_bytes = count * ES;
  char* acc = msg + (size_t)c * chunk_bytes;
  // the chunk's place in step t's received half
  auto recv_chunk = [&](int t) -> const char* {
    const int shift = levels - 1 - t;
    const int lo_t = (rank >> shift) << shift;
    return recv + ((size_t)(nranks - (nranks >> t)) + (size_t)(c - lo_t)) * chunk_bytes;
  };
  const size_t nvec = count / VE;
  const size_t v = block * BLOCK + threadIdx.x;
  if (v < nvec) {
    const size_t tile = block * BLOCK * (4 * kW);
    const uint32_t lane_off = threadIdx.x * (4 * kW);
    uint32_t a[kW];
    ld_words<kW, ES, FAST>(acc, tile + lane_off, a);
    for (int t0 = 0; t0 < m; t0 += 4) {  // up to four received vectors in flight at a time (m is wave-uniform)
      uint32_t r[4][kW];
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (t0 + q < m) ld_words<kW, ES, FAST>(recv_chunk(t0 + q), tile + lane_off, r[q]);
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (t0 + q < m) add_words<DT>(a, r[q]);  // one step: the sum, stored in the message dtype
    }
    st_tile_words<kW, ES, FAST>(acc + tile, lane_off, a);
  }
  if (block == (nvec == 0 ? 0 : (nvec - 1) / BLOCK)) {
    const size_t e = nvec * VE + threadIdx.x;
    if (e < count) {
      float x = ld_elem<DT>(acc, e);
      for (int t = 0; t < m; ++t) x = round_through<DT>(x + ld_elem<DT>(recv_chunk(t), e));
      st_elem<DT>(acc, e, x);
    }
  }
}

// Many independent steps in one launch: a flat block space over the pairs (prefix as kernel
// argument, bisected per block).
template <int DT, bool FAST, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_accumulate_batched(const pccl_accumulate_pair_t* __restrict__ pairs,
                                                              BatchTiles tiles, int npairs) {
  const size_t block = linear_block_xz();
  if (block >= tiles.first_tile[npairs]) return;  // the x*z rectangle is rounded up
  int lo = 0, hi = npairs;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tiles.first_tile[mid] <= block)
      lo = mid;
    else
      hi = mid;
  }
  const pccl_accumulate_pair_t k = pairs[lo];
  accumulate_tile<DT, FAST, BLOCK>(reinterpret_cast<char*>(k.acc), reinterpret_cast<const char*>(k.recv), k.count,
                                   block - tiles.first_tile[lo]);
}

inline bool is16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <int DT, int BLOCK>
hipError_t launch_acc_b(char* acc, const char* recv, size_t count, hipStream_t st) {
  unsigned gx, gz;
  if (!split_grid_xz(blocks_for(count, narrow(DT), BLOCK), BLOCK, &gx, &gz)) return hipErrorInvalidValue;
  if (is16(acc) && is16(recv))
    hipLaunchKernelGGL((k_accumulate<DT, true, BLOCK>), dim3(gx, 1, gz), dim3(BLOCK), 0, st, acc, recv, count);
  else
    hipLaunchKernelGGL((k_accumulate<DT, false, BLOCK>), dim3(gx, 1, gz), dim3(BLOCK), 0, st, acc, recv, count);
  return hipGetLastError();
}

// Two streams only: here the two-wavefront block is the better one for large buffers (244
// against 252 us at 512 MB += 512 MB) and the four-wavefront block for small ones.
template <int DT>
hipError_t launch_acc(char* acc, const char* recv, size_t count, hipStream_t st) {
  const size_t bytes = count * (narrow(DT) ? 2 : 4);
  return bytes < ((size_t)32 << 20) ? launch_acc_b<DT, kBlock>(acc, recv, count, st)
                                    : launch_acc_b<DT, kBlockSmall>(acc, recv, count, st);
}

template <int DT>
hipError_t launch_ring(char* msg, const char* recv_base, size_t recv_stride, size_t count, int nranks, int rank,
                       hipStream_t st) {
  constexpr size_t ES = narrow(DT) ? 2 : 4;
  const int steps = nranks - 1;
  if (steps < 1 || steps > 65535) return hipErrorInvalidValue;
  unsigned gx, gz;
  if (!split_grid_xz(blocks_for(count, narrow(DT), kBlockSmall), kBlockSmall, &gx, &gz)) return hipErrorInvalidValue;
  const dim3 grid(gx, (unsigned)steps, gz);
  const bool fast = is16(msg) && is16(recv_base) && recv_stride % 16 == 0 && (count * ES) % 16 == 0;
  if (fast)
    hipLaunchKernelGGL((k_ring_steps<DT, true, kBlockSmall>), grid, dim3(kBlockSmall), 0, st, msg, recv_base,
                       recv_stride, count, nranks, rank);
  else
    hipLaunchKernelGGL((k_ring_steps<DT, false, kBlockSmall>), grid, dim3(kBlockSmall), 0, st, msg, recv_base,
                       recv_stride, count, nranks, rank);
  return hipGetLastError();
}

template <int DT>
hipError_t launch_halving(char* msg, const char* recv, size_t count, int nranks, int rank, hipStream_t st) {
  constexpr size_t ES = narrow(DT) ? 2 : 4;
  int levels = 0;
  while ((1 << levels) < nranks) ++levels;
  if (levels < 1 || (1 << levels) != nranks || (nranks >> 1) > 65535) return hipErrorInvalidValue;
  unsigned gx, gz;
  if (!split_grid_xz(blocks_for(count, narrow(DT), kBlockSmall), kBlockSmall, &gx, &gz)) return hipErrorInvalidValue;
  const dim3 grid(gx, (unsigned)(nranks >> 1), gz);
  const bool fast = is16(msg) && is16(recv) && (count * ES) % 16 == 0;
  if (fast)
    hipLaunchKernelGGL((k_halving_steps<DT, true, kBlockSmall>), grid, dim3(kBlockSmall), 0, st, msg, recv, count,
                       levels, rank);
  else
    hipLaunchKernelGGL((k_halving_steps<DT, false, kBlockSmall>), grid, dim3(kBlockSmall), 0, st, msg, recv, count,
                       levels, rank);
  return hipGetLastError();
}

template <int DT>
hipError_t launch_acc_batched(const pccl_accumulate_pair_t* d_pairs, const pccl_accumulate_pair_t* h_pairs, int npairs,
                              hipStream_t st) {
  BatchTiles tiles;
  size_t total = 0;
  bool fast = true;
  for (int b = 0; b < npairs; ++b) {
    tiles.first_tile[b] = (uint32_t)total;
    if (h_pairs[b].count != 0) {
      total += blocks_for(h_pairs[b].count, narrow(DT), kBlockSmall);
      fast = fast && is16(h_pairs[b].acc) && is16(h_pairs[b].recv);
    }
    if (total > 0xFFFFFFFFull) return hipErrorInvalidValue;  // the prefix holds 32-bit block indices
  }
  for (int b = npairs; b <= kMaxBuckets; ++b) tiles.first_tile[b] = (uint32_t)total;
  if (total == 0) return hipSuccess;
  unsigned gx, gz;
  if (!split_grid_xz(total, kBlockSmall, &gx, &gz)) return hipErrorInvalidValue;
  if (fast)
    hipLaunchKernelGGL((k_accumulate_batched<DT, true, kBlockSmall>), dim3(gx, 1, gz), dim3(kBlockSmall), 0, st,
                       d_pairs, tiles, npairs);
  else
    hipLaunchKernelGGL((k_accumulate_batched<DT, false, kBlockSmall>), dim3(gx, 1, gz), dim3(kBlockSmall), 0, st,
                       d_pairs, tiles, npairs);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_accumulate(void* acc, const void* recv, size_t count, int dt, hipStream_t st) {
  if (count == 0) return hipSuccess;
  char* a = reinterpret_cast<char*>(acc);
  const char* r = reinterpret_cast<const char*>(recv);
  if (dt == kF32) return launch_acc<kF32>(a, r, count, st);
  if (dt == kBF16) return launch_acc<kBF16>(a, r, count, st);
  if (dt == kF16) return launch_acc<kF16>(a, r, count, st);
  return hipErrorInvalidValue;
}

hipError_t launch_ring_steps(void* msg, const void* recv_base, size_t recv_stride, size_t count, int nranks, int rank,
                             int dt, hipStream_t st) {
  if (count == 0 || nranks < 2) return hipSuccess;
  char* m = reinterpret_cast<char*>(msg);
  const char* r = reinterpret_cast<const char*>(recv_base);
  if (dt == kF32) return launch_ring<kF32>(m, r, recv_stride, count, nranks, rank, st);
  if (dt == kBF16) return launch_ring<kBF16>(m, r, recv_stride, count, nranks, rank, st);
  if (dt == kF16) return launch_ring<kF16>(m, r, recv_stride, count, nranks, rank, st);
  return hipErrorInvalidValue;
}

hipError_t launch_halving_steps(void* msg, const void* recv, size_t count, int nranks, int rank, int dt,
                                hipStream_t st) {
  if (count == 0 || nranks < 2) return hipSuccess;
  char* m = reinterpret_cast<char*>(msg);
  const char* r = reinterpret_cast<const char*>(recv);
  if (dt == kF32) return launch_halving<kF32>(m, r, count, nranks, rank, st);
  if (dt == kBF16) return launch_halving<kBF16>(m, r, count, nranks, rank, st);
  if (dt == kF16) return launch_halving<kF16>(m, r, count, nranks, rank, st);
  return hipErrorInvalidValue;
}

hipError_t launch_accumulate_batched(const pccl_accumulate_pair_t* d_pairs, const pccl_accumulate_pair_t* h_pairs,
                                     int npairs, int dt, hipStream_t st) {
  if (dt == kF32) return launch_acc_batched<kF32>(d_pairs, h_pairs, npairs, st);
  if (dt == kBF16) return launch_acc_batched<kBF16>(d_pairs, h_pairs, npairs, st);
  if (dt == kF16) return launch_acc_batched<kF16>(d_pairs, h_pairs, npairs, st);
  return hipErrorInvalidValue;
}

}  // namespace pccl
