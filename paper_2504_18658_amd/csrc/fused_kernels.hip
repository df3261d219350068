// The tail of one rank's two-level all-reduce in ONE launch for gfx950 (Section IV-A: an
// all-reduce is the two-level reduce-scatter followed by the two-level all-gather, whose last
// step is the device-local shuffle; Section III-A counts the intra-GPU transposes in every
// timing).  The grid is the shuffle's: one-wavefront blocks (tile, source row, source column),
// each copying one 1 KB tile of one chunk from its hierarchical slot to rank order.  The
// rank's OWN chunk is not copied from anywhere: its blocks compute it,
//     shard[e] = round_io(sum over n' of inter_n'[e]),
// with the tile bodies of the stand-alone reduction kernels, and store it straight at its
// rank-order place -- the shard never exists as a separate buffer that a later pass copies, and
// the short reduction (a few percent of the bytes, half the bandwidth of a big launch when it
// runs alone) is spread through the long copy instead of running before it.
//   * up to 16 sources: block x of the own chunk sums 1 KB of every source (one 128-bit vector
//     per lane and source) -- the same 1 KB of output a copy block would have written;
//   * more than 16 (short) sources: the LDS-staged flat slice; a slice is 256 bytes of output,
//     so these blocks do not fit the own chunk's and take extra planes of the grid, ahead of
//     the copy (they walk every source, so they start first).
// HBM-bound: 2*(P-1)*chunk bytes of shuffle plus (N+1)*chunk bytes of reduction.
// Measured on MI355X, 256 MB of bf16 at 16 x 8 ranks: 79 us for the shuffle alone, 8.9 us for
// the inter-node phase alone; four-wavefront blocks (tried first, so that the LDS body and the
// copy share a shape) made the copy itself 15 % slower, and reduction blocks gathered at the
// head of the grid run before the copy rather than under it.
#include "device_utils.h"
#include "kernels.h"
#include "permute_device.h"
#include "reduce_device.h"

namespace pccl {

namespace {

// Words per lane and source in the own chunk's blocks.  A block owes 1 KB of output (16 bytes per
// lane); with many sources that many bytes of each in flight at once would cost registers, and
// registers are per kernel: the COPY blocks would lose occupancy with them (16 sources at 16 bytes
// each: 100 us for the launch instead of 83).  So the block takes its 1 KB in 4 / W passes.
constexpr int fused_words(int kind) { return kind == 0 ? 2 : (kind <= 4 ? 4 : (kind == 8 ? 2 : 1)); }

// KIND > 0: exactly KIND sources, unrolled; 0: any number up to 16, batches of four; -1: LDS-staged
// flat slice in f.reduce_planes extra planes.
// (Eight wavefronts per SIMD are asked for: the copy lives on occupancy, and the 16 source bases of the
// widest reduction body would otherwise cost the whole kernel one of them.)
template <int DT, int KIND>
__global__ __launch_bounds__(kPermBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_phase2_reassemble(ReduceProblem p, PermuteProblem q, FusedShape f) {
  if (KIND < 0 && blockIdx.z < f.reduce_planes) {
    const size_t t = ((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    if (t < f.reduce_tiles) flat_lds_slice<DT, DT, 1, true>(p, t);  // the planes are rounded up
    return;
  }
  // chunk (r, c) of the source = hierarchical slot r*cols + c
  const uint32_t r = blockIdx.y, c = blockIdx.z - f.reduce_planes;
  uint32_t tile = blockIdx.x;
  if ((int)r == f.own_r && (int)c == f.own_c) {  // the reduction writes this chunk
    if constexpr (KIND >= 0) {
      constexpr int W = fused_words(KIND), PASSES = 4 / W;
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        const size_t t = (size_t)tile * PASSES + i;
        if (t < f.reduce_tiles) reduce_tile<DT, DT, KIND, W, false, kPermBlock>(p, t);
      }
    }
    return;
  }
  if (f.skew) tile = (uint32_t)(((uint64_t)tile + (uint64_t)(r + c) * f.skew) % f.tiles_per_chunk);
  const size_t sidx = (size_t)r * q.cols + c;
  const char* sp = q.slots != nullptr ? ld_pointer(q.slots, (int)sidx) : q.src + sidx * q.chunk_bytes;
  char* dp = q.dst + ((size_t)c * q.rows + r) * q.chunk_bytes;
  copy_chunk_tile(sp, dp, q.chunk_bytes, tile);
}

template <int DT, int KIND>
hipError_t launch_kind(const ReduceProblem& p, const PermuteProblem& q, int own_r, int own_c, hipStream_t st) {
  constexpr int EPL = narrow(DT) ? 2 : 1;
  FusedShape f;
  f.own_r = own_r;
  f.own_c = own_c;
  const size_t tpc = tiles_per_chunk_for(q.dst, q.chunk_bytes);
  if (tpc == 0) return hipSuccess;
  if (tpc > kPermMaxTilesX || q.rows > 65535) return hipErrorInvalidValue;
  f.tiles_per_chunk = (uint32_t)tpc;
  f.skew = skew_pays(q.chunk_bytes) ? kSkewTiles : 0u;
  size_t rt, planes = 0;
  if (KIND >= 0) {
    // tiles of 64 vectors of W words, 4 / W of them per block: never more blocks than the chunk has 1 KB copy tiles
    constexpr int W = fused_words(KIND < 0 ? 0 : KIND);
    const size_t nvec = p.count / (size_t)(W * EPL);
    rt = (nvec + kPermBlock - 1) / kPermBlock;
    if (rt == 0) rt = 1;  // a lone ragged tail
    if ((rt + 4 / W - 1) / (4 / W) > tpc) return hipErrorInvalidValue;
  } else {
    const size_t nwords = (p.count + EPL - 1) / EPL;
    rt = ((nwords + 63) / 64 + 7) / 8 * 8;  // slices, dealt XCD-major in eighths
    if (p.nodes > (1 << 30) || rt > 0xFFFFFFFFull) return hipErrorInvalidValue;  // 32-bit source and tile indices
    planes = (rt + tpc * (size_t)q.rows - 1) / (tpc * (size_t)q.rows);
  }
  if (planes + (size_t)q.cols > 65535) return hipErrorInvalidValue;
  f.reduce_tiles = (uint32_t)rt;
  f.reduce_planes = (uint32_t)planes;
  hipLaunchKernelGGL((k_phase2_reassemble<DT, KIND>), dim3((unsigned)tpc, (unsigned)q.rows, (unsigned)(planes + q.cols)),
                     dim3(kPermBlock), 0, st, p, q, f);
  return hipGetLastError();
}

template <int DT>
hipError_t launch_dt(const ReduceProblem& p, const PermuteProblem& q, int own_r, int own_c, hipStream_t st) {
  // p is a flat sum of p.gpus sources; beyond 16 of them the LDS-staged slice takes it as p.nodes sources
  if (p.gpus > 16) {
    ReduceProblem z = p;
    z.nodes = p.gpus;
    z.gpus = 1;
    z.stride_n = p.stride_g;
    z.stride_g = 0;
    return launch_kind<DT, -1>(z, q, own_r, own_c, st);
  }
  switch (pick_m(p.gpus)) {
    case 1: return launch_kind<DT, 1>(p, q, own_r, own_c, st);
    case 2: return launch_kind<DT, 2>(p, q, own_r, own_c, st);
    case 4: return launch_kind<DT, 4>(p, q, own_r, own_c, st);
    case 8: return launch_kind<DT, 8>(p, q, own_r, own_c, st);
    case 16: return launch_kind<DT, 16>(p, q, own_r, own_c, st);
    default: return launch_kind<DT, 0>(p, q, own_r, own_c, st);
  }
}

}  // namespace

hipError_t launch_phase2_reassemble(const ReduceProblem& p, const PermuteProblem& q, int own_r, int own_c, int dt,
                                    hipStream_t st) {
  if (dt == kF32) return launch_dt<kF32>(p, q, own_r, own_c, st);
  if (dt == kBF16) return launch_dt<kBF16>(p, q, own_r, own_c, st);
  if (dt == kF16) return launch_dt<kF16>(p, q, own_r, own_c, st);
  return hipErrorInvalidValue;
}

}  // namespace pccl
