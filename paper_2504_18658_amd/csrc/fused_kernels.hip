// The tail of one rank's two-level all-reduce in ONE launch for gfx950 (Section IV-A: an
// all-reduce is the two-level reduce-scatter followed by the two-level all-gather, whose last
// step is the device-local shuffle; Section III-A counts the intra-GPU transposes in every
// timing).  The grid holds two kinds of blocks:
//   * inter-node phase: shard[e] = round_io(sum over n' of inter_n'[e]), the same tile bodies
//     as the stand-alone reduction kernels, storing straight into the rank's own chunk of the
//     rank-order result -- the shard never exists as a separate buffer that a later pass copies;
//   * shuffle: the P - 1 other chunks from their hierarchical slots to rank order, one 1 KB tile
//     per wavefront, four tiles per block.
// The short reduction (a few percent of the bytes, half the bandwidth of a big launch when it
// runs alone) disappears inside the long copy, and one launch is saved.
// Blocks are 256 threads so that both kinds fit one shape.  The reduction's blocks take the
// LOWEST block indices: they run longest (they walk every source), so they start first.
// HBM-bound: 2*(P-1)*chunk bytes of shuffle plus (N+1)*chunk bytes of reduction.
#include "device_utils.h"
#include "kernels.h"
#include "permute_device.h"
#include "reduce_device.h"

namespace pccl {

namespace {

constexpr int kFusedBlock = 256;
constexpr int kFusedWaves = kFusedBlock / 64;

// KIND > 0: exactly KIND sources, unrolled streaming tile; 0: any number, streaming tile in
// batches of four; -1: LDS-staged flat slice (more than 16 short sources).
template <int DT, int KIND>
__global__ __launch_bounds__(kFusedBlock) void k_phase2_reassemble(ReduceProblem p, PermuteProblem q, FusedShape f) {
  if (blockIdx.z < f.reduce_planes) {
    const size_t t = ((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    if (t >= f.reduce_tiles) return;  // the planes are rounded up
    if constexpr (KIND >= 0)
      reduce_tile<DT, DT, KIND, words_for(KIND), false, kFusedBlock>(p, t);
    else
      flat_lds_slice<DT, DT, kFusedWaves, true>(p, t);
    return;
  }
  // chunk (r, c) of the source = hierarchical slot r*cols + c; wavefront w of block x copies tile 4x + w
  const uint32_t r = blockIdx.y, c = blockIdx.z - f.reduce_planes;
  if ((int)r == f.own_r && (int)c == f.own_c) return;  // the reduction writes that chunk
  uint32_t tile = blockIdx.x * kFusedWaves + (threadIdx.x >> 6);
  if (tile >= f.tiles_per_chunk) return;
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
  if (tpc > 0xFFFFFFFFull || q.rows > 65535) return hipErrorInvalidValue;
  f.tiles_per_chunk = (uint32_t)tpc;
  f.skew = skew_pays(q.chunk_bytes) ? kSkewTiles : 0u;
  size_t rt;
  if (KIND >= 0) {
    rt = tiles_for(p.count, KIND, narrow(DT), kFusedBlock);
  } else {
    const size_t nwords = (p.count + EPL - 1) / EPL;
    rt = ((nwords + 63) / 64 + 7) / 8 * 8;  // slices, dealt XCD-major in eighths
    if (p.nodes > (1 << 30)) return hipErrorInvalidValue;  // source indices are formed in 32 bits
  }
  if (rt > 0xFFFFFFFFull) return hipErrorInvalidValue;
  f.reduce_tiles = (uint32_t)rt;
  const size_t gx = (tpc + kFusedWaves - 1) / kFusedWaves, gy = (size_t)q.rows;
  if (gx * kFusedBlock > ((size_t)1 << 31)) return hipErrorInvalidValue;  // work-items in x
  const size_t planes = (rt + gx * gy - 1) / (gx * gy);
  if (planes + (size_t)q.cols > 65535) return hipErrorInvalidValue;
  f.reduce_planes = (uint32_t)planes;
  hipLaunchKernelGGL((k_phase2_reassemble<DT, KIND>), dim3((unsigned)gx, (unsigned)gy, (unsigned)(planes + q.cols)),
                     dim3(kFusedBlock), 0, st, p, q, f);
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
