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
#include "device_utils.h"
#include "kernels.h"

namespace pccl {

namespace {

template <int DT, bool FAST, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_accumulate(char* acc, const char* recv, size_t count) {
  constexpr int W = 4;
  constexpr int VE = narrow(DT) ? 2 * W : W;
  constexpr int ES = narrow(DT) ? 2 : 4;
  const size_t nvec = count / VE;
  const size_t block = linear_block_xz();
  const size_t v = block * BLOCK + threadIdx.x;
  if (v < nvec) {
    const size_t tile = block * BLOCK * (4 * W);  // wave-uniform byte offset of the block's vectors
    const uint32_t lane_off = threadIdx.x * (4 * W);
    const size_t off = tile + lane_off;
    uint32_t a[W], r[W], o[W];
    ld_words<W, ES, FAST>(acc, off, a);
    ld_words<W, ES, FAST>(recv, off, r);
#pragma unroll
    for (int k = 0; k < W; ++k) {
      if (narrow(DT))
        o[k] = pack16<DT>(lo16<DT>(a[k]) + lo16<DT>(r[k]), hi16<DT>(a[k]) + hi16<DT>(r[k]));
      else
        o[k] = __float_as_uint(__uint_as_float(a[k]) + __uint_as_float(r[k]));
    }
    st_tile_words<W, ES, FAST>(acc + tile, lane_off, o);
  }
  // ragged tail: fewer than VE <= 8 elements, taken by the last block that holds vectors
  if (block == (nvec == 0 ? 0 : (nvec - 1) / BLOCK)) {
    const size_t e = nvec * VE + threadIdx.x;
    if (e < count) st_elem<DT>(acc, e, ld_elem<DT>(acc, e) + ld_elem<DT>(recv, e));
  }
}

inline bool is16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <int DT, int BLOCK>
hipError_t launch_acc_b(char* acc, const char* recv, size_t count, hipStream_t st) {
  constexpr size_t VE = narrow(DT) ? 8 : 4;
  const size_t nvec = count / VE;
  size_t blocks = (nvec + BLOCK - 1) / BLOCK;
  if (blocks == 0) blocks = 1;  // a lone ragged tail still needs one block
  unsigned gx, gz;
  if (!split_grid_xz(blocks, BLOCK, &gx, &gz)) return hipErrorInvalidValue;
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

}  // namespace pccl
