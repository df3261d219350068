// Many-source local reduction for gfx950 (the GPU vector-reduction kernel of the paper's
// Sections III-B and IV-B, generalised from "received + local" to N x M sources summed in
// the fixed intra-node-then-inter-node order of Section IV-A).
//
// Two kernel families:
//   k_reduce            streaming: one thread owns a 16-byte input vector position and
//                       walks the sources in order; bandwidth comes from the M independent
//                       128-bit loads per lane and from occupancy.
//   k_reduce2l_lds      many small chunks (2048 ranks x 64 KB): a wavefront owns a node,
//                       the per-node sums of one element slice are staged in LDS and a
//                       final pass adds them in node order.
// Both are HBM-bound: (sources - 1) adds per element against >= 2 bytes per operand.
#include "device_utils.h"
#include "kernels.h"

namespace pccl {

namespace {

// ------------------------------------------------------------------------------------------
// source addressing (everything here is wave-uniform)
__device__ __forceinline__ const char* src_ptr(const ReduceProblem& p, int n, int g) {
  if (p.ptrs != nullptr) {
    const int idx = n * p.gpus + g;
    return idx == p.override_index ? reinterpret_cast<const char*>(p.override_ptr)
                                   : reinterpret_cast<const char*>(p.ptrs[idx]);
  }
  return p.base + (size_t)n * p.stride_n + (size_t)g * p.stride_g;
}

template <bool IN_BF16>
__device__ __forceinline__ void unpack(u32x4 v, float* f) {
  if (IN_BF16) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      f[2 * k] = bf16_lo(v[k]);
      f[2 * k + 1] = bf16_hi(v[k]);
    }
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) f[k] = __uint_as_float(v[k]);
  }
}

// ------------------------------------------------------------------------------------------
// element-wise path: ragged tails, and the reference semantics in the simplest form
template <bool IN_BF16, bool OUT_BF16>
__device__ void reduce_elem(const ReduceProblem& p, size_t e) {
  float acc = 0.0f;
  for (int n = 0; n < p.nodes; ++n) {
    float t = ld_elem<IN_BF16>(src_ptr(p, n, 0), e);
    for (int g = 1; g < p.gpus; ++g) t = t + ld_elem<IN_BF16>(src_ptr(p, n, g), e);
    if (IN_BF16 && p.round_partial) t = round_through_bf16(t);
    if (p.partial != nullptr)
      st_elem<IN_BF16>(reinterpret_cast<char*>(p.partial), (size_t)n * p.count + e, t);
    acc = (n == 0) ? t : acc + t;
  }
  st_elem<OUT_BF16>(reinterpret_cast<char*>(p.dst), e, acc);
}

// ------------------------------------------------------------------------------------------
// streaming path.  A tile is kBlock*U consecutive 16-byte input vectors; thread t owns
// vectors t, t + kBlock, ... of the tile, so every wavefront load is one contiguous 1 KB.
// M > 0: exactly M sources per node, fully unrolled (M loads in flight per lane and vector);
// M == 0: any number of sources, walked in batches of four.
template <bool IN_BF16, bool OUT_BF16, int M, int U>
__device__ __forceinline__ void reduce_tile(const ReduceProblem& p, size_t tile) {
  constexpr int VE = IN_BF16 ? 8 : 4;  // elements per 16-byte input vector
  constexpr int ES = IN_BF16 ? 2 : 4;
  const size_t nvec = p.count / VE;
  const size_t ntiles_vec = (nvec + (size_t)kBlock * U - 1) / ((size_t)kBlock * U);
  const size_t last_tile = ntiles_vec == 0 ? 0 : ntiles_vec - 1;

  size_t v[U];
  bool live[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    v[u] = tile * ((size_t)kBlock * U) + (size_t)u * kBlock + threadIdx.x;
    live[u] = v[u] < nvec;
  }

  float acc[U][VE];
  for (int n = 0; n < p.nodes; ++n) {
    float t[U][VE];
    if (M > 0) {
      u32x4 raw[M > 0 ? M : 1][U];
#pragma unroll
      for (int g = 0; g < M; ++g) {
        const char* sp = src_ptr(p, n, g);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          raw[g][u] = u32x4{0u, 0u, 0u, 0u};
          if (live[u]) raw[g][u] = ld16<ES>(sp, v[u] * 16);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        unpack<IN_BF16>(raw[0][u], t[u]);
#pragma unroll
        for (int g = 1; g < M; ++g) {
          float x[VE];
          unpack<IN_BF16>(raw[g][u], x);
#pragma unroll
          for (int k = 0; k < VE; ++k) t[u][k] = t[u][k] + x[k];
        }
      }
    } else {
      {
        const char* sp = src_ptr(p, n, 0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          u32x4 r = {0u, 0u, 0u, 0u};
          if (live[u]) r = ld16<ES>(sp, v[u] * 16);
          unpack<IN_BF16>(r, t[u]);
        }
      }
      int g = 1;
      for (; g + 4 <= p.gpus; g += 4) {
        u32x4 raw[4][U];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const char* sp = src_ptr(p, n, g + j);
#pragma unroll
          for (int u = 0; u < U; ++u) {
            raw[j][u] = u32x4{0u, 0u, 0u, 0u};
            if (live[u]) raw[j][u] = ld16<ES>(sp, v[u] * 16);
          }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int u = 0; u < U; ++u) {
            float x[VE];
            unpack<IN_BF16>(raw[j][u], x);
#pragma unroll
            for (int k = 0; k < VE; ++k) t[u][k] = t[u][k] + x[k];
          }
      }
      for (; g < p.gpus; ++g) {
        const char* sp = src_ptr(p, n, g);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          u32x4 r = {0u, 0u, 0u, 0u};
          if (live[u]) r = ld16<ES>(sp, v[u] * 16);
          float x[VE];
          unpack<IN_BF16>(r, x);
#pragma unroll
          for (int k = 0; k < VE; ++k) t[u][k] = t[u][k] + x[k];
        }
      }
    }

    // node partial: round through the message dtype, optionally keep it
    const bool keep = p.partial != nullptr;
    if (IN_BF16 && (p.round_partial || keep)) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        u32x4 w;
#pragma unroll
        for (int k = 0; k < 4; ++k) w[k] = pack_bf16(t[u][2 * k], t[u][2 * k + 1]);
        if (keep && live[u])
          st16<ES>(reinterpret_cast<char*>(p.partial) + (size_t)n * p.count * ES, v[u] * 16, w);
        if (p.round_partial) unpack<true>(w, t[u]);
      }
    } else if (keep) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        u32x4 w;
#pragma unroll
        for (int k = 0; k < 4; ++k) w[k] = __float_as_uint(t[u][k]);
        if (live[u])
          st16<ES>(reinterpret_cast<char*>(p.partial) + (size_t)n * p.count * ES, v[u] * 16, w);
      }
    }

    if (n == 0) {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < VE; ++k) acc[u][k] = t[u][k];
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < VE; ++k) acc[u][k] = acc[u][k] + t[u][k];
    }
  }

  char* dst = reinterpret_cast<char*>(p.dst);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (!live[u]) continue;
    if (IN_BF16 && OUT_BF16) {
      u32x4 w;
#pragma unroll
      for (int k = 0; k < 4; ++k) w[k] = pack_bf16(acc[u][2 * k], acc[u][2 * k + 1]);
      st16<2>(dst, v[u] * 16, w);
    } else if (IN_BF16 && !OUT_BF16) {
      u32x4 w0, w1;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        w0[k] = __float_as_uint(acc[u][k]);
        w1[k] = __float_as_uint(acc[u][4 + k]);
      }
      st16<4>(dst, v[u] * 32, w0);
      st16<4>(dst, v[u] * 32 + 16, w1);
    } else if (!IN_BF16 && OUT_BF16) {
      u32x2 w = {pack_bf16(acc[u][0], acc[u][1]), pack_bf16(acc[u][2], acc[u][3])};
      st8_bf16(dst, v[u] * 8, w);
    } else {
      u32x4 w;
#pragma unroll
      for (int k = 0; k < 4; ++k) w[k] = __float_as_uint(acc[u][k]);
      st16<4>(dst, v[u] * 16, w);
    }
  }

  // ragged tail (count not a multiple of the vector width): fewer than VE elements
  if (tile == last_tile) {
    const size_t e = nvec * VE + threadIdx.x;
    if (e < p.count) reduce_elem<IN_BF16, OUT_BF16>(p, e);
  }
}

template <bool IN_BF16, bool OUT_BF16, int M, int U>
__global__ __launch_bounds__(kBlock) void k_reduce(ReduceProblem p) {
  reduce_tile<IN_BF16, OUT_BF16, M, U>(p, blockIdx.x);
}

// inner unroll and vectors per thread chosen for a source count
constexpr int unroll_u(int m) { return m == 0 ? 2 : (m <= 2 ? 4 : (m == 4 ? 2 : 1)); }
inline int pick_m(int gpus) {
  return (gpus == 1 || gpus == 2 || gpus == 4 || gpus == 8 || gpus == 16) ? gpus : 0;
}

inline size_t tiles_for(size_t count, int m, bool in_bf16) {
  const size_t ve = in_bf16 ? 8 : 4;
  const size_t per_tile = (size_t)kBlock * unroll_u(m);
  const size_t nvec = count / ve;
  const size_t t = (nvec + per_tile - 1) / per_tile;
  return t == 0 ? 1 : t;  // a lone ragged tail still needs one block
}

template <bool IN_BF16, bool OUT_BF16, int M>
hipError_t launch_m(const ReduceProblem& p, hipStream_t st) {
  const size_t tiles = tiles_for(p.count, M, IN_BF16);
  if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
  hipLaunchKernelGGL((k_reduce<IN_BF16, OUT_BF16, M, unroll_u(M)>), dim3((unsigned)tiles),
                     dim3(kBlock), 0, st, p);
  return hipGetLastError();
}

template <bool IN_BF16, bool OUT_BF16>
hipError_t launch_io(const ReduceProblem& p, hipStream_t st) {
  switch (pick_m(p.gpus)) {
    case 1: return launch_m<IN_BF16, OUT_BF16, 1>(p, st);
    case 2: return launch_m<IN_BF16, OUT_BF16, 2>(p, st);
    case 4: return launch_m<IN_BF16, OUT_BF16, 4>(p, st);
    case 8: return launch_m<IN_BF16, OUT_BF16, 8>(p, st);
    case 16: return launch_m<IN_BF16, OUT_BF16, 16>(p, st);
    default: return launch_m<IN_BF16, OUT_BF16, 0>(p, st);
  }
}

// ------------------------------------------------------------------------------------------
// LDS-staged two-level reduction for many small chunks.
//   block  = 16 wavefronts, owns E = 64 * EPL consecutive elements (EPL = elements in one
//            32-bit word: 1 for fp32, 2 for bf16) of every source;
//   wave w = sums the M sources of nodes w, w+16, ... of the current node tile (the M
//            loads of a node are independent, so they are all in flight together) and
//            parks the rounded node partial in LDS as fp32;
//   then E threads add the parked partials in ascending node order.
// Which wave computed which partial never changes the value: the association is fixed by
// the node-major order, not by the schedule.
constexpr int kLdsBlock = 1024;
constexpr int kLdsWaves = kLdsBlock / 64;

template <bool IN_BF16, int EPL>
__device__ __forceinline__ void ld_word(const char* sp, size_t le, size_t count, float* x) {
  if (!IN_BF16) {
    x[0] = (le < count) ? ld_stream<float>(sp + 4 * le) : 0.0f;
  } else {
    if (le + 1 < count && aligned_to(sp, 4)) {
      const uint32_t w = ld_stream<uint32_t>(sp + 2 * le);
      x[0] = bf16_lo(w);
      x[1] = bf16_hi(w);
    } else {
      x[0] = (le < count) ? ld_elem<true>(sp, le) : 0.0f;
      x[1] = (le + 1 < count) ? ld_elem<true>(sp, le + 1) : 0.0f;
    }
  }
}

template <bool IN_BF16, bool OUT_BF16, int M>
__global__ __launch_bounds__(kLdsBlock) void k_reduce2l_lds(ReduceProblem p, int node_tile) {
  extern __shared__ float parked[];  // [node_tile][E]
  constexpr int EPL = IN_BF16 ? 2 : 1;
  constexpr int E = 64 * EPL;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const size_t e0 = (size_t)blockIdx.x * E;
  const size_t le = e0 + (size_t)lane * EPL;

  float acc = 0.0f;
  for (int n0 = 0; n0 < p.nodes; n0 += node_tile) {
    const int tn = min(node_tile, p.nodes - n0);
#pragma unroll 2
    for (int j = wave; j < tn; j += kLdsWaves) {
      const int n = n0 + j;
      float t[EPL];
      if (M > 0) {
        float x[M > 0 ? M : 1][EPL];
#pragma unroll
        for (int g = 0; g < M; ++g) ld_word<IN_BF16, EPL>(src_ptr(p, n, g), le, p.count, x[g]);
#pragma unroll
        for (int k = 0; k < EPL; ++k) {
          t[k] = x[0][k];
#pragma unroll
          for (int g = 1; g < M; ++g) t[k] = t[k] + x[g][k];
        }
      } else {
        ld_word<IN_BF16, EPL>(src_ptr(p, n, 0), le, p.count, t);
        for (int g = 1; g < p.gpus; ++g) {
          float x[EPL];
          ld_word<IN_BF16, EPL>(src_ptr(p, n, g), le, p.count, x);
#pragma unroll
          for (int k = 0; k < EPL; ++k) t[k] = t[k] + x[k];
        }
      }
#pragma unroll
      for (int k = 0; k < EPL; ++k) {
        if (IN_BF16 && p.round_partial) t[k] = round_through_bf16(t[k]);
        parked[j * E + lane * EPL + k] = t[k];
      }
    }
    __syncthreads();
    if (threadIdx.x < E) {
      int j = 0;
      if (n0 == 0) {
        acc = parked[threadIdx.x];
        j = 1;
      }
#pragma unroll 8
      for (; j < tn; ++j) acc = acc + parked[j * E + threadIdx.x];
    }
    __syncthreads();
  }
  if (threadIdx.x < E && e0 + threadIdx.x < p.count)
    st_elem<OUT_BF16>(reinterpret_cast<char*>(p.dst), e0 + threadIdx.x, acc);
}

template <bool IN_BF16, bool OUT_BF16, int M>
hipError_t launch_lds_m(const ReduceProblem& p, hipStream_t st) {
  constexpr int E = IN_BF16 ? 128 : 64;
  const int max_tile = (64 * 1024) / (E * 4);  // 64 KB of LDS per block
  const int node_tile = p.nodes < max_tile ? p.nodes : max_tile;
  const size_t blocks = (p.count + E - 1) / E;
  if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
  const size_t lds_bytes = (size_t)node_tile * E * sizeof(float);
  hipLaunchKernelGGL((k_reduce2l_lds<IN_BF16, OUT_BF16, M>), dim3((unsigned)blocks),
                     dim3(kLdsBlock), lds_bytes, st, p, node_tile);
  return hipGetLastError();
}

template <bool IN_BF16, bool OUT_BF16>
hipError_t launch_lds_io(const ReduceProblem& p, hipStream_t st) {
  switch (p.gpus) {
    case 1: return launch_lds_m<IN_BF16, OUT_BF16, 1>(p, st);
    case 2: return launch_lds_m<IN_BF16, OUT_BF16, 2>(p, st);
    case 4: return launch_lds_m<IN_BF16, OUT_BF16, 4>(p, st);
    case 8: return launch_lds_m<IN_BF16, OUT_BF16, 8>(p, st);
    default: return launch_lds_m<IN_BF16, OUT_BF16, 0>(p, st);
  }
}

// ------------------------------------------------------------------------------------------
// batched two-level reduce-scatter share: a flat tile space over all buckets, one launch
// per phase.  Each block finds its bucket by bisection in the tile prefix (kernel argument).
template <bool BF16, int M, int PHASE>
__global__ __launch_bounds__(kBlock) void k_rs_batched(const pccl_bucket_t* __restrict__ buckets,
                                                       BatchTiles tiles, int nbuckets, int nodes,
                                                       int gpus) {
  constexpr int ES = BF16 ? 2 : 4;
  int lo = 0, hi = nbuckets;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tiles.first_tile[mid] <= blockIdx.x)
      lo = mid;
    else
      hi = mid;
  }
  const pccl_bucket_t b = buckets[lo];
  ReduceProblem p;
  p.ptrs = nullptr;
  p.override_ptr = nullptr;
  p.override_index = -1;
  p.partial = nullptr;
  p.round_partial = 0;
  p.nodes = 1;
  p.stride_n = 0;
  if (PHASE == 1) {  // partial[n][e] = sum over g' of piece_g'[n][e]
    p.dst = b.partial;
    p.base = reinterpret_cast<const char*>(b.intra_base);
    p.stride_g = b.intra_stride_bytes;
    p.count = (size_t)nodes * b.chunk_count;
    p.gpus = gpus;
  } else {  // shard[e] = sum over n' of partial[n'][e]
    p.dst = b.shard;
    p.base = reinterpret_cast<const char*>(b.partial);
    p.stride_g = b.chunk_count * ES;
    p.count = b.chunk_count;
    p.gpus = nodes;
  }
  reduce_tile<BF16, BF16, M, unroll_u(M)>(p, blockIdx.x - tiles.first_tile[lo]);
}

template <bool BF16, int M, int PHASE>
hipError_t launch_batched_phase(const pccl_bucket_t* d_buckets, const pccl_bucket_t* h_buckets,
                                int nbuckets, int nodes, int gpus, hipStream_t st) {
  BatchTiles tiles;
  size_t total = 0;
  for (int b = 0; b < nbuckets; ++b) {
    tiles.first_tile[b] = (uint32_t)total;
    const size_t count = PHASE == 1 ? (size_t)nodes * h_buckets[b].chunk_count
                                    : h_buckets[b].chunk_count;
    if (count != 0) total += tiles_for(count, M, BF16);
    if (total > 0x7FFFFFFFull) return hipErrorInvalidValue;
  }
  for (int b = nbuckets; b <= kMaxBuckets; ++b) tiles.first_tile[b] = (uint32_t)total;
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL((k_rs_batched<BF16, M, PHASE>), dim3((unsigned)total), dim3(kBlock), 0, st,
                     d_buckets, tiles, nbuckets, nodes, gpus);
  return hipGetLastError();
}

template <bool BF16, int PHASE>
hipError_t launch_batched_io(const pccl_bucket_t* d, const pccl_bucket_t* h, int nb, int nodes,
                             int gpus, hipStream_t st) {
  const int srcs = PHASE == 1 ? gpus : nodes;
  switch (pick_m(srcs)) {
    case 1: return launch_batched_phase<BF16, 1, PHASE>(d, h, nb, nodes, gpus, st);
    case 2: return launch_batched_phase<BF16, 2, PHASE>(d, h, nb, nodes, gpus, st);
    case 4: return launch_batched_phase<BF16, 4, PHASE>(d, h, nb, nodes, gpus, st);
    case 8: return launch_batched_phase<BF16, 8, PHASE>(d, h, nb, nodes, gpus, st);
    case 16: return launch_batched_phase<BF16, 16, PHASE>(d, h, nb, nodes, gpus, st);
    default: return launch_batched_phase<BF16, 0, PHASE>(d, h, nb, nodes, gpus, st);
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------
hipError_t launch_reduce(const ReduceProblem& p, bool in_bf16, bool out_bf16, hipStream_t st) {
  if (in_bf16) return out_bf16 ? launch_io<true, true>(p, st) : launch_io<true, false>(p, st);
  return out_bf16 ? launch_io<false, true>(p, st) : launch_io<false, false>(p, st);
}

hipError_t launch_reduce_two_level_lds(const ReduceProblem& p, bool in_bf16, bool out_bf16,
                                       hipStream_t st) {
  if (in_bf16)
    return out_bf16 ? launch_lds_io<true, true>(p, st) : launch_lds_io<true, false>(p, st);
  return out_bf16 ? launch_lds_io<false, true>(p, st) : launch_lds_io<false, false>(p, st);
}

bool prefer_lds_two_level(const ReduceProblem& p, bool in_bf16) {
  // The streaming kernel has count/VE threads, each walking all sources one after another.
  // Below about two wavefronts per SIMD of the chip that leaves HBM idle; the LDS kernel
  // spreads the nodes over 16 wavefronts per element slice instead.
  const size_t ve = in_bf16 ? 8 : 4;
  const size_t stream_threads = p.count / ve;
  return p.nodes * p.gpus >= 16 && stream_threads < (size_t)256 * 4 * 2 * 64;
}

hipError_t launch_rs_batched(const pccl_bucket_t* d_buckets, const pccl_bucket_t* h_buckets,
                             int nbuckets, int nodes, int gpus, bool bf16, hipStream_t st) {
  hipError_t e = bf16 ? launch_batched_io<true, 1>(d_buckets, h_buckets, nbuckets, nodes, gpus, st)
                      : launch_batched_io<false, 1>(d_buckets, h_buckets, nbuckets, nodes, gpus, st);
  if (e != hipSuccess) return e;
  return bf16 ? launch_batched_io<true, 2>(d_buckets, h_buckets, nbuckets, nodes, gpus, st)
              : launch_batched_io<false, 2>(d_buckets, h_buckets, nbuckets, nodes, gpus, st);
}

}  // namespace pccl
