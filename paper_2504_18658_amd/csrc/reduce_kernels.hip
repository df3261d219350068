// Many-source local reduction for gfx950 (the GPU vector-reduction kernel of the paper's
// Sections III-B and IV-B, generalised from "received + local" to N x M sources summed in
// the fixed intra-node-then-inter-node order of Section IV-A).
//
// Kernel families:
//   k_reduce            streaming: one thread owns a 4..16-byte vector position and walks
//                       the sources in order; bandwidth comes from the M independent
//                       loads per lane and from occupancy.  With grid.y > 1 the same over
//                       strided rows (the share straight from rank-order messages).
//   k_reduce2l_lds      many small chunks (2048 ranks x 64 KB): a wavefront owns a node,
//                       the per-node sums of one element slice are staged in LDS and a
//                       final pass adds them in node order.
//   k_flat_lds          flat sum of more than 16 short sources (phase 2 at large node
//                       counts): raw words staged in LDS, ordered pass one tile behind.
//   k_rs_batched[_rows] the streaming tile body over a flat tile space of many buckets.
// All are HBM-bound: (sources - 1) adds per element against >= 2 bytes per operand.
#include "device_utils.h"
#include "kernels.h"
#include "knobs.h"
#include "reduce_device.h"

namespace pccl {

namespace {

// Tile `tile` of row `row` of a launch over strided rows (the share straight from rank-order
// messages): rows start at rotated tiles, and a row that may start off a cache line is shifted
// so that wavefront loads start on line boundaries.
template <int IN, int OUT, int M, bool FAST, int BLOCK>
__device__ __forceinline__ void reduce_row_tile(ReduceProblem p, size_t tile, size_t row) {
  constexpr size_t VE = (size_t)words_for(M) * (narrow(IN) ? 2 : 1);
  const size_t nvec = p.count / VE;
  size_t ntiles = (nvec + BLOCK - 1) / BLOCK;
  if (ntiles == 0) ntiles = 1;       // a lone ragged tail
  ntiles += p.row_pad;               // room for the line shift below
  if (tile >= ntiles) return;        // the x*z rectangle is rounded up
  size_t shift = 0, head = 0;
  tile = (tile + row * kRowSkewTiles) % ntiles;
  p.base += row * p.row_stride_src;
  p.src_offset += row * p.row_stride_src;
  p.dst = reinterpret_cast<char*>(p.dst) + row * p.row_stride_dst;
  if (p.row_pad) {
    const char* row_start = src_ptr<FAST>(p, 0, 0);
    head = word_head<IN>(row_start);
    shift = line_shift<4 * words_for(M)>(row_start + 2 * head);
  }
  reduce_tile<IN, OUT, M, words_for(M), FAST, BLOCK>(p, tile, shift, head);
}

template <int IN, int OUT, int M, bool FAST, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_reduce(ReduceProblem p) {
  const size_t tile = linear_block_xz();
  if (gridDim.y > 1)
    reduce_row_tile<IN, OUT, M, FAST, BLOCK>(p, tile, blockIdx.y);
  else
    reduce_tile<IN, OUT, M, words_for(M), FAST, BLOCK>(p, tile, 0, 0);
}

// strided sources with every base, stride, row and output 16-byte aligned
inline bool fast_eligible(const ReduceProblem& p, bool in_narrow) {
  const size_t es = in_narrow ? 2 : 4;
  return p.ptrs == nullptr && is16(p.base) && is16(p.dst) && p.stride_n % 16 == 0 &&
         p.stride_g % 16 == 0 && p.row_stride_src % 16 == 0 && p.row_stride_dst % 16 == 0 &&
         (p.partial == nullptr || (is16(p.partial) && (p.count * es) % 16 == 0));
}

template <int IN, int OUT, int M, int BLOCK>
hipError_t launch_mb(const ReduceProblem& p, hipStream_t st) {
  // rows that may start off a cache line: one more tile per row, for the line shift
  const size_t tiles = tiles_for(p.count, M, narrow(IN), BLOCK) + (p.rows > 1 ? p.row_pad : 0);
  unsigned gx, gz;
  if (p.rows < 1 || p.rows > 65535 || !split_grid_xz(tiles, BLOCK, &gx, &gz)) return hipErrorInvalidValue;
  if (p.rows > 1 && p.partial != nullptr) return hipErrorInvalidValue;
  const dim3 grid(gx, (unsigned)p.rows, gz);  // tiles past the last one find nothing to do
  if (fast_eligible(p, narrow(IN)))
    hipLaunchKernelGGL((k_reduce<IN, OUT, M, true, BLOCK>), grid, dim3(BLOCK), 0, st, p);
  else
    hipLaunchKernelGGL((k_reduce<IN, OUT, M, false, BLOCK>), grid, dim3(BLOCK), 0, st, p);
  return hipGetLastError();
}

template <int IN, int OUT, int M>
hipError_t launch_m(const ReduceProblem& p, hipStream_t st) {
  // bytes the launch reads: small launches take two-wavefront blocks
  const size_t es = narrow(IN) ? 2 : 4;
  const size_t sources = (size_t)p.nodes * (size_t)p.gpus;
  const size_t per_source = p.count * es * (size_t)p.rows;
  // rows: two-wavefront blocks at any size (measured with the row rotation above: 46-48 us
  // against 48-56 us with four-wavefront blocks)
  // one or two sources: two-wavefront blocks at any size too (256 MB as 2 x 128 MB: 62.0 us
  // against 64.4 us)
  const bool small = p.rows > 1 || (M > 0 && M <= 2) || per_source < kSmallLaunchBytes / (sources == 0 ? 1 : sources);
  return small ? launch_mb<IN, OUT, M, kBlockSmall>(p, st) : launch_mb<IN, OUT, M, kBlock>(p, st);
}

template <int IN, int OUT>
hipError_t launch_io(const ReduceProblem& p, hipStream_t st) {
  switch (pick_m(p.gpus)) {
    case 1: return launch_m<IN, OUT, 1>(p, st);
    case 2: return launch_m<IN, OUT, 2>(p, st);
    case 4: return launch_m<IN, OUT, 4>(p, st);
    case 8: return launch_m<IN, OUT, 8>(p, st);
    case 16: return launch_m<IN, OUT, 16>(p, st);
    default: return launch_m<IN, OUT, 0>(p, st);
  }
}

// ------------------------------------------------------------------------------------------
// LDS-staged two-level reduction for many small chunks.
//   block  = 16 wavefronts, owns E = 64 * EPL consecutive elements (EPL = elements in one
//            32-bit word: 1 for fp32, 2 for bf16 / fp16) of every source;
//   tile   = TN = 16 * NPT consecutive nodes; wave w sums the M sources of nodes
//            w*NPT .. w*NPT+NPT-1 of the tile (NPT*M independent loads in flight per lane)
//            and parks the rounded node partials in LDS as fp32;
//   then E threads add the parked partials in ascending node order.
// Which wave computed which partial never changes the value: the association is fixed by
// the node-major order, not by the schedule.
// Two things keep HBM busy from the first to the last cycle of a block:
//   * no address table and no barrier ahead of the first load: the NPT*M <= 64 source
//     addresses a wave needs for a tile are consecutive entries of the node-major pointer
//     array, so ONE per-lane load fetches them (a tile ahead) and v_readlane hands each to
//     the scalar unit as the base of a load;
//   * the parking area is double-buffered: the ordered sum of tile k-1 runs while the loads
//     of tile k are in flight, so only the last tile's sum is exposed;
//   * on whole shapes (UNITS > 0 below) the next tile's loads are issued ahead of the barrier
//     and the ordered sum follows half a tile behind.
constexpr int kLdsBlock = 1024;
constexpr int kLdsWaves = kLdsBlock / 64;
constexpr int kLdsBatch = 8;  // sources per batch when the per-node count is not a template constant

// nodes per wave and tile: about 32 loads in flight per lane, parking area <= 2 x 32 KB
constexpr int lds_npt(int m, bool in_narrow) {
  if (m <= 0) return 1;
  int npt = 32 / m;
  // 16-bit sources park two floats per word loaded: four nodes keep two blocks on a CU (64 KB each),
  // except for one source per node, where eight are what keeps enough loads in flight
  const int cap = (in_narrow && m > 1) ? 4 : 8;
  if (npt > cap) npt = cap;
  return npt < 1 ? 1 : npt;
}

// one 32-bit word of a source as EPL fp32 values; CHECKED adds bounds and alignment handling
template <int IN, int EPL, bool CHECKED>
__device__ __forceinline__ void ld_word(const char* sp, size_t le, size_t count, float* x) {
  if (!narrow(IN)) {
    if (CHECKED)
      x[0] = (le < count) ? ld_stream<float>(sp + 4 * le) : 0.0f;
    else
      x[0] = ld_stream<float>(sp + 4 * le);
  } else {
    if (!CHECKED || (le + 1 < count && aligned_to(sp, 4))) {
      const uint32_t w = ld_stream<uint32_t>(sp + 2 * le);
      x[0] = lo16<IN>(w);
      x[1] = hi16<IN>(w);
    } else {
      x[0] = (le < count) ? ld_elem<IN>(sp, le) : 0.0f;
      x[1] = (le + 1 < count) ? ld_elem<IN>(sp, le + 1) : 0.0f;
    }
  }
}

// acc (+)= parked[0..tn) of one element, ascending node order; `first` starts the chain.
template <int E>
__device__ __forceinline__ float ordered_sum(const float* parked, int tn, bool first, float acc) {
  int j = 0;
  if (first) {
    acc = parked[threadIdx.x];
    j = 1;
  }
#pragma unroll 8
  for (; j < tn; ++j) acc = acc + parked[j * E + threadIdx.x];
  return acc;
}

// UNITS > 0 (chosen by the host): a whole tile of a whole element slice whose sources all start on
// 32-bit words needs no check on any load; a wave's share of such a tile is loaded, summed and
// chained in UNITS parts (below).  The nodes past the last whole tile, the block of a ragged last
// slice, and everything from the first tile with a 16-bit source in mid-word on take the plain loop.
template <int IN, int OUT, int M, int NPT = lds_npt(M, narrow(IN)), int UNITS = 0>
__global__ __launch_bounds__(kLdsBlock) void k_reduce2l_lds(ReduceProblem p) {
  constexpr int EPL = narrow(IN) ? 2 : 1;
  constexpr int E = 64 * EPL;
  constexpr int TN = kLdsWaves * NPT;
  constexpr int MM = M > 0 ? M : kLdsBatch;
  __shared__ float parked[2][TN * E];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const size_t e0 = linear_block_xz() * E;
  if (e0 >= p.count) return;  // the x*z rectangle is rounded up: whole blocks past the end leave
  const size_t le = e0 + (size_t)lane * EPL;
  const int gpus = M > 0 ? M : p.gpus;
  const bool slice_full = e0 + E <= p.count;  // block-uniform
  const int ntiles = (p.nodes + TN - 1) / TN;

  auto park = [&](float* buf, int j, const float* t) {
#pragma unroll
    for (int k = 0; k < EPL; ++k) {
      float r = t[k];
      if (narrow(IN) && p.round_partial) r = round_through<IN>(r);
      buf[j * E + lane * EPL + k] = r;
    }
  };

  float acc = 0.0f;
  int k0 = 0;  // tiles [0, k0) are done, their ordered sums included
  if constexpr (M > 0 && UNITS > 0) {
    const int ntf = slice_full ? p.nodes / TN : 0;  // whole tiles; block-uniform
    if (ntf > 0) {
      // A wave's NPT nodes of a tile are loaded and summed in UNITS parts, and the loads of the NEXT
      // tile's part are issued as soon as the registers of this tile's are free -- ahead of the
      // barrier -- so a wave always has nearly a whole tile of loads in flight and the memory
      // pipeline of the CU does not drain at a tile boundary (one 1024-thread block per CU: nothing
      // else would fill such a gap).  Part u of all waves together is nodes [u*UT, (u+1)*UT) of the
      // tile, so the ordered sum runs one part behind the loads and only the last part's is
      // exposed.  Addresses are fetched two tiles ahead, so that the fetch is older than the loads
      // it would otherwise wait behind (loads return in order).
      static_assert(NPT % UNITS == 0, "whole parts");
      constexpr int H = NPT / UNITS;  // nodes of a wave in one part
      constexpr int UT = TN / UNITS;  // nodes of the tile in one part
      // Lane l < NPT*M holds source (node, l % M), node = part (q / H), place wave*H + q % H in it,
      // q = l / M.  No branch around the load and no use of its result here (either would make the
      // wave wait for every load ahead of it): lanes past NPT*M repeat the last source, and the
      // caller's own-slot override is applied by `resolve` when the addresses are used, a tile later.
      const int l = lane < NPT * M ? lane : NPT * M - 1;
      const int lq = l / M, lg = l % M;
      const int lnode = (lq / H) * UT + wave * H + lq % H;
      auto fetch = [&](int tile) -> uint64_t {
        const int n = tile * TN + lnode;
        if (p.ptrs != nullptr) return reinterpret_cast<uint64_t>(ld_pointer_lane(p.ptrs, (size_t)n * M + lg));
        return reinterpret_cast<uint64_t>(p.base + (size_t)n * p.stride_n + (size_t)lg * p.stride_g);
      };
      auto resolve = [&](uint64_t a, int tile) -> uint64_t {
        const int s = (tile * TN + lnode) * M + lg;
        return (p.ptrs != nullptr && s == p.override_index) ? reinterpret_cast<uint64_t>(p.override_ptr) : a;
      };
      // part u of this wave's share: lanes (u*H + q)*M + g.  The registers hold the raw words (two
      // 16-bit elements each), unpacked when summed.
      const size_t lane_byte = le * (narrow(IN) ? 2 : 4);
      auto issue = [&](uint32_t (&x)[H][MM], uint64_t a, int u) {
#pragma unroll
        for (int q = 0; q < H; ++q)
#pragma unroll
          for (int g = 0; g < MM; ++g) x[q][g] = ld_stream<uint32_t>(lane_pointer(a, (u * H + q) * M + g) + lane_byte);
      };
      auto word = [&](uint32_t w, float* v) {
        if constexpr (narrow(IN)) {
          v[0] = lo16<IN>(w);
          v[1] = hi16<IN>(w);
        } else {
          v[0] = __uint_as_float(w);
        }
      };
      auto sum_park = [&](float* buf, const uint32_t (&x)[H][MM], int u) {
#pragma unroll
        for (int q = 0; q < H; ++q) {
          float t[EPL];
          word(x[q][0], t);
#pragma unroll
          for (int g = 1; g < MM; ++g) {
            float v[EPL];
            word(x[q][g], v);
#pragma unroll
            for (int e = 0; e < EPL; ++e) t[e] = t[e] + v[e];
          }
          park(buf, u * UT + wave * H + q, t);
        }
      };
      // acc (+)= the UT parked partials of one element, ascending node order, 16 reads at a time
      static_assert(UT % 16 == 0, "whole rounds of 16");
      auto chain = [&](const float* part, bool first) {
#pragma unroll
        for (int j0 = 0; j0 < UT; j0 += 16) {
          float v[16];
#pragma unroll
          for (int j = 0; j < 16; ++j) v[j] = part[(j0 + j) * E + threadIdx.x];
#pragma unroll
          for (int j = 0; j < 16; ++j) acc = (first && j0 + j == 0) ? v[j] : acc + v[j];
        }
      };
      // 16-bit sources may start in the middle of a 32-bit word, which only their addresses tell:
      // the block votes on every tile's addresses before that tile's loads are issued (they arrive
      // a tile ahead), and the first tile with such a source ends this loop: the plain loop takes
      // it and the rest.  The vote is block-uniform, so every wavefront leaves at the same tile.
      constexpr bool kVote = narrow(IN);
      uint64_t nxt = ntf > 1 ? fetch(1) : 0;
      uint32_t x[UNITS][H][MM];
      int npipe = ntf;  // whole tiles this loop takes
      const uint64_t cur = resolve(fetch(0), 0);
      if (kVote && __syncthreads_or((int)__any((int)(cur & 3)))) npipe = 0;
      if (npipe > 0) {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) issue(x[u], cur, u);
        for (int k = 0; k + 1 < npipe; ++k) {
          float* buf = parked[k & 1];
          const uint64_t nn = k + 2 < ntf ? fetch(k + 2) : 0;
          const uint64_t a = resolve(nxt, k + 1);
          if (kVote && __syncthreads_or((int)__any((int)(a & 3)))) {
            npipe = k + 1;  // tile k, whose loads are in flight, is the last one here
            break;
          }
#pragma unroll
          for (int u = 0; u < UNITS; ++u) {
            sum_park(buf, x[u], u);
            issue(x[u], a, u);
            __syncthreads();
            if (threadIdx.x < E) chain(buf + u * UT * E, k == 0 && u == 0);
          }
          nxt = nn;
        }
        {
          const int k = npipe - 1;
          float* buf = parked[k & 1];
#pragma unroll
          for (int u = 0; u < UNITS; ++u) {
            sum_park(buf, x[u], u);
            __syncthreads();
            if (threadIdx.x < E) chain(buf + u * UT * E, k == 0 && u == 0);
          }
        }
      }
      k0 = npipe;
    }
  }
  if constexpr (M > 0) {
    if (k0 < ntiles) {
      // lane l < NPT*M of wave w holds the address of source (tile*TN + w*NPT + l/M, l%M)
      auto fetch = [&](int tile) -> uint64_t {
        const int n = tile * TN + wave * NPT + lane / M;
        return lane_src_fetch(p, n, lane % M, M, lane < NPT * M && n < p.nodes);
      };
      auto resolve = [&](uint64_t a, int tile) -> uint64_t {
        const int n = tile * TN + wave * NPT + lane / M;
        return lane_src_resolve(p, a, n, lane % M, M, lane < NPT * M && n < p.nodes);
      };
      uint64_t cur = resolve(fetch(k0), k0);
      for (int k = k0; k < ntiles; ++k) {
        float* buf = parked[k & 1];
        const uint64_t nxt = k + 1 < ntiles ? fetch(k + 1) : 0;  // resolved at the bottom of the loop
        const int nvalid = min(NPT, max(0, p.nodes - (k * TN + wave * NPT)));  // wave-uniform
        float x[NPT][MM][EPL];
        const bool plain = nvalid == NPT && slice_full && !__any((int)(cur & 3));
        if (plain) {
          // the whole trip without a check: NPT*M loads issue back to back
#pragma unroll
          for (int q = 0; q < NPT; ++q)
#pragma unroll
            for (int g = 0; g < MM; ++g)
              ld_word<IN, EPL, false>(lane_pointer(cur, q * M + g), le, p.count, x[q][g]);
        } else {
#pragma unroll
          for (int q = 0; q < NPT; ++q)
            if (q < nvalid) {
#pragma unroll
              for (int g = 0; g < MM; ++g)
                ld_word<IN, EPL, true>(lane_pointer(cur, q * M + g), le, p.count, x[q][g]);
            }
        }
        // ordered sum of the previous tile while this tile's loads are in flight
        if (threadIdx.x < E && k > k0) acc = ordered_sum<E>(parked[(k - 1) & 1], TN, k == 1, acc);
#pragma unroll
        for (int q = 0; q < NPT; ++q)
          if (q < nvalid) {
            float t[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
              t[e] = x[q][0][e];
#pragma unroll
              for (int g = 1; g < MM; ++g) t[e] = t[e] + x[q][g][e];
            }
            park(buf, wave * NPT + q, t);
          }
        cur = resolve(nxt, k + 1);
        __syncthreads();
      }
    }
  } else {
    // any number of sources per node: one node per wave and tile, sources in batches of 8
    for (int k = 0; k < ntiles; ++k) {
      float* buf = parked[k & 1];
      const int n = k * TN + wave;
      if (threadIdx.x < E && k > 0) acc = ordered_sum<E>(parked[(k - 1) & 1], TN, k == 1, acc);
      if (n < p.nodes) {
        float t[EPL];
        for (int g0 = 0; g0 < gpus; g0 += kLdsBatch) {
          const int nb = min(kLdsBatch, gpus - g0);
          const uint64_t a = lds_lane_src(p, n, g0 + lane, gpus, lane < nb);
          float x[kLdsBatch][EPL];
#pragma unroll
          for (int j = 0; j < kLdsBatch; ++j)
            if (j < nb) ld_word<IN, EPL, true>(lane_pointer(a, j), le, p.count, x[j]);
#pragma unroll
          for (int j = 0; j < kLdsBatch; ++j)
            if (j < nb) {
#pragma unroll
              for (int e = 0; e < EPL; ++e) t[e] = (g0 + j == 0) ? x[j][e] : t[e] + x[j][e];
            }
        }
        park(buf, wave, t);
      }
      __syncthreads();
    }
  }
  if (threadIdx.x < E) {
    const int last = ntiles - 1;
    if (k0 < ntiles) acc = ordered_sum<E>(parked[last & 1], p.nodes - last * TN, last == 0, acc);
    if (p.divisor != 0.0f) acc = acc / p.divisor;
    if (e0 + threadIdx.x < p.count)
      st_elem<OUT>(reinterpret_cast<char*>(p.dst), e0 + threadIdx.x, acc);
  }
}

template <int IN, int OUT, int M>
hipError_t launch_lds_m(const ReduceProblem& p, hipStream_t st) {
  constexpr int E = narrow(IN) ? 128 : 64;
  const size_t blocks = (p.count + E - 1) / E;
  // node and source indices are formed in 32 bits, tile padding included
  if (p.nodes > (1 << 30) || (size_t)p.nodes * (size_t)p.gpus > ((size_t)1 << 30)) return hipErrorInvalidValue;
  unsigned gx, gz;
  if (!split_grid_xz(blocks, kLdsBlock, &gx, &gz)) return hipErrorInvalidValue;
  // At least one whole tile of nodes and one whole slice: the variant that loads, sums and chains a
  // whole tile in two parts and keeps loads in flight across tile boundaries (16-bit sources that
  // start in mid-word make it hand over to the plain loop, tile by tile).  2048 x 64 KB of fp32:
  // 23.25 us against 24.9 us back to back.  PCCL_TWO_LEVEL_PIPE=0 keeps the plain loop (tests run both).
  auto piped_ok = [&](int npt) {
    return knobs().two_level_pipe && p.nodes >= kLdsWaves * npt && p.count >= (size_t)E;
  };
  const dim3 grid(gx, 1, gz), blk(kLdsBlock);
  if constexpr (M > 0) {
    constexpr int NPT = lds_npt(M, narrow(IN));
    if (piped_ok(NPT)) {
      hipLaunchKernelGGL((k_reduce2l_lds<IN, OUT, M, NPT, 2>), grid, blk, 0, st, p);
      return hipGetLastError();
    }
  }
  if constexpr (M == 8 && !narrow(IN)) {
    // the plain loop on 2048 ranks x 64 KB of fp32: eight nodes per wavefront and tile (64 loads in flight per
    // lane, two barriers fewer) measured 24.5 us against 25.1 us with four; PCCL_TWO_LEVEL_NPT=4 keeps the four.
    // (The in-flight variant above stays at four: 23.25 us, and with eight it does not fit the register file.)
    if (knobs().two_level_npt != 4) {
      hipLaunchKernelGGL((k_reduce2l_lds<IN, OUT, M, 8>), grid, blk, 0, st, p);
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL((k_reduce2l_lds<IN, OUT, M>), grid, blk, 0, st, p);
  return hipGetLastError();
}

template <int IN, int OUT>
hipError_t launch_lds_io(const ReduceProblem& p, hipStream_t st) {
  switch (p.gpus) {
    case 1: return launch_lds_m<IN, OUT, 1>(p, st);
    case 2: return launch_lds_m<IN, OUT, 2>(p, st);
    case 4: return launch_lds_m<IN, OUT, 4>(p, st);
    case 8: return launch_lds_m<IN, OUT, 8>(p, st);
    case 16: return launch_lds_m<IN, OUT, 16>(p, st);
    default: return launch_lds_m<IN, OUT, 0>(p, st);
  }
}

// ------------------------------------------------------------------------------------------
// The LDS-staged flat sum (flat_lds_slice in reduce_device.h) as a kernel of its own.
template <int IN, int OUT, int WAVES, bool LOCAL>
__global__ __launch_bounds__(WAVES * 64) void k_flat_lds(ReduceProblem p) {
  flat_lds_slice<IN, OUT, WAVES, LOCAL>(p, linear_block_xz());
}

template <int IN, int OUT>
hipError_t launch_flat_lds_io(const ReduceProblem& p, hipStream_t st) {
  constexpr int EPL = narrow(IN) ? 2 : 1;
  const size_t nwords = (p.count + EPL - 1) / EPL;
  const size_t blocks = (nwords + 63) / 64;
  if (p.gpus != 1 || p.rows != 1 || p.partial != nullptr) return hipErrorInvalidValue;
  if (p.nodes > (1 << 30)) return hipErrorInvalidValue;  // source indices are formed in 32 bits, tile padding included
  unsigned gx, gz;
  // Block shape, measured over 2-512 MB of sources and 24-256 of them: four wavefronts (more
  // blocks per CU, so that one block's ordered pass hides behind the others' loads) unless the
  // sources are many and short, where sixteen put a whole slice's loads in flight at once.
  const size_t src_bytes = p.count * (narrow(IN) ? 2 : 4);
  int waves = (p.nodes <= 32 || src_bytes >= ((size_t)256 << 10)) ? 4 : (p.nodes <= 64 ? 8 : 16);
  if (knobs().flat_waves != 0) waves = knobs().flat_waves;
  const bool local = knobs().flat_local != 0;  // off for A/B runs only
  const size_t launch_blocks = local ? (blocks + 7) / 8 * 8 : blocks;
  if (!split_grid_xz(launch_blocks, (unsigned)waves * 64, &gx, &gz)) return hipErrorInvalidValue;
  const dim3 grid(gx, 1, gz), block((unsigned)waves * 64);
  if (waves == 4 && local)
    hipLaunchKernelGGL((k_flat_lds<IN, OUT, 4, true>), grid, block, 0, st, p);
  else if (waves == 4)
    hipLaunchKernelGGL((k_flat_lds<IN, OUT, 4, false>), grid, block, 0, st, p);
  else if (waves == 8 && local)
    hipLaunchKernelGGL((k_flat_lds<IN, OUT, 8, true>), grid, block, 0, st, p);
  else if (waves == 8)
    hipLaunchKernelGGL((k_flat_lds<IN, OUT, 8, false>), grid, block, 0, st, p);
  else if (local)
    hipLaunchKernelGGL((k_flat_lds<IN, OUT, 16, true>), grid, block, 0, st, p);
  else
    hipLaunchKernelGGL((k_flat_lds<IN, OUT, 16, false>), grid, block, 0, st, p);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Both phases of a two-level reduce-scatter share in one launch, when the other nodes' chunks
// are there already (d_inter).  Of the partial, only the row of the rank's own node feeds phase 2
// (the other rows leave for the other nodes), so nothing forces a second launch to wait for the
// whole of phase 1: the tiles of the OWN row go on, in the same block, to add the received
// chunks in node order and store the shard.  The own row is then written but never read back
// (2*C*e bytes of the 35 MB a separate phase 2 moves at half the bandwidth of a large launch),
// and a dispatch with its fixed cost disappears.
//   T0 tiles of the own row: phase 1 of C elements, then phase 2 of the same
//   TA tiles: phase 1 of the rows below my_node (one flat reduction of my_node*C elements)
//   TB tiles: phase 1 of the rows above it
// The own row's tiles (M + N - 1 loads per lane) take the lowest block indices.  Dealing them evenly among the
// others instead measured the same (52.2 against 52.0 us at 16 x 8 x 2 MB) -- provided their places cycle
// through the residues mod 8: blocks go to the 8 XCDs round-robin, and with one such tile at every 16th block
// ALL of them ran on one XCD, which finished 30 us after the other seven (81 us for the launch).
// Same adds in the same order as the two-launch form, so the same bits.
// MANY = more than kShareFusedMaxNodes nodes: the received chunks are then loaded and added in
// rounds of kShareFusedMaxNodes (still ascending node order, one sequential chain per element).
template <int DT, int M, bool FAST, int BLOCK, bool MANY>
__device__ __forceinline__ void own_row_tile(const ShareProblem& s, size_t tile) {
  constexpr int W = words_for(M);
  constexpr int VE = narrow(DT) ? 2 * W : W;
  constexpr int ES = narrow(DT) ? 2 : 4;
  constexpr int VB = 4 * W;
  constexpr int NMAX = kShareFusedMaxNodes;
  const size_t count = s.chunk_count;
  const size_t row_off = (size_t)s.my_node * count * ES;
  const char* own = s.own_src;
  char* prow = reinterpret_cast<char*>(s.partial) + row_off;
  char* shard = reinterpret_cast<char*>(s.shard);
  const size_t nvec = count / VE;
  const size_t ntiles = (nvec + BLOCK - 1) / BLOCK;
  const size_t last_tile = ntiles == 0 ? 0 : ntiles - 1;
  const size_t v = tile * BLOCK + threadIdx.x;
  const size_t tile_off = tile * BLOCK * (size_t)VB;
  const uint32_t lane_off = threadIdx.x * VB;
  if (v < nvec) {
    const char* sp[M];
#pragma unroll
    for (int g = 0; g < M; ++g) sp[g] = own + (size_t)g * s.intra_stride + tile_off;
    uint32_t raw[M][W];
    ld_batch<M, W, ES, FAST>(sp, lane_off, raw);
    uint32_t rin[NMAX][W];
#pragma unroll
    for (int n = 0; n < NMAX; ++n)
      if (n < s.nodes && n != s.my_node) ld_words<W, ES, false>(ld_pointer(s.d_inter, n) + tile_off, lane_off, rin[n]);
    // (with MANY these are the first round's loads, in flight under phase 1 like the others)
    float t[VE];
    unpack<DT, W>(raw[0], t);
#pragma unroll
    for (int g = 1; g < M; ++g) {
      float x[VE];
      unpack<DT, W>(raw[g], x);
#pragma unroll
      for (int k = 0; k < VE; ++k) t[k] = t[k] + x[k];
    }
    // the own node's partial: rounded through the message dtype, stored, and used as rounded
    uint32_t w[W];
    if (narrow(DT)) {
#pragma unroll
      for (int k = 0; k < W; ++k) w[k] = pack16<DT>(t[2 * k], t[2 * k + 1]);
      unpack<DT, W>(w, t);
    } else {
#pragma unroll
      for (int k = 0; k < W; ++k) w[k] = __float_as_uint(t[k]);
    }
    st_tile_words<W, ES, FAST>(prow + tile_off, lane_off, w);
    float acc[VE];
#pragma unroll
    for (int n = 0; n < NMAX; ++n)
      if (n < s.nodes) {
        float x[VE];
        if (n == s.my_node) {
#pragma unroll
          for (int k = 0; k < VE; ++k) x[k] = t[k];
        } else {
          unpack<DT, W>(rin[n], x);
        }
#pragma unroll
        for (int k = 0; k < VE; ++k) acc[k] = (n == 0) ? x[k] : acc[k] + x[k];
      }
    if (MANY) {
      for (int n0 = NMAX; n0 < s.nodes; n0 += NMAX) {
#pragma unroll
        for (int j = 0; j < NMAX; ++j)
          if (n0 + j < s.nodes && n0 + j != s.my_node)
            ld_words<W, ES, false>(ld_pointer(s.d_inter, n0 + j) + tile_off, lane_off, rin[j]);
#pragma unroll
        for (int j = 0; j < NMAX; ++j)
          if (n0 + j < s.nodes) {
            float x[VE];
            if (n0 + j == s.my_node) {
#pragma unroll
              for (int k = 0; k < VE; ++k) x[k] = t[k];
            } else {
              unpack<DT, W>(rin[j], x);
            }
#pragma unroll
            for (int k = 0; k < VE; ++k) acc[k] = acc[k] + x[k];
          }
      }
    }
    if (s.divisor != 0.0f) {
#pragma unroll
      for (int k = 0; k < VE; ++k) acc[k] = acc[k] / s.divisor;
    }
    store_vals<DT, VE, FAST>(shard + tile_off, acc, true);
  }
  if (tile == last_tile) {  // the ragged tail: fewer than VE elements
    const size_t e = nvec * VE + threadIdx.x;
    if (e < count) {
      float t = ld_elem<DT>(own, e);
      for (int g = 1; g < M; ++g) t = t + ld_elem<DT>(own + (size_t)g * s.intra_stride, e);
      t = round_through<DT>(t);
      st_elem<DT>(prow, e, t);
      float acc = 0.0f;
      for (int n = 0; n < s.nodes; ++n) {
        const float x = n == s.my_node ? t : ld_elem<DT>(ld_pointer(s.d_inter, n), e);
        acc = n == 0 ? x : acc + x;
      }
      if (s.divisor != 0.0f) acc = acc / s.divisor;
      st_elem<DT>(shard, e, acc);
    }
  }
}

inline size_t own_row_tiles(size_t count, int m, bool in_narrow, int block) { return tiles_for(count, m, in_narrow, block); }

template <int DT, int M, bool FAST, bool MANY>
__global__ __launch_bounds__(kBlock) void k_share_fused(ShareProblem s, uint32_t t0, uint32_t ta, uint32_t tb) {
  constexpr size_t ES = narrow(DT) ? 2 : 4;
  const size_t block = linear_block_xz();
  if (block < t0) {
    own_row_tile<DT, M, FAST, kBlock, MANY>(s, block);
    return;
  }
  if (block >= (size_t)t0 + ta + tb) return;  // the x*z rectangle is rounded up
  const bool above = block >= (size_t)t0 + ta;
  const size_t first_row = above ? (size_t)s.my_node + 1 : 0;
  const size_t off = first_row * s.chunk_count * ES;
  ReduceProblem p;
  p.ptrs = nullptr;
  p.override_ptr = nullptr;
  p.override_index = -1;
  p.partial = nullptr;
  p.round_partial = 0;
  p.nodes = 1;
  p.stride_n = 0;
  p.src_offset = 0;
  p.row_stride_src = 0;
  p.row_stride_dst = 0;
  p.rows = 1;
  p.row_pad = 0;
  p.keep_cached = 0;
  p.divisor = 0.0f;
  p.dst = reinterpret_cast<char*>(s.partial) + off;
  p.base = s.intra_base + off;
  p.stride_g = s.intra_stride;
  p.count = (above ? (size_t)(s.nodes - 1 - s.my_node) : (size_t)s.my_node) * s.chunk_count;
  p.gpus = M;
  reduce_tile<DT, DT, M, words_for(M), FAST, kBlock>(p, block - t0 - (above ? ta : 0));
}

template <int DT, int M>
hipError_t launch_share_m(const ShareProblem& s, hipStream_t st) {
  const size_t es = narrow(DT) ? 2 : 4;
  const size_t t0 = own_row_tiles(s.chunk_count, M, narrow(DT), kBlock);
  const size_t ca = (size_t)s.my_node * s.chunk_count, cb = (size_t)(s.nodes - 1 - s.my_node) * s.chunk_count;
  const size_t ta = ca ? tiles_for(ca, M, narrow(DT), kBlock) : 0, tb = cb ? tiles_for(cb, M, narrow(DT), kBlock) : 0;
  if (t0 > 0xFFFFFFFFull || ta > 0xFFFFFFFFull || tb > 0xFFFFFFFFull) return hipErrorInvalidValue;
  unsigned gx, gz;
  if (!split_grid_xz(t0 + ta + tb, kBlock, &gx, &gz)) return hipErrorInvalidValue;
  const bool fast = is16(s.shard) && is16(s.partial) && is16(s.intra_base) && s.intra_stride % 16 == 0 &&
                    (s.chunk_count * es) % 16 == 0;
  const bool many = s.nodes > kShareFusedMaxNodes;
  const dim3 grid(gx, 1, gz), blk(kBlock);
  const uint32_t a0 = (uint32_t)t0, a1 = (uint32_t)ta, a2 = (uint32_t)tb;
  if (fast && !many)
    hipLaunchKernelGGL((k_share_fused<DT, M, true, false>), grid, blk, 0, st, s, a0, a1, a2);
  else if (fast)
    hipLaunchKernelGGL((k_share_fused<DT, M, true, true>), grid, blk, 0, st, s, a0, a1, a2);
  else if (!many)
    hipLaunchKernelGGL((k_share_fused<DT, M, false, false>), grid, blk, 0, st, s, a0, a1, a2);
  else
    hipLaunchKernelGGL((k_share_fused<DT, M, false, true>), grid, blk, 0, st, s, a0, a1, a2);
  return hipGetLastError();
}

template <int DT>
hipError_t launch_share_dt(const ShareProblem& s, hipStream_t st) {
  switch (pick_m(s.gpus)) {
    case 1: return launch_share_m<DT, 1>(s, st);
    case 2: return launch_share_m<DT, 2>(s, st);
    case 4: return launch_share_m<DT, 4>(s, st);
    case 8: return launch_share_m<DT, 8>(s, st);
    case 16: return launch_share_m<DT, 16>(s, st);
    default: return hipErrorNotSupported;
  }
}

// The same over the rows of rank-order messages: plane y = 0 holds the own row's tiles (phase 1
// and phase 2; first in dispatch order), plane y > 0 row y - 1, or y past the own row.
template <int DT, int M, bool FAST, bool MANY>
__global__ __launch_bounds__(kBlockSmall) void k_share_rows_fused(ShareProblem s, ReduceProblem rows) {
  const size_t tile = linear_block_xz();
  if (blockIdx.y == 0) {
    own_row_tile<DT, M, FAST, kBlockSmall, MANY>(s, tile);  // tiles past the row's last find nothing to do
    return;
  }
  const size_t row = (int)blockIdx.y - 1 < s.my_node ? blockIdx.y - 1 : blockIdx.y;
  reduce_row_tile<DT, DT, M, FAST, kBlockSmall>(rows, tile, row);
}

template <int DT, int M>
hipError_t launch_share_rows_m(const ShareProblem& s, const ReduceProblem& rows, hipStream_t st) {
  const size_t es = narrow(DT) ? 2 : 4;
  const size_t tiles = tiles_for(rows.count, M, narrow(DT), kBlockSmall) + rows.row_pad;
  unsigned gx, gz;
  if (rows.rows < 1 || rows.rows > 65535 || !split_grid_xz(tiles, kBlockSmall, &gx, &gz)) return hipErrorInvalidValue;
  const bool fast = fast_eligible(rows, narrow(DT)) && is16(s.shard) && is16(s.own_src) && s.intra_stride % 16 == 0 &&
                    (s.chunk_count * es) % 16 == 0;
  const bool many = s.nodes > kShareFusedMaxNodes;
  const dim3 grid(gx, (unsigned)rows.rows, gz), blk(kBlockSmall);
  if (fast && !many)
    hipLaunchKernelGGL((k_share_rows_fused<DT, M, true, false>), grid, blk, 0, st, s, rows);
  else if (fast)
    hipLaunchKernelGGL((k_share_rows_fused<DT, M, true, true>), grid, blk, 0, st, s, rows);
  else if (!many)
    hipLaunchKernelGGL((k_share_rows_fused<DT, M, false, false>), grid, blk, 0, st, s, rows);
  else
    hipLaunchKernelGGL((k_share_rows_fused<DT, M, false, true>), grid, blk, 0, st, s, rows);
  return hipGetLastError();
}

template <int DT>
hipError_t launch_share_rows_dt(const ShareProblem& s, const ReduceProblem& rows, hipStream_t st) {
  switch (pick_m(s.gpus)) {
    case 1: return launch_share_rows_m<DT, 1>(s, rows, st);
    case 2: return launch_share_rows_m<DT, 2>(s, rows, st);
    case 4: return launch_share_rows_m<DT, 4>(s, rows, st);
    case 8: return launch_share_rows_m<DT, 8>(s, rows, st);
    case 16: return launch_share_rows_m<DT, 16>(s, rows, st);
    default: return hipErrorNotSupported;
  }
}

// ------------------------------------------------------------------------------------------
// batched two-level reduce-scatter share: a flat tile space over all buckets, one launch
// per phase.  Each block finds its bucket by bisection in the tile prefix (kernel argument).
template <int DT, int M, int PHASE, bool FAST>
__global__ __launch_bounds__(kBlock) void k_rs_batched(const pccl_bucket_t* __restrict__ buckets,
                                                       BatchTiles tiles, int nbuckets, int nodes,
                                                       int gpus, float divisor) {
  constexpr int ES = narrow(DT) ? 2 : 4;
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
  const pccl_bucket_t b = buckets[lo];
  ReduceProblem p;
  p.ptrs = nullptr;
  p.override_ptr = nullptr;
  p.override_index = -1;
  p.partial = nullptr;
  p.round_partial = 0;
  p.nodes = 1;
  p.stride_n = 0;
  p.src_offset = 0;
  p.row_stride_src = 0;
  p.row_stride_dst = 0;
  p.rows = 1;
  p.row_pad = 0;
  p.keep_cached = PHASE == 1 ? 1 : 0;  // phase 2 of the batch reads every partial phase 1 writes
  p.divisor = PHASE == 2 ? divisor : 0.0f;
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
  reduce_tile<DT, DT, M, words_for(M), FAST, kBlock>(p, block - tiles.first_tile[lo]);
}

template <int DT, int M, int PHASE>
hipError_t launch_batched_phase(const pccl_bucket_t* d_buckets, const pccl_bucket_t* h_buckets,
                                int nbuckets, int nodes, int gpus, float divisor, hipStream_t st) {
  BatchTiles tiles;
  size_t total = 0;
  for (int b = 0; b < nbuckets; ++b) {
    tiles.first_tile[b] = (uint32_t)total;
    const size_t count = PHASE == 1 ? (size_t)nodes * h_buckets[b].chunk_count
                                    : h_buckets[b].chunk_count;
    if (count != 0) total += tiles_for(count, M, narrow(DT));
    if (total > 0xFFFFFFFFull) return hipErrorInvalidValue;  // the prefix holds 32-bit tile indices
  }
  for (int b = nbuckets; b <= kMaxBuckets; ++b) tiles.first_tile[b] = (uint32_t)total;
  if (total == 0) return hipSuccess;
  // every bucket 16-byte aligned in all its bases, strides and rows -> no run-time checks
  bool fast = true;
  const size_t es = narrow(DT) ? 2 : 4;
  for (int b = 0; b < nbuckets; ++b) {
    const pccl_bucket_t& k = h_buckets[b];
    if (k.chunk_count == 0) continue;
    fast = fast && is16(k.shard) && is16(k.partial) && is16(k.intra_base) &&
           k.intra_stride_bytes % 16 == 0 && (k.chunk_count * es) % 16 == 0;
  }
  unsigned gx, gz;
  if (!split_grid_xz(total, kBlock, &gx, &gz)) return hipErrorInvalidValue;
  if (fast)
    hipLaunchKernelGGL((k_rs_batched<DT, M, PHASE, true>), dim3(gx, 1, gz), dim3(kBlock), 0, st,
                       d_buckets, tiles, nbuckets, nodes, gpus, divisor);
  else
    hipLaunchKernelGGL((k_rs_batched<DT, M, PHASE, false>), dim3(gx, 1, gz), dim3(kBlock), 0, st,
                       d_buckets, tiles, nbuckets, nodes, gpus, divisor);
  return hipGetLastError();
}

// Phase 1 of the batched share straight from rank-order messages: bucket b reads chunk
// (n, my_gpu) of each of its `gpus` messages (intra_base = the first message, messages
// intra_stride_bytes apart) and writes row n of its partial.  The tile space of a bucket is
// nodes x tiles-of-a-row; rows start their tiles kRowSkewTiles apart as in k_reduce.
template <int DT, int M, bool FAST>
__global__ __launch_bounds__(kBlockSmall) void k_rs_batched_rows(const pccl_bucket_t* __restrict__ buckets,
                                                                 BatchTiles tiles, int nbuckets, int nodes,
                                                                 int gpus, int my_gpu) {
  constexpr int ES = narrow(DT) ? 2 : 4;
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
  const pccl_bucket_t b = buckets[lo];
  const uint32_t t = (uint32_t)(block - tiles.first_tile[lo]);
  const uint32_t row_tiles = (tiles.first_tile[lo + 1] - tiles.first_tile[lo]) / (uint32_t)nodes;
  const uint32_t row = t / row_tiles;
  const uint32_t tile = (uint32_t)(((uint64_t)(t - row * row_tiles) + (uint64_t)row * kRowSkewTiles) % row_tiles);
  const size_t chunk_bytes = b.chunk_count * ES;
  ReduceProblem p;
  p.ptrs = nullptr;
  p.override_ptr = nullptr;
  p.override_index = -1;
  p.partial = nullptr;
  p.round_partial = 0;
  p.nodes = 1;
  p.stride_n = 0;
  p.src_offset = 0;
  p.row_stride_src = 0;
  p.row_stride_dst = 0;
  p.rows = 1;
  p.row_pad = 0;
  p.keep_cached = 1;  // phase 2 of the batch reads every partial this launch writes
  p.divisor = 0.0f;
  p.dst = reinterpret_cast<char*>(b.partial) + (size_t)row * chunk_bytes;
  p.base = reinterpret_cast<const char*>(b.intra_base) + ((size_t)row * gpus + my_gpu) * chunk_bytes;
  p.stride_g = b.intra_stride_bytes;
  p.count = b.chunk_count;
  p.gpus = gpus;
  const size_t head = word_head<DT>(p.base);
  reduce_tile<DT, DT, M, words_for(M), FAST, kBlockSmall>(p, tile, line_shift<4 * words_for(M)>(p.base + 2 * head), head);
}

template <int DT, int M>
hipError_t launch_batched_rows(const pccl_bucket_t* d_buckets, const pccl_bucket_t* h_buckets, int nbuckets,
                               int nodes, int gpus, int my_gpu, hipStream_t st) {
  BatchTiles tiles;
  size_t total = 0;
  for (int b = 0; b < nbuckets; ++b) {
    tiles.first_tile[b] = (uint32_t)total;
    if (h_buckets[b].chunk_count != 0)
      total += (size_t)nodes * (tiles_for(h_buckets[b].chunk_count, M, narrow(DT), kBlockSmall) + 1);  // + line shift
    if (total > 0xFFFFFFFFull) return hipErrorInvalidValue;  // the prefix holds 32-bit tile indices
  }
  for (int b = nbuckets; b <= kMaxBuckets; ++b) tiles.first_tile[b] = (uint32_t)total;
  if (total == 0) return hipSuccess;
  bool fast = true;
  const size_t es = narrow(DT) ? 2 : 4;
  for (int b = 0; b < nbuckets; ++b) {
    const pccl_bucket_t& k = h_buckets[b];
    if (k.chunk_count == 0) continue;
    fast = fast && is16(k.partial) && is16(k.intra_base) && k.intra_stride_bytes % 16 == 0 &&
           (k.chunk_count * es) % 16 == 0;
  }
  unsigned gx, gz;
  if (!split_grid_xz(total, kBlockSmall, &gx, &gz)) return hipErrorInvalidValue;
  if (fast)
    hipLaunchKernelGGL((k_rs_batched_rows<DT, M, true>), dim3(gx, 1, gz), dim3(kBlockSmall), 0, st, d_buckets,
                       tiles, nbuckets, nodes, gpus, my_gpu);
  else
    hipLaunchKernelGGL((k_rs_batched_rows<DT, M, false>), dim3(gx, 1, gz), dim3(kBlockSmall), 0, st, d_buckets,
                       tiles, nbuckets, nodes, gpus, my_gpu);
  return hipGetLastError();
}

template <int DT>
hipError_t launch_batched_rows_io(const pccl_bucket_t* d, const pccl_bucket_t* h, int nb, int nodes, int gpus,
                                  int my_gpu, hipStream_t st) {
  switch (pick_m(gpus)) {
    case 1: return launch_batched_rows<DT, 1>(d, h, nb, nodes, gpus, my_gpu, st);
    case 2: return launch_batched_rows<DT, 2>(d, h, nb, nodes, gpus, my_gpu, st);
    case 4: return launch_batched_rows<DT, 4>(d, h, nb, nodes, gpus, my_gpu, st);
    case 8: return launch_batched_rows<DT, 8>(d, h, nb, nodes, gpus, my_gpu, st);
    case 16: return launch_batched_rows<DT, 16>(d, h, nb, nodes, gpus, my_gpu, st);
    default: return launch_batched_rows<DT, 0>(d, h, nb, nodes, gpus, my_gpu, st);
  }
}

template <int DT, int PHASE>
hipError_t launch_batched_io(const pccl_bucket_t* d, const pccl_bucket_t* h, int nb, int nodes,
                             int gpus, float divisor, hipStream_t st) {
  const int srcs = PHASE == 1 ? gpus : nodes;
  switch (pick_m(srcs)) {
    case 1: return launch_batched_phase<DT, 1, PHASE>(d, h, nb, nodes, gpus, divisor, st);
    case 2: return launch_batched_phase<DT, 2, PHASE>(d, h, nb, nodes, gpus, divisor, st);
    case 4: return launch_batched_phase<DT, 4, PHASE>(d, h, nb, nodes, gpus, divisor, st);
    case 8: return launch_batched_phase<DT, 8, PHASE>(d, h, nb, nodes, gpus, divisor, st);
    case 16: return launch_batched_phase<DT, 16, PHASE>(d, h, nb, nodes, gpus, divisor, st);
    default: return launch_batched_phase<DT, 0, PHASE>(d, h, nb, nodes, gpus, divisor, st);
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------
// The (input, output) dtype pairs the kernels are built for: fp32 with itself, and each 16-bit
// message type with itself or with fp32 on either side.
#define PCCL_DISPATCH_IO(FN, in_dt, out_dt, ...)                                   \
  do {                                                                             \
    if (in_dt == kF32 && out_dt == kF32) return FN<kF32, kF32>(__VA_ARGS__);       \
    if (in_dt == kBF16 && out_dt == kBF16) return FN<kBF16, kBF16>(__VA_ARGS__);   \
    if (in_dt == kBF16 && out_dt == kF32) return FN<kBF16, kF32>(__VA_ARGS__);     \
    if (in_dt == kF32 && out_dt == kBF16) return FN<kF32, kBF16>(__VA_ARGS__);     \
    if (in_dt == kF16 && out_dt == kF16) return FN<kF16, kF16>(__VA_ARGS__);       \
    if (in_dt == kF16 && out_dt == kF32) return FN<kF16, kF32>(__VA_ARGS__);       \
    if (in_dt == kF32 && out_dt == kF16) return FN<kF32, kF16>(__VA_ARGS__);       \
    return hipErrorInvalidValue;                                                   \
  } while (0)

hipError_t launch_reduce(const ReduceProblem& p, int in_dt, int out_dt, hipStream_t st) {
  PCCL_DISPATCH_IO(launch_io, in_dt, out_dt, p, st);
}

hipError_t launch_reduce_two_level_lds(const ReduceProblem& p, int in_dt, int out_dt,
                                       hipStream_t st) {
  PCCL_DISPATCH_IO(launch_lds_io, in_dt, out_dt, p, st);
}

hipError_t launch_reduce_flat_lds(const ReduceProblem& p, int in_dt, int out_dt, hipStream_t st) {
  PCCL_DISPATCH_IO(launch_flat_lds_io, in_dt, out_dt, p, st);
}

// Beyond kShareFusedMaxNodes nodes: is phase 1 long enough to cover the own row's walk?
bool share_fused_pays(const ShareProblem& s, int dt);

hipError_t launch_share_rows_fused(const ShareProblem& s, const ReduceProblem& rows, int dt, bool any_shape,
                                   hipStream_t st) {
  if (s.d_inter == nullptr || s.chunk_count == 0 || rows.ptrs != nullptr || rows.partial != nullptr)
    return hipErrorNotSupported;
  if (!any_shape && !share_fused_pays(s, dt)) return hipErrorNotSupported;
  if (dt == kF32) return launch_share_rows_dt<kF32>(s, rows, st);
  if (dt == kBF16) return launch_share_rows_dt<kBF16>(s, rows, st);
  if (dt == kF16) return launch_share_rows_dt<kF16>(s, rows, st);
  return hipErrorInvalidValue;
}

hipError_t launch_share_fused(const ShareProblem& s, int dt, bool any_shape, hipStream_t st) {
  if (s.d_inter == nullptr || s.chunk_count == 0) return hipErrorNotSupported;
  // Beyond kShareFusedMaxNodes nodes a block of the own row walks the received chunks in rounds, each
  // a pointer fetch and a load behind the last (about 1.8 us); phase 1 has to run long enough to
  // cover that chain.  Measured, bf16, 8 per node, one launch against two: 256 MB at 32-256 nodes
  // 52-53 against 57-59 us; 64 MB at 64 nodes 16.9 against 17.7, at 128 nodes 21.3 against 18.5;
  // 16 MB at 64 nodes 10.3 against 8.3.
  if (!any_shape && !share_fused_pays(s, dt)) return hipErrorNotSupported;
  if (dt == kF32) return launch_share_dt<kF32>(s, st);
  if (dt == kBF16) return launch_share_dt<kBF16>(s, st);
  if (dt == kF16) return launch_share_dt<kF16>(s, st);
  return hipErrorInvalidValue;
}

bool share_fused_pays(const ShareProblem& s, int dt) {
  if (s.nodes <= kShareFusedMaxNodes) return true;
  const size_t rounds = ((size_t)s.nodes + kShareFusedMaxNodes - 1) / kShareFusedMaxNodes;
  const size_t es = (dt == kF32) ? 4 : 2;
  const size_t phase1_in = (size_t)s.gpus * s.nodes * s.chunk_count * es;
  return phase1_in >= rounds * ((size_t)10 << 20);
}

bool prefer_flat_lds(const ReduceProblem& p, int in_dt) {
  // Up to 16 sources the streaming kernel keeps every load of a lane in flight (fully
  // unrolled); beyond, it walks the sources in batches of four and needs long sources to hide
  // that: measured equal to the LDS kernel from about 4 MB per source (24-31 sources) or
  // 16 MB (more), 2-4 times slower at 64-512 KB per source.
  const size_t src_bytes = p.count * (narrow(in_dt) ? 2 : 4);
  if (p.gpus != 1 || p.nodes <= 16) return false;
  if (src_bytes >= ((size_t)16 << 20)) return false;
  return !(src_bytes >= ((size_t)4 << 20) && p.nodes < 32);
}

bool prefer_two_level_for_flat(const ReduceProblem& p, int in_dt) {
  // A flat sum is a two-level sum with one source per node, and on many SHORT sources the
  // two-level LDS kernel's in-flight variant beats the flat LDS kernel, which drains its loads at
  // every tile of 128 sources.  Measured, fp32 through a pointer array, flat LDS against this:
  // 2048 / 1024 / 128 x 64 KB 33.7 / 18.6 / 4.7 against 22.1 / 12.4 / 4.0 us, 512 x 128 KB 16.3
  // against 12.8, 256 x 256 KB 13.9 against 13.2; 128 x 256 KB 8.3 against 8.9 and longer
  // sources within a few per cent either way; ragged shapes the same (2040 x 64 KB 33.6 against
  // 24.0, 300 x 100 KB 10.4 against 9.3).  16-bit sources mostly stay with the flat kernel, which parks
  // two elements per 32-bit word where this one parks two floats (strided bf16: 2048 x 64 KB
  // 36.8 against 36.2 us, 256 x 256 KB 13.2 against 16.4) -- except up to 64 KB per source, where
  // this one wins (bf16 through a pointer array: 2048 / 1024 / 128 x 64 KB 39.7 / 21.7 / 5.3 against
  // 30.6 / 16.5 / 4.7 us, 256 x 32 KB 7.1 against 5.7; 512 x 128 KB 17.5 against 18.0).
  // (p as launch_flat hands it on: nodes = sources.)
  if (p.gpus != 1 || !knobs().two_level_pipe) return false;
  if (p.nodes < kLdsWaves * lds_npt(1, narrow(in_dt))) return false;
  if (narrow(in_dt)) return p.count * 2 <= ((size_t)64 << 10);
  const size_t src_bytes = p.count * 4;
  return src_bytes <= ((size_t)128 << 10) || (src_bytes <= ((size_t)256 << 10) && p.nodes >= 256);
}

bool prefer_lds_two_level(const ReduceProblem& p, int in_dt) {
  // The streaming kernel has count/VE threads, each walking all sources one after another.
  // Below about two wavefronts per SIMD of the chip that leaves HBM idle; the LDS kernel
  // spreads the nodes over 16 wavefronts per element slice instead.
  const size_t ve = narrow(in_dt) ? 8 : 4;
  const size_t stream_threads = p.count / ve;
  return p.nodes * p.gpus >= 16 && stream_threads < (size_t)256 * 4 * 2 * 64;
}

hipError_t launch_rs_batched(const pccl_bucket_t* d_buckets, const pccl_bucket_t* h_buckets,
                             int nbuckets, int nodes, int gpus, int dt, float divisor,
                             hipStream_t st, int my_gpu) {
  hipError_t e = hipErrorInvalidValue;
  if (my_gpu >= 0) {  // phase 1 straight from rank-order messages
    if (dt == kF32) e = launch_batched_rows_io<kF32>(d_buckets, h_buckets, nbuckets, nodes, gpus, my_gpu, st);
    if (dt == kBF16) e = launch_batched_rows_io<kBF16>(d_buckets, h_buckets, nbuckets, nodes, gpus, my_gpu, st);
    if (dt == kF16) e = launch_batched_rows_io<kF16>(d_buckets, h_buckets, nbuckets, nodes, gpus, my_gpu, st);
  } else {
    if (dt == kF32) e = launch_batched_io<kF32, 1>(d_buckets, h_buckets, nbuckets, nodes, gpus, 0.0f, st);
    if (dt == kBF16) e = launch_batched_io<kBF16, 1>(d_buckets, h_buckets, nbuckets, nodes, gpus, 0.0f, st);
    if (dt == kF16) e = launch_batched_io<kF16, 1>(d_buckets, h_buckets, nbuckets, nodes, gpus, 0.0f, st);
  }
  if (e != hipSuccess) return e;
  if (dt == kF32) return launch_batched_io<kF32, 2>(d_buckets, h_buckets, nbuckets, nodes, gpus, divisor, st);
  if (dt == kBF16) return launch_batched_io<kBF16, 2>(d_buckets, h_buckets, nbuckets, nodes, gpus, divisor, st);
  return launch_batched_io<kF16, 2>(d_buckets, h_buckets, nbuckets, nodes, gpus, divisor, st);
}

}  // namespace pccl
