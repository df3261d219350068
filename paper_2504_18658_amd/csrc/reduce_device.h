// Device-side bodies of the reductions for gfx950, shared by the kernels that run them alone
// (reduce_kernels.hip) and by the kernel that runs the inter-node phase next to the all-gather
// shuffle (fused_kernels.hip): source addressing, the streaming tile, the LDS-staged flat slice.
#pragma once
#include "device_utils.h"
#include "kernels.h"

namespace pccl {

namespace {

// ------------------------------------------------------------------------------------------
// source addressing (everything here is wave-uniform)
// FAST: the host has checked that the sources are strided (no pointer array) and that every
// base, stride and output is 16-byte aligned, so no run-time checks are compiled in.
template <bool FAST = false>
__device__ __forceinline__ const char* src_ptr(const ReduceProblem& p, int n, int g) {
  if (!FAST && p.ptrs != nullptr) {
    const int idx = n * p.gpus + g;
    return (idx == p.override_index ? reinterpret_cast<const char*>(p.override_ptr)
                                    : ld_pointer(p.ptrs, idx)) +
           p.src_offset;
  }
  return p.base + (size_t)n * p.stride_n + (size_t)g * p.stride_g;
}

// W packed words -> fp32 values (2 per word for bf16 / fp16, 1 per word for fp32)
template <int IN, int W>
__device__ __forceinline__ void unpack(const uint32_t* w, float* f) {
#pragma unroll
  for (int k = 0; k < W; ++k) {
    if (narrow(IN)) {
      f[2 * k] = lo16<IN>(w[k]);
      f[2 * k + 1] = hi16<IN>(w[k]);
    } else {
      f[k] = __uint_as_float(w[k]);
    }
  }
}

// K vectors from K wave-uniform sources.  Unless the host has vouched for alignment (FAST),
// one vote over all K addresses picks between a body without per-load checks -- so that the
// K loads issue back to back -- and the checked, element-wise capable body.
template <int K, int W, int ES, bool FAST>
__device__ __forceinline__ void ld_batch(const char* const* sp, uint32_t lane_off, uint32_t (*raw)[W]) {
  uintptr_t bits = 0;
  if (!FAST) {
#pragma unroll
    for (int k = 0; k < K; ++k) bits |= reinterpret_cast<uintptr_t>(sp[k]);
  }
  if (FAST || (bits & (4 * W - 1)) == 0) {
#pragma unroll
    for (int k = 0; k < K; ++k) ld_words<W, ES, true>(sp[k], lane_off, raw[k]);
  } else {
#pragma unroll
    for (int k = 0; k < K; ++k) ld_words<W, ES, false>(sp[k], lane_off, raw[k]);
  }
}

// VE consecutive results of this lane, converted to the output dtype: element threadIdx.x * VE
// of the tile that starts at `dtile` (wave-uniform).  `through` (wave-uniform) picks the store's
// cache policy: written through to memory, or non-temporal (the lines may stay in the L2 and the
// last-level cache for a while).  Measured on MI355X: a result nobody reads soon is best written
// through (the 8 x 32 MB -> 32 MB reduce and the 16-chunk phase 2 behind it: 54.0 against 55.5 us
// per call; 52.0 against 54.8 us even when phase 2 then reads all 32 MB of it); hundreds of MB that
// the NEXT launch reads in full are best left non-temporal (the 40-bucket batch, whose phase 2
// reads the 650 MB of partials phase 1 has just written: 1080 against 1107 us).
template <int OUT, int VE, bool ALIGNED>
__device__ __forceinline__ void store_vals(char* dtile, const float* a, bool through) {
  const uint32_t e = threadIdx.x * VE;
  if constexpr (narrow(OUT)) {
    if constexpr (VE == 1) {
      st_elem<OUT>(dtile, e, a[0]);
    } else {
      uint32_t w[VE / 2];
#pragma unroll
      for (int k = 0; k < VE / 2; ++k) w[k] = pack16<OUT>(a[2 * k], a[2 * k + 1]);
      if (through)
        st_tile_words<VE / 2, 2, ALIGNED>(dtile, e * 2, w);
      else
        st_words<VE / 2, 2, ALIGNED>(dtile, e * 2, w);
    }
  } else {
    uint32_t w[VE];
#pragma unroll
    for (int k = 0; k < VE; ++k) w[k] = __float_as_uint(a[k]);
    constexpr int W1 = VE == 8 ? 4 : VE;
    if (through) {
      st_tile_words<W1, 4, ALIGNED>(dtile, e * 4, w);
      if constexpr (VE == 8) st_tile_words<4, 4, ALIGNED>(dtile, e * 4 + 16, w + 4);
    } else {
      st_words<W1, 4, ALIGNED>(dtile, e * 4, w);
      if constexpr (VE == 8) st_words<4, 4, ALIGNED>(dtile, e * 4 + 16, w + 4);
    }
  }
}

// ------------------------------------------------------------------------------------------
// element-wise path: ragged tails, and the reference semantics in the simplest form
template <int IN, int OUT>
__device__ void reduce_elem(const ReduceProblem& p, size_t e) {
  float acc = 0.0f;
  for (int n = 0; n < p.nodes; ++n) {
    float t = ld_elem<IN>(src_ptr<>(p, n, 0), e);
    for (int g = 1; g < p.gpus; ++g) t = t + ld_elem<IN>(src_ptr<>(p, n, g), e);
    if (narrow(IN) && p.round_partial) t = round_through<IN>(t);
    if (p.partial != nullptr)
      st_elem<IN>(reinterpret_cast<char*>(p.partial), (size_t)n * p.count + e, t);
    acc = (n == 0) ? t : acc + t;
  }
  if (p.divisor != 0.0f) acc = acc / p.divisor;
  st_elem<OUT>(reinterpret_cast<char*>(p.dst), e, acc);
}

// ------------------------------------------------------------------------------------------
// streaming path.  A thread owns one vector of W 32-bit words per source; a tile is BLOCK
// consecutive vectors, so every wavefront load is one contiguous 256*W bytes.
// M > 0: exactly M sources per node, fully unrolled (M loads in flight per lane);
// M == 0: any number of sources, walked in batches of four.
// W is picked so that a lane keeps about 32 bytes of loads in flight (M * 4W): measured on
// MI355X, more bytes per lane at full occupancy lowers the achieved HBM bandwidth.
// `shift` (< BLOCK, in vectors) moves the tile grid: thread t of tile k owns vector
// k*BLOCK + t - shift, so that the first `shift` threads of tile 0 idle and one more tile may
// be needed; the caller picks it so that wavefront loads start on cache-line boundaries.
// `head` (0 or 1 element; only without a kept partial) starts the vectors one element into the
// buffers, for 16-bit sources that begin in the middle of a 32-bit word; that element joins
// the ragged tail.
template <int IN, int OUT, int M, int W, bool FAST, int BLOCK>
__device__ __forceinline__ void reduce_tile(const ReduceProblem& p, size_t tile, size_t shift = 0,
                                            size_t head = 0) {
  constexpr int VE = narrow(IN) ? 2 * W : W;  // elements per vector
  constexpr int ES = narrow(IN) ? 2 : 4;
  constexpr int VB = 4 * W;  // bytes per vector
  const size_t nvec = (p.count - (head < p.count ? head : p.count)) / VE;
  const size_t ntiles_vec = (nvec + shift + BLOCK - 1) / BLOCK;
  const size_t last_tile = ntiles_vec == 0 ? 0 : ntiles_vec - 1;
  // both wrap below zero for the idle head of tile 0: v then fails v < nvec, and tile_off is
  // only ever added to a lane offset that brings the sum back to v * VB
  const size_t v = tile * BLOCK + threadIdx.x - shift;
  const size_t tile_off = (tile * BLOCK - shift) * (size_t)VB + head * ES;  // wave-uniform byte offset of the tile
  const uint32_t lane_off = threadIdx.x * VB;                    // this lane's offset inside the tile

  if (v < nvec) {
    float acc[VE];
    for (int n = 0; n < p.nodes; ++n) {
      float t[VE];
      if (M > 0) {
        const char* sp[M > 0 ? M : 1];
#pragma unroll
        for (int g = 0; g < M; ++g) sp[g] = src_ptr<FAST>(p, n, g) + tile_off;
        uint32_t raw[M > 0 ? M : 1][W];
        ld_batch<(M > 0 ? M : 1), W, ES, FAST>(sp, lane_off, raw);
        unpack<IN, W>(raw[0], t);
#pragma unroll
        for (int g = 1; g < M; ++g) {
          float x[VE];
          unpack<IN, W>(raw[g], x);
#pragma unroll
          for (int k = 0; k < VE; ++k) t[k] = t[k] + x[k];
        }
      } else {
        {
          uint32_t r[W];
          ld_words<W, ES, FAST>(src_ptr<FAST>(p, n, 0) + tile_off, lane_off, r);
          unpack<IN, W>(r, t);
        }
        int g = 1;
        for (; g + 4 <= p.gpus; g += 4) {
          const char* sp[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) sp[j] = src_ptr<FAST>(p, n, g + j) + tile_off;
          uint32_t raw[4][W];
          ld_batch<4, W, ES, FAST>(sp, lane_off, raw);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            float x[VE];
            unpack<IN, W>(raw[j], x);
#pragma unroll
            for (int k = 0; k < VE; ++k) t[k] = t[k] + x[k];
          }
        }
        for (; g < p.gpus; ++g) {
          uint32_t r[W];
          ld_words<W, ES, FAST>(src_ptr<FAST>(p, n, g) + tile_off, lane_off, r);
          float x[VE];
          unpack<IN, W>(r, x);
#pragma unroll
          for (int k = 0; k < VE; ++k) t[k] = t[k] + x[k];
        }
      }

      // node partial: round through the message dtype, optionally keep it
      const bool keep = p.partial != nullptr;
      char* prow = reinterpret_cast<char*>(p.partial) + (size_t)n * p.count * ES + tile_off;
      if (narrow(IN)) {
        if (p.round_partial || keep) {
          uint32_t w[W];
#pragma unroll
          for (int k = 0; k < W; ++k) w[k] = pack16<IN>(t[2 * k], t[2 * k + 1]);
          if (keep) st_tile_words<W, ES, FAST>(prow, lane_off, w);
          if (p.round_partial) unpack<IN, W>(w, t);
        }
      } else if (keep) {
        uint32_t w[W];
#pragma unroll
        for (int k = 0; k < W; ++k) w[k] = __float_as_uint(t[k]);
        st_tile_words<W, ES, FAST>(prow, lane_off, w);
      }

#pragma unroll
      for (int k = 0; k < VE; ++k) acc[k] = (n == 0) ? t[k] : acc[k] + t[k];
    }
    if (p.divisor != 0.0f) {  // op = average: one IEEE division of the finished sum
#pragma unroll
      for (int k = 0; k < VE; ++k) acc[k] = acc[k] / p.divisor;
    }
    // the tile's first output element (the head offset included: the store checks this pointer's
    // alignment; below the buffer for the idle head of tile 0, as tile_off is)
    constexpr size_t EO = narrow(OUT) ? 2 : 4;
    store_vals<OUT, VE, FAST>(reinterpret_cast<char*>(p.dst) + ((tile * BLOCK - shift) * VE + head) * EO, acc, p.keep_cached == 0);
  }

  // the head element and the ragged tail (what the vectors leave): at most VE <= 8 elements
  if (tile == last_tile) {
    const size_t e = threadIdx.x < head ? threadIdx.x : nvec * VE + threadIdx.x;
    if (e < p.count) reduce_elem<IN, OUT>(p, e);
  }
}

// words per lane and load for a given inner unroll
constexpr int words_for(int m) { return m == 0 ? 2 : (m <= 2 ? 4 : (m == 4 ? 2 : 1)); }
inline int pick_m(int gpus) {
  return (gpus == 1 || gpus == 2 || gpus == 4 || gpus == 8 || gpus == 16) ? gpus : 0;
}

// Vectors by which a row's tile grid is moved so that every wavefront load but the row's
// first starts on a 128-byte line of the first source (the others share its alignment when
// they are a multiple of 128 bytes apart, as whole messages are).  Rows start wherever the
// chunk size puts them; with chunk sizes that are multiples of 16 bytes only, line-straddling
// loads cost the 8-source row reduce 22 % (16 x 8 ranks, 2 MB + 16 B chunks: 69.6 us against
// 55.0 us for 2 MB chunks).
template <int VB>
__device__ __forceinline__ size_t line_shift(const void* row_start) {
  const uintptr_t a = reinterpret_cast<uintptr_t>(row_start);
  return (a % VB == 0) ? (a & 127) / VB : 0;
}
// 1 when a row of 16-bit elements starts in the middle of a 32-bit word: the vectors then start
// at its second element (odd chunk element counts put every other row there; measured 78-90 us
// against 56-58 us for the 8-message share when such rows take the element-wise loads).
template <int IN>
__device__ __forceinline__ size_t word_head(const void* row_start) {
  return narrow(IN) ? (reinterpret_cast<uintptr_t>(row_start) >> 1) & 1 : 0;
}

// Rows (grid.y > 1: the same reduction over `rows` strided rows of every source) start their
// tiles kRowSkewTiles further along than the row before, modulo the tiles of a row.  Rows
// are a power-of-two number of bytes apart in every source, and the blocks resident at one
// time span several rows at the SAME offsets; measured on MI355X that costs up to a third of
// the bandwidth (8 bf16 sources, 32 MB out: 48-74 us for rows of 128 KB-1 MB, 46-47 us
// with the rotation; an odd number of tiles is 1 us better than an even one, powers of two do
// not help at all).
constexpr size_t kRowSkewTiles = 131;

inline size_t tiles_for(size_t count, int m, bool in_narrow, int block = kBlock) {
  const size_t ve = (size_t)words_for(m) * (in_narrow ? 2 : 1);
  const size_t nvec = count / ve;
  const size_t t = (nvec + block - 1) / block;
  return t == 0 ? 1 : t;  // a lone ragged tail still needs one block
}

inline bool is16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Address of source s = n*gpus + g (per lane; 0 when `valid` is false).
__device__ __forceinline__ uint64_t lds_lane_src(const ReduceProblem& p, int n, int g, int gpus,
                                                 bool valid) {
  if (!valid) return 0;
  if (p.ptrs != nullptr) {
    const size_t s = (size_t)n * gpus + g;
    return (int)s == p.override_index
               ? reinterpret_cast<uint64_t>(p.override_ptr)
               : reinterpret_cast<uint64_t>(ld_pointer_lane(p.ptrs, s));
  }
  return reinterpret_cast<uint64_t>(p.base + (size_t)n * p.stride_n + (size_t)g * p.stride_g);
}

// The same in two steps for loops that fetch the addresses of the NEXT tile while this tile's
// loads are in flight.  Loads return in order, so a branch around the fetch or any use of its
// result right behind it makes the wave wait for every load ahead of the fetch.  lane_src_fetch
// therefore always loads (lanes without a source read slot 0 of the table; no entry read this
// way is ever dereferenced) and lane_src_resolve applies "no source" and the caller's own-slot
// override where the addresses are first used, a tile later.
__device__ __forceinline__ uint64_t lane_src_fetch(const ReduceProblem& p, int n, int g, int gpus,
                                                   bool valid) {
  if (p.ptrs != nullptr) {
    const size_t s = valid ? (size_t)n * gpus + g : 0;
    return reinterpret_cast<uint64_t>(ld_pointer_lane(p.ptrs, s));
  }
  return reinterpret_cast<uint64_t>(p.base + (size_t)n * p.stride_n + (size_t)g * p.stride_g);
}
__device__ __forceinline__ uint64_t lane_src_resolve(const ReduceProblem& p, uint64_t a, int n, int g,
                                                     int gpus, bool valid) {
  const bool own = p.ptrs != nullptr && (int)((size_t)n * gpus + g) == p.override_index;
  const uint64_t r = own ? reinterpret_cast<uint64_t>(p.override_ptr) : a;
  return valid ? r : 0;
}

// Lane `l`'s 64-bit value as a wave-uniform pointer.
__device__ __forceinline__ const char* lane_pointer(uint64_t v, int l) {
  const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, l);
  const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
  return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
}

// ------------------------------------------------------------------------------------------
// LDS-staged FLAT sum of many sources (phase 2 at large node counts: N sources of a few
// hundred KB each).  The streaming kernel has too few threads for such a shape and each walks
// N sources one batch after another; here every load of a slice is in flight at once.
//   block  = WAVES wavefronts, owns one slice of 64 consecutive 32-bit words (64 fp32 or 128
//            16-bit elements) of every source;
//   tile   = TN = WAVES * 8 consecutive sources: wave w loads its 8 sources' words (8 loads in
//            flight per lane, each wavefront load one contiguous 256 bytes) and parks the RAW
//            words in LDS -- in a flat sum the addend is the source value itself, so nothing
//            is computed before the ordered pass;
//   then wavefront 0 adds the parked words in ascending source order (two chains per lane
//   for 16-bit elements), one tile behind the loads (the parking area is double-buffered).
// The accumulator starts from source 0 and every add is sequential in source order, so the
// result is bit-identical to the streaming kernel's.
// A slice is only 256 bytes of each source, so when sources do not start on a cache line every
// line a block touches at the edge of its slice is also needed by the block of the next slice.
// Two measures (template LOCAL) keep that second access out of HBM: neighbouring slices run
// on the same XCD, and the loads are ordinary cached ones rather than streaming ones.
// Measured over 40 rotating 32 MB sets of bf16 (far more than the last-level cache holds), in
// 32 / 64 / 128 / 256 sources whose size is 16 bytes off a multiple of 128: 13.1 / 17.3 /
// 21.6 / 21.5 us without, 10.0 / 10.3 / 13.7 / 15.4 us with; sources on line boundaries run
// the same either way (9.1-9.5 / 9.0-9.5 / 8.9 / 10.7-11.4 us).
constexpr int kFlatNpt = 8;

// `slice` is the block's index among the launch's slices (rounded up to a multiple of 8 when
// LOCAL); every thread of the WAVES * 64-thread block must call this.
template <int IN, int OUT, int WAVES, bool LOCAL>
__device__ __forceinline__ void flat_lds_slice(const ReduceProblem& p, size_t slice) {
  constexpr int EPL = narrow(IN) ? 2 : 1;
  constexpr int TN = WAVES * kFlatNpt;
  __shared__ uint32_t parked[2][TN * 64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const size_t nwords = (p.count + EPL - 1) / EPL;  // a ragged last word counts
  if (LOCAL) {
    // workgroups are dealt to the 8 XCDs round-robin: give XCD x the contiguous range of
    // slices [x*per, (x+1)*per), so that neighbouring slices share an L2
    const size_t per = ((nwords + 63) / 64 + 7) / 8;
    if (slice >= 8 * per) return;  // the x*z rectangle is rounded up
    slice = (slice & 7) * per + (slice >> 3);
  }
  const size_t w0 = slice * 64;
  if (w0 >= nwords) return;  // the launch is rounded up: whole blocks past the end leave
  const size_t le = (w0 + lane) * EPL;  // this lane's first element
  const bool slice_full = (w0 + 64) * EPL <= p.count;  // block-uniform
  const int nsrc = p.nodes;
  const int ntiles = (nsrc + TN - 1) / TN;

  // lane l < 8 of wave w holds the address of source tile*TN + w*8 + l
  auto fetch = [&](int tile) -> uint64_t {
    const int n = tile * TN + wave * kFlatNpt + lane;
    return lane_src_fetch(p, n, 0, 1, lane < kFlatNpt && n < nsrc);
  };
  auto resolve = [&](uint64_t a, int tile) -> uint64_t {
    const int n = tile * TN + wave * kFlatNpt + lane;
    return lane_src_resolve(p, a, n, 0, 1, lane < kFlatNpt && n < nsrc);
  };
  // acc (+)= the tn parked words of this lane, ascending source order
  float acc[EPL];
  auto ordered = [&](const uint32_t* buf, int tn, bool first) {
    int j = 0;
    if (first) {
      const uint32_t w = buf[lane];
      if constexpr (narrow(IN)) {
        acc[0] = lo16<IN>(w);
        acc[1] = hi16<IN>(w);
      } else {
        acc[0] = __uint_as_float(w);
      }
      j = 1;
    }
#pragma unroll 8
    for (; j < tn; ++j) {
      const uint32_t w = buf[j * 64 + lane];
      if constexpr (narrow(IN)) {
        acc[0] = acc[0] + lo16<IN>(w);
        acc[1] = acc[1] + hi16<IN>(w);
      } else {
        acc[0] = acc[0] + __uint_as_float(w);
      }
    }
  };

  uint64_t cur = resolve(fetch(0), 0);
  for (int k = 0; k < ntiles; ++k) {
    const uint64_t nxt = k + 1 < ntiles ? fetch(k + 1) : 0;  // resolved at the bottom of the loop
    const int nvalid = min(kFlatNpt, max(0, nsrc - (k * TN + wave * kFlatNpt)));  // wave-uniform
    uint32_t raw[kFlatNpt];
    if (nvalid == kFlatNpt && slice_full && !__any((int)(cur & 3))) {
      // the whole trip without a check: 8 loads issue back to back
#pragma unroll
      for (int q = 0; q < kFlatNpt; ++q) {
        const char* a = lane_pointer(cur, q) + 4 * (w0 + lane);
        if constexpr (LOCAL)
          raw[q] = *((const PCCL_GLOBAL uint32_t*)a);
        else
          raw[q] = ld_stream<uint32_t>(a);
      }
    } else if (narrow(IN) && nvalid == kFlatNpt && slice_full && !__any((int)(cur & 1))) {
      // Some source starts in the middle of a 32-bit word (an odd number of 16-bit elements
      // per chunk puts every other chunk there).  Every lane loads the ALIGNED word that
      // holds its first element; for a mid-word source the lane's second element is the low
      // half of the next lane's word (lane 63 fetches that word itself).  Every word read
      // holds at least one element of the slice, and no access is narrower than 32 bits.
      uint32_t lo_word[kFlatNpt], next_word[kFlatNpt];
#pragma unroll
      for (int q = 0; q < kFlatNpt; ++q) {
        const uintptr_t sp = reinterpret_cast<uintptr_t>(lane_pointer(cur, q));
        const char* a = reinterpret_cast<const char*>(sp & ~(uintptr_t)3) + 4 * (w0 + lane);
        if constexpr (LOCAL)
          lo_word[q] = *((const PCCL_GLOBAL uint32_t*)a);
        else
          lo_word[q] = ld_stream<uint32_t>(a);
      }
#pragma unroll
      for (int q = 0; q < kFlatNpt; ++q) {
        const uintptr_t sp = reinterpret_cast<uintptr_t>(lane_pointer(cur, q));
        next_word[q] = 0;
        if ((sp & 2) && lane == 63)
          next_word[q] = ld_stream<uint32_t>(reinterpret_cast<const char*>(sp & ~(uintptr_t)3) + 4 * (w0 + 64));
      }
#pragma unroll
      for (int q = 0; q < kFlatNpt; ++q) {
        const uintptr_t sp = reinterpret_cast<uintptr_t>(lane_pointer(cur, q));
        if (sp & 2) {
          uint32_t nb = __shfl_down(lo_word[q], 1);
          if (lane == 63) nb = next_word[q];
          raw[q] = (lo_word[q] >> 16) | (nb << 16);
        } else {
          raw[q] = lo_word[q];
        }
      }
    } else {
#pragma unroll
      for (int q = 0; q < kFlatNpt; ++q)
        if (q < nvalid) {
          const char* sp = lane_pointer(cur, q);
          if constexpr (narrow(IN)) {
            if (le + 1 < p.count && aligned_to(sp, 4)) {
              raw[q] = ld_stream<uint32_t>(sp + 2 * le);
            } else {
              const uint32_t a = le < p.count ? ld_stream<uint16_t>(sp + 2 * le) : 0u;
              const uint32_t b = le + 1 < p.count ? ld_stream<uint16_t>(sp + 2 * le + 2) : 0u;
              raw[q] = a | (b << 16);
            }
          } else {
            raw[q] = le < p.count ? ld_stream<uint32_t>(sp + 4 * le) : 0u;
          }
        }
    }
    // ordered sum of the previous tile while this tile's loads are in flight
    if (wave == 0 && k > 0) ordered(parked[(k - 1) & 1], TN, k == 1);
    uint32_t* buf = parked[k & 1];
#pragma unroll
    for (int q = 0; q < kFlatNpt; ++q)
      if (q < nvalid) buf[(wave * kFlatNpt + q) * 64 + lane] = raw[q];
    cur = resolve(nxt, k + 1);
    __syncthreads();
  }
  if (wave == 0) {
    const int last = ntiles - 1;
    ordered(parked[last & 1], nsrc - last * TN, last == 0);
    if (p.divisor != 0.0f) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] = acc[e] / p.divisor;
    }
    char* dst = reinterpret_cast<char*>(p.dst);
    if constexpr (narrow(OUT) && narrow(IN)) {
      if (slice_full && aligned_to(dst, 4)) {
        st_stream<uint32_t>(dst + 2 * le, pack16<OUT>(acc[0], acc[1]));
        return;
      }
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e)
      if (le + e < p.count) st_elem<OUT>(dst, le + e, acc[e]);
  }
}

}  // namespace

}  // namespace pccl
