// Device-side helpers for the gfx950 kernels: 128-bit streaming loads/stores with an
// element-wise fallback for unaligned buffers, and bf16 / fp16 <-> fp32 conversion.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pccl {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Threads per block of the streaming kernels.  Measured on MI355X for the 8-source reduce:
// two-wavefront blocks win up to ~150 MB moved per launch (13.3 against 15.2 us at 72 MB,
// 25.4 against 27.6 at 144 MB), four-wavefront blocks from there on (47.6 against 49.3 us at
// 288 MB, 183 against 190 at 1.1 GB); the host picks by the bytes a launch moves.
constexpr int kBlock = 256;       // large launches, and the batched kernels
constexpr int kBlockSmall = 128;  // small launches
constexpr size_t kSmallLaunchBytes = (size_t)192 << 20;

// A grid dimension holds fewer than 2^32 work-items (blocks x threads), so a launch with more
// blocks than that spreads them over x and z; this is the block's index in the whole launch.
// Blocks past the last one (the x*z rectangle is rounded up) must return at once.
__device__ __forceinline__ size_t linear_block_xz() {
  return (size_t)blockIdx.z * gridDim.x + blockIdx.x;
}

// ---- message dtypes ----------------------------------------------------------------------
// Values of pccl_dtype_t, used as template parameters.  A 32-bit word holds two 16-bit
// elements: element 2k in the low half, 2k+1 in the high half.
constexpr int kF32 = 0;
constexpr int kBF16 = 1;
constexpr int kF16 = 2;
constexpr bool narrow(int dt) { return dt != kF32; }  // a 16-bit element type

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// low / high element of a packed pair, widened to fp32 (exact for both 16-bit types)
template <int DT>
__device__ __forceinline__ float lo16(uint32_t w) {
  if constexpr (DT == kF16) return (float)__builtin_bit_cast(f16x2, w)[0];
  return __uint_as_float(w << 16);
}
template <int DT>
__device__ __forceinline__ float hi16(uint32_t w) {
  if constexpr (DT == kF16) return (float)__builtin_bit_cast(f16x2, w)[1];
  return __uint_as_float(w & 0xFFFF0000u);
}

// fp32 pair -> packed 16-bit pair, round to nearest even (v_cvt_pk_bf16_f32 on gfx950 for
// bf16; v_cvt_f16_f32 for fp16, which rounds to nearest even and keeps subnormal halves).
template <int DT>
__device__ __forceinline__ uint32_t pack16(float lo, float hi) {
  f32x2 v = {lo, hi};
  if constexpr (DT == kF16) {
    f16x2 h = __builtin_convertvector(v, f16x2);
    return __builtin_bit_cast(uint32_t, h);
  } else {
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
  }
}
template <int DT>
__device__ __forceinline__ uint16_t to16(float x) {
  return (uint16_t)(pack16<DT>(x, 0.0f) & 0xFFFFu);
}
// Value of x after a trip through storage of type DT.
template <int DT>
__device__ __forceinline__ float round_through(float x) {
  if constexpr (DT == kF32) return x;
  return lo16<DT>(pack16<DT>(x, 0.0f));
}

// ---- streaming global access ------------------------------------------------------------
// Every buffer the library touches is device global memory.  Pointers arrive inside
// by-value parameter blocks, where the compiler would otherwise treat them as generic
// (flat) pointers; the casts below pin them to the global / constant address spaces so that
// global_load / global_store / s_load are emitted.  Data is touched once, so loads and
// stores carry the non-temporal hint.
#define PCCL_GLOBAL __attribute__((address_space(1)))
#define PCCL_CONSTANT __attribute__((address_space(4)))

template <typename T>
__device__ __forceinline__ T ld_stream(const void* p) {
  return __builtin_nontemporal_load((const PCCL_GLOBAL T*)p);
}
template <typename T>
__device__ __forceinline__ void st_stream(void* p, T v) {
  __builtin_nontemporal_store(v, (PCCL_GLOBAL T*)p);
}

// A pointer every lane of the wavefront holds alike, handed to the scalar unit (the compiler
// cannot always prove that; a buffer descriptor built from a per-lane pointer costs a loop).
template <typename T>
__device__ __forceinline__ T* wave_uniform(T* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((int)(uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
  return reinterpret_cast<T*>(((uint64_t)hi << 32) | lo);
}

// W words per lane stored with the write-through cache policy (sc0 sc1: the line goes to memory
// at once instead of staying dirty in the L2 until the kernel ends).  `tile` is wave-uniform,
// `off` this lane's byte offset from it (a multiple of 4*W, and tile + off aligned to 4*W);
// a lane whose [off, off + 4*W) does not lie inside [0, range) stores nothing.  The compiler
// offers this policy for 128-bit data through buffer stores only, hence the descriptor (base,
// range in bytes, 32-bit raw data).  Measured on MI355X against the non-temporal global store:
// 64 / 128 / 256 MB copies 21.2 / 40.8 / 80.1 -> 19.4 / 40.1 / 79.5 us, the 8-source bf16 sum
// moving 72 / 144 / 288 MB 13.3 / 25.6 / 48.3 -> 13.0 / 24.9 / 46.3 us; the same policy on
// loads gains nothing, and loads without the non-temporal hint lose 10-20 %.
template <int W>
__device__ __forceinline__ void st_through(char* tile, uint32_t off, uint32_t range, const uint32_t* w) {
  constexpr int kRawDwords = 0x00020000;  // descriptor word 3 on gfx9: untyped 32-bit data
  constexpr int kWriteThrough = 17;       // cache policy bits: sc0 (1) | sc1 (16)
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(tile, 0, (int)range, kRawDwords);
  if constexpr (W == 1) {
    __builtin_amdgcn_raw_buffer_store_b32(w[0], rs, (int)off, 0, kWriteThrough);
  } else if constexpr (W == 2) {
    const u32x2 v = {w[0], w[1]};
    __builtin_amdgcn_raw_buffer_store_b64(v, rs, (int)off, 0, kWriteThrough);
  } else {
    const u32x4 v = {w[0], w[1], w[2], w[3]};
    __builtin_amdgcn_raw_buffer_store_b128(v, rs, (int)off, 0, kWriteThrough);
  }
}

// Entry `idx` of a device-resident pointer array that no kernel writes (wave-uniform idx).
typedef const void* pccl_cvoidp;
__device__ __forceinline__ const char* ld_pointer(const void* const* table, int idx) {
  return reinterpret_cast<const char*>(((const PCCL_CONSTANT pccl_cvoidp*)table)[idx]);
}
// The same with a per-lane index.
__device__ __forceinline__ const char* ld_pointer_lane(const void* const* table, size_t idx) {
  return reinterpret_cast<const char*>(((const PCCL_GLOBAL pccl_cvoidp*)table)[idx]);
}

__device__ __forceinline__ bool aligned_to(const void* p, uintptr_t a) {
  return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

// W consecutive 32-bit words from base+byte_off (W = 1, 2 or 4).  The vector instruction
// needs base aligned to 4*W bytes (byte_off is always a multiple of that); otherwise the
// words are gathered with dword or halfword loads.  ES = element size the buffer is
// guaranteed aligned to (2 or 4).  ALIGNED = the caller has checked 16-byte alignment.
template <int W>
struct Words;
template <>
struct Words<1> { typedef uint32_t T; };
template <>
struct Words<2> { typedef u32x2 T; };
template <>
struct Words<4> { typedef u32x4 T; };

template <int W, int ES, bool ALIGNED = false>
__device__ __forceinline__ void ld_words(const char* base, size_t byte_off, uint32_t* w) {
  const char* p = base + byte_off;
  if (ALIGNED || aligned_to(base, 4 * W)) {
    if constexpr (W == 1) {
      w[0] = ld_stream<uint32_t>(p);
    } else {
      const typename Words<W>::T v = ld_stream<typename Words<W>::T>(p);
#pragma unroll
      for (int k = 0; k < W; ++k) w[k] = v[k];
    }
  } else if (ES == 4 || aligned_to(base, 4)) {
#pragma unroll
    for (int k = 0; k < W; ++k) w[k] = ld_stream<uint32_t>(p + 4 * k);
  } else {
#pragma unroll
    for (int k = 0; k < W; ++k) {
      const uint32_t lo = ld_stream<uint16_t>(p + 4 * k);
      const uint32_t hi = ld_stream<uint16_t>(p + 4 * k + 2);
      w[k] = lo | (hi << 16);
    }
  }
}

template <int W, int ES, bool ALIGNED = false>
__device__ __forceinline__ void st_words(char* base, size_t byte_off, const uint32_t* w) {
  char* p = base + byte_off;
  if (ALIGNED || aligned_to(base, 4 * W)) {
    if constexpr (W == 1) {
      st_stream<uint32_t>(p, w[0]);
    } else {
      typename Words<W>::T v;
#pragma unroll
      for (int k = 0; k < W; ++k) v[k] = w[k];
      st_stream<typename Words<W>::T>(p, v);
    }
  } else if (ES == 4 || aligned_to(base, 4)) {
#pragma unroll
    for (int k = 0; k < W; ++k) st_stream<uint32_t>(p + 4 * k, w[k]);
  } else {
#pragma unroll
    for (int k = 0; k < W; ++k) {
      st_stream<uint16_t>(p + 4 * k, (uint16_t)(w[k] & 0xFFFFu));
      st_stream<uint16_t>(p + 4 * k + 2, (uint16_t)(w[k] >> 16));
    }
  }
}

// The same for the vector position of a tile: `tile` is wave-uniform, `off` (< 2^31) this
// lane's byte offset inside it.  Aligned vectors are written through, the rest as above.
template <int W, int ES, bool ALIGNED = false>
__device__ __forceinline__ void st_tile_words(char* tile, uint32_t off, const uint32_t* w) {
  if (ALIGNED || aligned_to(tile, 4 * W))
    st_through<W>(wave_uniform(tile), off, 0x7FFFFFFFu, w);
  else
    st_words<W, ES, false>(tile, off, w);
}

// One element as fp32 / from fp32.
template <int DT>
__device__ __forceinline__ float ld_elem(const char* base, size_t e) {
  if constexpr (DT == kF32) return ld_stream<float>(base + 4 * e);
  return lo16<DT>((uint32_t)ld_stream<uint16_t>(base + 2 * e));
}
template <int DT>
__device__ __forceinline__ void st_elem(char* base, size_t e, float v) {
  if constexpr (DT == kF32)
    st_stream<float>(base + 4 * e, v);
  else
    st_stream<uint16_t>(base + 2 * e, to16<DT>(v));
}

}  // namespace pccl
