// Device-side helpers for the gfx950 kernels: 128-bit streaming loads/stores with an
// element-wise fallback for unaligned buffers, and bf16 <-> fp32 conversion.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pccl {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kBlock = 256;  // threads per block of the streaming kernels (4 wavefronts)

// ---- bf16 ----------------------------------------------------------------------------
// A 32-bit word holds two bf16: element 2k in the low half, 2k+1 in the high half.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp32 pair -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ uint16_t to_bf16(float x) { return (uint16_t)(pack_bf16(x, 0.0f) & 0xFFFFu); }
// Value of x after a trip through bf16 storage.
__device__ __forceinline__ float round_through_bf16(float x) { return bf16_lo(pack_bf16(x, 0.0f)); }

// ---- streaming global access ------------------------------------------------------------
// `base` is wave-uniform, `byte_off` is per lane.  Data is touched once, so loads and stores
// carry the non-temporal hint.

template <typename T>
__device__ __forceinline__ T ld_stream(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
}
template <typename T>
__device__ __forceinline__ void st_stream(void* p, T v) {
  __builtin_nontemporal_store(v, reinterpret_cast<T*>(p));
}

__device__ __forceinline__ bool aligned_to(const void* p, uintptr_t a) {
  return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

// 16 bytes from base+byte_off; ES = element size the buffer is guaranteed aligned to (2 or 4).
template <int ES>
__device__ __forceinline__ u32x4 ld16(const char* base, size_t byte_off) {
  const char* p = base + byte_off;
  if (aligned_to(base, 16)) return ld_stream<u32x4>(p);
  u32x4 v;
  if (ES == 4 || aligned_to(base, 4)) {
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = ld_stream<uint32_t>(p + 4 * k);
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      uint32_t lo = ld_stream<uint16_t>(p + 4 * k);
      uint32_t hi = ld_stream<uint16_t>(p + 4 * k + 2);
      v[k] = lo | (hi << 16);
    }
  }
  return v;
}

template <int ES>
__device__ __forceinline__ void st16(char* base, size_t byte_off, u32x4 v) {
  char* p = base + byte_off;
  if (aligned_to(base, 16)) {
    st_stream<u32x4>(p, v);
    return;
  }
  if (ES == 4 || aligned_to(base, 4)) {
#pragma unroll
    for (int k = 0; k < 4; ++k) st_stream<uint32_t>(p + 4 * k, v[k]);
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      st_stream<uint16_t>(p + 4 * k, (uint16_t)(v[k] & 0xFFFFu));
      st_stream<uint16_t>(p + 4 * k + 2, (uint16_t)(v[k] >> 16));
    }
  }
}

// 8 bytes (two words) of bf16 output from an fp32-input vector.
__device__ __forceinline__ void st8_bf16(char* base, size_t byte_off, u32x2 v) {
  char* p = base + byte_off;
  if (aligned_to(base, 8)) {
    st_stream<u32x2>(p, v);
  } else if (aligned_to(base, 4)) {
    st_stream<uint32_t>(p, v[0]);
    st_stream<uint32_t>(p + 4, v[1]);
  } else {
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      st_stream<uint16_t>(p + 4 * k, (uint16_t)(v[k] & 0xFFFFu));
      st_stream<uint16_t>(p + 4 * k + 2, (uint16_t)(v[k] >> 16));
    }
  }
}

// One element as fp32 / from fp32.
template <bool BF16>
__device__ __forceinline__ float ld_elem(const char* base, size_t e) {
  if (BF16) return __uint_as_float((uint32_t)ld_stream<uint16_t>(base + 2 * e) << 16);
  return ld_stream<float>(base + 4 * e);
}
template <bool BF16>
__device__ __forceinline__ void st_elem(char* base, size_t e, float v) {
  if (BF16)
    st_stream<uint16_t>(base + 2 * e, to_bf16(v));
  else
    st_stream<float>(base + 4 * e, v);
}

}  // namespace pccl
