// Host-only: address checks behind PCCL_CHECK_POINTERS (see address_check.h).
#include "address_check.h"

#include "knobs.h"

#include <cstdint>
#include <cstring>
#include <vector>

namespace pccl {

int address_check_level() { return knobs().check_pointers; }

pccl_status_t check_range(const void* p, size_t bytes) {
  if (bytes == 0) return PCCL_OK;
  if (p == nullptr) return PCCL_ERR_NULL;
  hipPointerAttribute_t attr;
  std::memset(&attr, 0, sizeof(attr));
  hipError_t e = hipPointerGetAttributes(&attr, p);
  if (e != hipSuccess) {
    (void)hipGetLastError();  // a failed query must not be reported by the next launch
    return PCCL_ERR_ADDRESS;
  }
  if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged &&
      attr.type != hipMemoryTypeHost)
    return PCCL_ERR_ADDRESS;
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  e = hipMemGetAddressRange(&base, &size, const_cast<void*>(p));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return PCCL_ERR_ADDRESS;
  }
  const uintptr_t lo = reinterpret_cast<uintptr_t>(base), x = reinterpret_cast<uintptr_t>(p);
  if (x < lo || x - lo > size || bytes > size - (x - lo)) return PCCL_ERR_ADDRESS;
  return PCCL_OK;
}

namespace {

// device -> host on the caller's stream, then wait for it
bool fetch(void* host, const void* dev, size_t bytes, hipStream_t st) {
  if (hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return true;
}

}  // namespace

pccl_status_t check_pointer_table(const void* const* d_table, size_t n, size_t offset_bytes,
                                  size_t bytes_each, long long skip, int level, hipStream_t st) {
  if (n == 0) return PCCL_OK;
  if (n > SIZE_MAX / sizeof(void*)) return PCCL_ERR_INVALID;
  if (pccl_status_t s = check_range(d_table, n * sizeof(void*))) return s;
  if (level < 2) return PCCL_OK;
  std::vector<const void*> host(n);
  if (!fetch(host.data(), d_table, n * sizeof(void*), st)) return PCCL_ERR_HIP;
  for (size_t i = 0; i < n; ++i) {
    if ((long long)i == skip) continue;
    if (host[i] == nullptr) return PCCL_ERR_NULL;
    if (pccl_status_t s = check_range(reinterpret_cast<const char*>(host[i]) + offset_bytes, bytes_each))
      return s;
  }
  return PCCL_OK;
}

pccl_status_t check_descriptor_table(const void* d_table, const void* h_table, size_t bytes, int level,
                                     hipStream_t st) {
  if (bytes == 0) return PCCL_OK;
  if (pccl_status_t s = check_range(d_table, bytes)) return s;
  if (level < 2) return PCCL_OK;
  std::vector<char> host(bytes);
  if (!fetch(host.data(), d_table, bytes, st)) return PCCL_ERR_HIP;
  return std::memcmp(host.data(), h_table, bytes) == 0 ? PCCL_OK : PCCL_ERR_INVALID;
}

}  // namespace pccl
