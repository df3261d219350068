// Opt-in address checks for the C ABI (environment PCCL_CHECK_POINTERS): every entry point
// takes raw device pointers, and a kernel given a host pointer or a range longer than its
// allocation takes a memory fault that can cost the whole process.  With the variable set the
// host asks the HIP runtime, before a launch, whether each range lies inside one allocation a
// kernel can reach.  Off by default: a query costs about a microsecond per range.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>

#include "../../include/pccl_local.h"

namespace pccl {

// 0 = off, 1 = ranges the host can see, 2 = also pointer arrays and descriptor tables that
// live in device memory (copied back on the caller's stream, which is then synchronised).
int address_check_level();

// PCCL_OK when [p, p + bytes) lies inside one allocation that kernels of the current device
// can address (device, managed or pinned host memory); bytes == 0 always passes.
pccl_status_t check_range(const void* p, size_t bytes);

// A device-resident array of n pointers: its own range, and at level 2 every entry e as the
// range [entry + offset_bytes, + bytes_each); entry `skip` (or -1) is never dereferenced by
// the kernel and is not looked at.
pccl_status_t check_pointer_table(const void* const* d_table, size_t n, size_t offset_bytes,
                                  size_t bytes_each, long long skip, int level, hipStream_t st);

// A device-resident descriptor table with a host mirror: its own range, and at level 2 that
// the device copy equals the mirror byte for byte (PCCL_ERR_INVALID otherwise).
pccl_status_t check_descriptor_table(const void* d_table, const void* h_table, size_t bytes, int level,
                                     hipStream_t st);

}  // namespace pccl
