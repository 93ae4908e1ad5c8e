// Fixed device array of the allocation-free entry point (see static_scratch.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace ens {

// 32 MiB per GPU: per-member logits of one request (members x n x classes fp32) behind a
// 4 KiB table of the members' logits pointers.
constexpr size_t STATIC_SCRATCH_BYTES = 32u << 20;
constexpr size_t STATIC_SCRATCH_TABLE_BYTES = 4096;

// Address and size of the array on the current device.  The address is resolved once per device
// and kept; no memory is allocated.
hipError_t static_scratch(void** ptr, size_t* bytes);

}  // namespace ens
