// Direct access to the workgroup's LDS by byte offset, for kernels that compute LDS addresses with
// integer instructions (the flat-pointer form would add the segment base to every address).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dcpq {

typedef int lds_v4i __attribute__((ext_vector_type(4)));

// Byte offset within the workgroup's LDS of an object in __shared__ memory.
__device__ inline uint32_t lds_offset_of(const void *p)
{
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const uint8_t *)p));
}

// 16 bytes at LDS byte offset `off` (16-byte aligned): one ds_read_b128.
__device__ inline lds_v4i lds_read_v4i(uint32_t off)
{
    typedef const lds_v4i __attribute__((address_space(3))) *ptr_t;
    return *reinterpret_cast<ptr_t>(static_cast<uintptr_t>(off));
}

}  // namespace dcpq
