// Raw buffer descriptors for the kernels' global memory traffic (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace svdq {

// A raw buffer descriptor over [base, base + bytes): loads and stores take a per-thread byte offset in a VGPR
// and a uniform byte offset in an SGPR, so walking the K dimension costs scalar adds only, and accesses past the
// end return zero / are dropped instead of faulting.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, size_t bytes) {
    const uint32_t n = bytes > 0xffffffffull ? 0xffffffffu : (uint32_t)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)n, 0x00020000);
}

}  // namespace svdq
