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

// 16-byte buffer store with the uniform offset in an SGPR.  After a store of more than 8 bytes per lane the vector ALU
// must not overwrite the data registers in the very next cycles; the compiler inserts that wait state for global
// stores and for buffer stores with an immediate uniform offset, but not for buffer stores whose uniform offset sits in
// a register.  On gfx950 that form needs it too (seen with the accumulators of the activation kernel: the first data
// register came out, in the last four lanes of every row of 16, with the value the next instruction had written
// there), so the wait states follow the store here and nothing is scheduled in between.
typedef uint32_t buffer_u32x4 __attribute__((ext_vector_type(4)));
template <int AUX>
__device__ __forceinline__ void buffer_store_b128(buffer_u32x4 v, __amdgpu_buffer_rsrc_t rs, int voffset, int soffset) {
    __builtin_amdgcn_raw_buffer_store_b128(v, rs, voffset, soffset, AUX);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 3");
    __builtin_amdgcn_sched_barrier(0);
}

}  // namespace svdq
