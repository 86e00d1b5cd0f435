// LDS-DMA loads for gfx950 (global -> LDS without a register stop) and the explicit
// vector-memory wait that goes with them.  The loads are issued through inline asm: the
// compiler does not see them, so it neither waits for them before LDS reads (which would
// serialise a software pipeline) nor counts them; the kernels that use them place their own
// s_waitcnt vmcnt(n) and a barrier before the data is read.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mquant {

typedef const void __attribute__((address_space(1))) *global_ptr_t;
typedef void __attribute__((address_space(3))) *lds_ptr_t;

// 16 bytes per lane, global -> LDS; LDS address = wave-uniform base + lane * 16.
__device__ __forceinline__ void lds_dma16(const uint8_t *gsrc, uint8_t *lds_wave_base)
{
    const uint32_t m0v =
        __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
            (lds_ptr_t)lds_wave_base)));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(m0v), "v"(gsrc)
                 : "memory", "m0");
}

// The same with a wave-uniform 64-bit base (kept in scalar registers) plus a 32-bit byte offset
// per lane, and the LDS destination given as a byte address inside the work-group's LDS.
__device__ __forceinline__ void lds_dma16_uniform_base(const uint8_t *base_uniform, uint32_t lane_offset,
                                                       uint32_t lds_wave_base)
{
    const uint64_t b = reinterpret_cast<uint64_t>(base_uniform);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b >> 32));
    const uint64_t sb = (static_cast<uint64_t>(hi) << 32) | lo;
    const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_wave_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(m0v), "v"(lane_offset), "s"(sb)
                 : "memory", "m0");
}

// LDS byte address of a __shared__ object.
template <typename T>
__device__ __forceinline__ uint32_t lds_address(T *shared_object)
{
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)shared_object));
}

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt in bits [3:0] and [15:14]).
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

}  // namespace mquant
