// Loads from global memory straight into LDS, and the wait for them (device helpers shared by the kernels that stream
// operands or factor words into LDS without passing through registers).
#pragma once
#include <cstdint>

#include <hip/hip_runtime.h>

namespace lrbi {

// 16 bytes per lane from global memory (uniform base + per-lane byte offset) straight into LDS at
// (uniform byte address lds_addr) + 16 * lane.  The compiler does not see the LDS write: the kernel waits for
// it with wait_loads() before the barrier that hands the stage over.  lds_addr must be the same in all lanes (the
// first lane's value is taken).
__device__ __forceinline__ void load_to_lds16(uint32_t lds_addr, const void *gbase, uint32_t voff)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(__builtin_amdgcn_readfirstlane((int)lds_addr)), "v"(voff), "s"(gbase)
                 : "memory");
#endif
}
// the same with 4 bytes per lane: lands at lds_addr + 4 * lane
__device__ __forceinline__ void load_to_lds4(uint32_t lds_addr, const void *gbase, uint32_t voff)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :
                 : "s"(__builtin_amdgcn_readfirstlane((int)lds_addr)), "v"(voff), "s"(gbase)
                 : "memory");
#endif
}
template <int N> __device__ __forceinline__ void wait_loads()
{
#if defined(__HIP_DEVICE_COMPILE__)
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
#endif
}

// byte address of an LDS object, as the load-to-LDS instructions take it
__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char *)p;
}

} // namespace lrbi
