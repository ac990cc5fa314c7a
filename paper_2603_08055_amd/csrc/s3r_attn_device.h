// Device-side helpers of the bf16 MFMA attention kernels (selection and dense): the LDS-direct load,
// explicit vmcnt waits, exchanges between the two halves of a wave, and the constants of the 64-key unit.
#pragma once
#include "s3r_device.h"

namespace s3r {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr float kRescaleSlack = 8.0f;
constexpr int kUnitKeys = 64;
constexpr int kUnitElems = kUnitKeys * 64;  // bf16 elements of one K (or V) unit: 8 KiB

__device__ __forceinline__ float max_with_other_half(float x)
{
    // v_permlane32_swap exchanges the two half-waves: one VALU instruction, no LDS traffic
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float sum_with_other_half(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// One LDS-direct load: 64 lanes x 16 bytes from `src` (per-lane address) to LDS byte address
// `lds_byte` (wave-uniform) + 16 * lane.  Counted by vmcnt like any vector memory load.
__device__ __forceinline__ void lds_dma_16(const void *src, unsigned lds_byte)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_byte)
                 : "memory", "m0");
}

// Four consecutive 1 KiB chunks of a contiguous run with a wave-uniform start address: lane L's 16 bytes of chunk
// c come from base + voff + c KiB (voff = 16 L, or 16 L + 4096 for the second half of an 8 KiB run: the
// constant offset of the instruction reaches 4095 bytes) and land at LDS byte lds_byte + c KiB + 16 L: the
// instruction's constant offset moves the LDS address along with the global one, so M0 is set once.
__device__ __forceinline__ void lds_dma_16_x4(const void *base, unsigned voff, unsigned lds_byte)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %0, %1\n\t"
                 "global_load_lds_dwordx4 %0, %1 offset:1024\n\t"
                 "global_load_lds_dwordx4 %0, %1 offset:2048\n\t"
                 "global_load_lds_dwordx4 %0, %1 offset:3072"
                 ::"v"(voff), "s"(base), "s"(lds_byte)
                 : "memory", "m0");
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

}  // namespace s3r
