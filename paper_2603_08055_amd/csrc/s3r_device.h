// Device-side helpers shared by the gfx950 kernels: vector types for the bf16 MFMA
// instructions, bf16 conversion, the operand-tile layouts, and cross-half-wave exchange.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s3r {

typedef __bf16 bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

constexpr int kHeadDim = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ---- operand tiles ---------------------------------------------------------------------------
// A "row tile" holds 32 rows x 64 columns of bf16 (4 KiB) in the order the 32x32x16 MFMA wants
// an operand whose contraction index is the column: chunk (s, lane) = 8 consecutive columns
// 16 s + 8 (lane / 32) .. + 7 of row (lane % 32), stored at element offset ((s * 64) + lane) * 8.
// One ds_read_b128 / global 16-byte load per lane fetches one MFMA operand, conflict-free.
constexpr int kRowTileElems = 32 * 64;

__device__ __forceinline__ int row_tile_chunk_offset(int row_in_tile, int col_chunk /*0..7*/)
{
    const int s = col_chunk >> 1, g = col_chunk & 1;
    return ((s * 64) + g * 32 + row_in_tile) * 8;
}

// A "transposed tile" holds 32 rows (keys) x 64 columns (channels) of bf16 in the order the MFMA
// wants for P.V with the contraction over keys: chunk (u, dt, lane), u = 0..1, dt = 0..1, is the
// 8 keys  16 u + 8 (i / 4) + 4 (lane / 32) + (i % 4),  i = 0..7,  of channel 32 dt + lane % 32,
// at element offset ((u * 2 + dt) * 64 + lane) * 8.  The key order matches the registers in which
// a 32x32 MFMA leaves the transposed score tile, so probabilities feed the next MFMA unshuffled.
__device__ __forceinline__ int tr_tile_key(int u, int lane, int i)
{
    return 16 * u + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
}

// Row index inside a 32x32 MFMA result held by (lane, register r).
__device__ __forceinline__ int acc_row(int lane, int r) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

__device__ __forceinline__ float bf16_to_float(bf16_t x) { return static_cast<float>(x); }
__device__ __forceinline__ bf16_t float_to_bf16(float x) { return static_cast<bf16_t>(x); }

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return static_cast<float>(x); }
template <typename T> __device__ __forceinline__ T from_float(float x);
template <> __device__ __forceinline__ float from_float<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float x) { return static_cast<bf16_t>(x); }

// Value held by the lane 32 positions away (wave64).
__device__ __forceinline__ float other_half(float x)
{
    return __shfl_xor(x, 32, 64);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Monotone map float -> uint32 (larger float <=> larger key); -0.0 is folded onto +0.0 first so
// that equal scores compare equal.  Keys of real numbers are never 0.
__device__ __forceinline__ uint32_t order_key(float x)
{
    x += 0.f;
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Inverse of order_key (the key of -inf maps back to -inf).
__device__ __forceinline__ float key_to_float(uint32_t key)
{
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// Number of set bits of `mask` below the calling lane.
__device__ __forceinline__ int lanes_below(unsigned long long mask)
{
    return __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(mask), 0u));
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also fences global memory, which
// makes the compiler drain every outstanding vector load and store (s_waitcnt vmcnt(0)) before the
// barrier; kernels that keep LDS-direct loads or fire-and-forget stores in flight across a barrier
// pace those themselves and use this one instead.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

}  // namespace s3r
