// Shared device helpers of the matrix-core kernels: MFMA wrappers, output rounding, the mask
// select on packed 16-bit values, the transposing LDS read, and the panel geometry.
#pragma once
#include <type_traits>
#include <utility>

#include "lrbi_internal.hpp"

namespace lrbi {

static constexpr int BK = 64; // columns of W (reduction steps) per slab

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <typename F, int... Is> __device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct F16Tag {};
struct BF16Tag {};

__device__ __forceinline__ f32x16 mfma_32x32x16(F16Tag, uint4 a, uint4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                  0, 0);
}
__device__ __forceinline__ f32x16 mfma_32x32x16(BF16Tag, uint4 a, uint4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                   0, 0, 0);
}

// fp32 -> storage dtype, round to nearest even
__device__ __forceinline__ uint16_t cvt_store(F16Tag, float v)
{
    return __builtin_bit_cast(uint16_t, (_Float16)v);
}
__device__ __forceinline__ uint16_t cvt_store(BF16Tag, float v)
{
    uint32_t u = __builtin_bit_cast(uint32_t, v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u); // quiet NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Zero the 16-bit halves of w whose mask bit is clear.  `pair` holds 0 or 1 in each half; a packed
// 16-bit integer multiply by 0 / 1 is an exact select on the bit pattern (no floating-point
// arithmetic touches the value, so NaN and Inf under a 0 bit disappear).
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t select2(uint32_t w, uint32_t pair)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2, w) * __builtin_bit_cast(u16x2, pair));
}
// 16-byte register piece as a native vector (kept in registers by construction; an array of
// class-type vectors indexed by pipeline stage was demoted to private memory by the compiler)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4 apply_mask8(u32x4 w, uint32_t bits8)
{
    const uint32_t y = bits8 | (bits8 << 15);
    u32x4 o;
    o.x = select2(w.x, y & 0x00010001u);
    o.y = select2(w.y, (y >> 2) & 0x00010001u);
    o.z = select2(w.z, (y >> 4) & 0x00010001u);
    o.w = select2(w.w, (y >> 6) & 0x00010001u);
    return o;
}
__device__ __forceinline__ uint4 apply_mask8(uint4 w, uint32_t bits8)
{
    // y holds bit j of bits8 at positions j and j + 15: (y >> 2q) & 0x00010001 = (b_2q, b_2q+1) per half
    const uint32_t y = bits8 | (bits8 << 15);
    w.x = select2(w.x, y & 0x00010001u);
    w.y = select2(w.y, (y >> 2) & 0x00010001u);
    w.z = select2(w.z, (y >> 4) & 0x00010001u);
    w.w = select2(w.w, (y >> 6) & 0x00010001u);
    return w;
}

typedef __attribute__((ext_vector_type(4))) short s16x4;

// 4(k) x 16(n) block of 16-bit values -> lane d of each 16-lane group gets column d, rows 0..3.
// Lane s of the group passes the address of row s / 4, columns 4 * (s % 4) .. + 3.
__device__ __forceinline__ uint2 lds_read_tr16(const uint16_t *p)
{
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(p));
    return __builtin_bit_cast(uint2, v);
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x2 lds_read_tr16_v(const uint16_t *p)
{
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(p));
    return __builtin_bit_cast(u32x2, v);
}
__device__ __forceinline__ f32x16 mfma_32x32x16(F16Tag, u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                  0, 0);
}
__device__ __forceinline__ f32x16 mfma_32x32x16(BF16Tag, u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                   0, 0, 0);
}

static constexpr int PW = 512;           // panel width in columns
static constexpr int PANEL_SLABS = PW / BK;
static constexpr int PANEL_WORDS = PW / 32;
static constexpr int PANEL_UNITS = PW / 128; // 128-column units; each lies inside one tile
static constexpr int FAST_MAX_K = 64;


} // namespace lrbi
