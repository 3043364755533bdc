// Device-side helpers for the gfx950 kernels: vector types, element conversion, tile addressing.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#include "ts_internal.h"

namespace ts {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;

// Read-only work lists and page tables are read through the constant address space: a load from
// a wave-uniform address then goes through the scalar cache (its own counter, out of order with
// respect to the vector-memory queue) even in kernels that also store to global memory.
#define TS_CONSTANT __attribute__((address_space(4)))
template <typename T>
__device__ __forceinline__ const T TS_CONSTANT* as_constant(const T* p)
{
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
    return (const T TS_CONSTANT*)p;
#pragma clang diagnostic pop
}

// An opaque copy of a value: whatever is derived from the copy is worked out where it is used.  The
// optimiser otherwise moves lane-index arithmetic and masks of rarely taken paths to the top of a kernel
// and keeps them in registers across its main loops.
__device__ __forceinline__ int opaque(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}
__device__ __forceinline__ int opaque_uniform(int v)
{
    asm volatile("" : "+s"(v));
    return v;
}

// Lanes l and l ^ 32 of a wave exchange through one register swap between the halves of the wave (no lane
// index register, no trip through the LDS crossbar): both results of the swap hold, in every lane, one
// of the two values of the lane pair.
__device__ __forceinline__ float pair32_max(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair32_sum(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// bf16 bits <-> float
__device__ __forceinline__ float bf16_bits_to_float(uint32_t h) { return __uint_as_float(h << 16); }

// round-to-nearest-even float -> bf16 bits (NaN kept quiet)
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// OCP e4m3 (bias 7, max 448, S.1111.111 = NaN, no inf) -> float, from the format definition.
__device__ __forceinline__ float e4m3_bits_to_float(uint32_t b)
{
    uint32_t mag = b & 0x7fu;
    // exponent/mantissa moved into fp32 position give value * 2^-120; subnormals come out
    // right because the product below is exact.
    float v = __uint_as_float(mag << 20) * 0x1p120f;
    if (mag == 0x7fu) v = __uint_as_float(0x7fc00000u);
    return (b & 0x80u) ? -v : v;
}

// float -> e4m3 bits: nearest-even, saturating to +-448 (inf too), NaN -> S.1111.111
__device__ __forceinline__ uint32_t float_to_e4m3_bits(float y)
{
    uint32_t u = __float_as_uint(y);
    uint32_t sign = (u >> 24) & 0x80u;
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return sign | 0x7fu;
    if (a >= 0x43e00000u) return sign | 0x7eu;             // |y| >= 448
    if (a < 0x3c800000u) {                                 // |y| < 2^-6: spacing 2^-9
        float q = __builtin_rintf(__uint_as_float(a) * 512.0f);
        return sign | (uint32_t)(int)q;                    // q == 8 is the first normal code
    }
    uint32_t r = (a + 0x7ffffu + ((a >> 20) & 1u)) >> 20;  // keep 3 mantissa bits, ties to even
    return sign | (r - (120u << 3));                       // rebias 127 -> 7
}

// ---- cache tile addressing (element offsets inside one cache buffer) ---------------------------
// tiles ordered [page][kv_head]; K tile [D/x][16][x], V tile [D][16]; x = 16 bytes / element size.

template <int ES> struct chunk_elems { static constexpr int value = 16 / ES; };

__device__ __forceinline__ int64_t tile_elem_base(int64_t page, int Hkv, int g, int D)
{
    return (page * Hkv + g) * (int64_t)(kPage * D);
}

// Stores of data this pass does not read again (new cache entries, outputs): the non-temporal hint
// sends them on to memory instead of leaving partially written lines in the L2, whose write-back in
// the middle of the decode scan was measured to cost ten times its byte share.
__device__ __forceinline__ void store_nt(void* p, uint4 v)
{
    __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, (u32x4*)p);
}
__device__ __forceinline__ uint4 load_nt4(const void* p)
{
    const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 load_nt2(const void* p)
{
    const u32x2 v = __builtin_nontemporal_load((const u32x2*)p);
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ void store_nt(void* p, uint2 v) { __builtin_nontemporal_store(u32x2{v.x, v.y}, (u32x2*)p); }

}  // namespace ts
