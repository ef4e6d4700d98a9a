// Shared device helpers: DPP wave reductions, exact fp64 -> fp16 rounding, streaming loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe {

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));

constexpr int WAVE = 64;
constexpr int MAX_ENTRIES = 16;   // (expert, token-chunk) work entries per launch
constexpr int MAX_NT = 4;         // tokens per entry

// ---------------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------------

__device__ __forceinline__ h2_t as_h2(uint32_t v) { return __builtin_bit_cast(h2_t, v); }
__device__ __forceinline__ float lo_half(uint32_t v) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(v & 0xffff)); }
__device__ __forceinline__ float hi_half(uint32_t v) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(v >> 16)); }
__device__ __forceinline__ double half_bits_to_f64(uint16_t v) { return (double)__builtin_bit_cast(_Float16, v); }

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_masked_f(float v)
{
    // lanes of rows outside ROW_MASK receive 0
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false));
}

// Sum over the 64 lanes; the total is valid in lane 63 only.  Fixed order, so deterministic.
__device__ __forceinline__ float wave_sum_l63(float v)
{
    v += dpp_f<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f<0x141>(v);   // row_half_mirror
    v += dpp_f<0x140>(v);   // row_mirror: every lane of a 16-lane row now holds the row's sum
    v += dpp_masked_f<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_masked_f<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

template <int CTRL>
__device__ __forceinline__ double dpp_d(double v)
{
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xf, 0xf, true);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

__device__ __forceinline__ double readlane_d(double v, int lane)
{
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffll), lane);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// fp64 sum over the 64 lanes, total in every lane
__device__ __forceinline__ double wave_sum_f64(double v)
{
    v += dpp_d<0xB1>(v);
    v += dpp_d<0x4E>(v);
    v += dpp_d<0x141>(v);
    v += dpp_d<0x140>(v);
    return (readlane_d(v, 0) + readlane_d(v, 16)) + (readlane_d(v, 32) + readlane_d(v, 48));
}

// Round-to-nearest-even conversion of a double straight to binary16 (no intermediate fp32 rounding,
// which could double-round).  NaN maps to a quiet NaN.
__device__ __forceinline__ uint16_t f64_to_f16_rne(double d)
{
    const uint64_t b = (uint64_t)__double_as_longlong(d);
    const uint16_t sign = (uint16_t)((b >> 48) & 0x8000u);
    const int ex = (int)((b >> 52) & 0x7ff);
    const uint64_t man = b & 0xFFFFFFFFFFFFFull;
    if (ex == 0x7ff) return sign | (man ? 0x7e00u : 0x7c00u);
    if (ex == 0) return sign;                        // zero or a double subnormal: far below half range
    const int e = ex - 1023;
    if (e > 15) return sign | 0x7c00u;
    const uint64_t m = man | (1ull << 52);
    int shift = 42;
    uint32_t base = (uint32_t)(e + 15) << 10;
    if (e < -14) {                                   // half subnormal
        shift = 42 + (-14 - e);
        base = 0;
        if (shift > 63) return sign;
    }
    uint64_t q = m >> shift;
    const uint64_t rem = m & ((1ull << shift) - 1), halfway = 1ull << (shift - 1);
    if (rem > halfway || (rem == halfway && (q & 1))) ++q;
    // normal: q is in [1024, 2048]; adding q-1024 to the exponent field carries correctly on 2048.
    // subnormal: q is in [0, 1024]; 1024 carries into the smallest normal.
    const uint32_t r = (e < -14) ? (uint32_t)q : base + (uint32_t)(q - 1024);
    return sign | (uint16_t)(r > 0x7c00u ? 0x7c00u : r);
}

// Weight loads.  Every weight byte is used exactly once per step, so the loads carry the streaming
// (non-temporal) hint: they need not displace the activations and gate matrices from L2.
#ifndef MOE_NT_LOADS
#define MOE_NT_LOADS 1
#endif
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 ldw4(const void *p, int idx)
{
#if MOE_NT_LOADS
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p) + idx);
#else
    const u32x4_t v = reinterpret_cast<const u32x4_t *>(p)[idx];
#endif
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 ldw2(const void *p, int idx)
{
#if MOE_NT_LOADS
    const u32x2_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(p) + idx);
#else
    const u32x2_t v = reinterpret_cast<const u32x2_t *>(p)[idx];
#endif
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ uint32_t ldw1(const void *p, int idx)
{
#if MOE_NT_LOADS
    return __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p) + idx);
#else
    return reinterpret_cast<const uint32_t *>(p)[idx];
#endif
}

// silu(u) * v; the reciprocal is the hardware approximation (1 ulp), far below the fp16 rounding that follows
__device__ __forceinline__ float silu_mul(float u, float v) { return u * __builtin_amdgcn_rcpf(1.f + __expf(-u)) * v; }

// (a & mask) | k in one instruction.  gfx9 VOP3 encodings take no 32-bit literals and at most one scalar
// operand, so the compiler splits this into v_and + v_or with literals; with the mask in an SGPR and k in a
// VGPR it is a single v_and_or_b32.
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t k)
{
    uint32_t d;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "s"(mask), "v"(k));
    return d;
}

// wave-uniform value as a scalar, so that addresses derived from it are computed on the scalar unit
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

}  // namespace moe
