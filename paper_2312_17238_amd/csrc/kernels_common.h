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

__device__ __forceinline__ double bpermute_d(double v, int src_lane)
{
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_ds_bpermute(src_lane * 4, (int)(b & 0xffffffffll));
    const int hi = __builtin_amdgcn_ds_bpermute(src_lane * 4, (int)(b >> 32));
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// fp64 sums of N values per lane over the 64 lanes, all at once.  A butterfly over one value costs the same six
// exchanges whatever the lane holds; here, in each of the first log2(N) stages a lane GIVES half of what it still
// holds to its partner and adds the partner's other half to the half it keeps, so the values in flight halve from
// stage to stage (N-1 exchanges in all instead of 6 N); the remaining stages are plain butterflies on v[0].
// Which half a lane keeps is decided by the lane bit that the stage's partner differs in: stage 0 pairs lane i with
// 7-i of its group of eight (bit 2), then i^1 (bit 0), i^2 (bit 1), i+8 within the row of 16 (bit 3), i^16 (bit 4),
// i^32 (bit 5).  Afterwards v[0] of every lane is the total of value wave_sum_index<N>(lane); lanes 0..N-1 cover
// all N.  Fixed order, so deterministic.
template <int N>
__device__ __forceinline__ int wave_sum_index(int lane)
{
    constexpr int BIT[6] = {2, 0, 1, 3, 4, 5};
    int idx = 0, n = N;
#pragma unroll
    for (int s = 0; s < 6; ++s)
        if (n > 1) { n >>= 1; idx += ((lane >> BIT[s]) & 1) * n; }
    return idx;
}

template <int STAGE>
__device__ __forceinline__ double wave_sum_exchange(double give, int lane)
{
    if constexpr (STAGE == 0) return dpp_d<0x141>(give);                  // row_half_mirror
    else if constexpr (STAGE == 1) return dpp_d<0xB1>(give);              // quad_perm [1,0,3,2]
    else if constexpr (STAGE == 2) return dpp_d<0x4E>(give);              // quad_perm [2,3,0,1]
    else if constexpr (STAGE == 3) return dpp_d<0x128>(give);             // row_ror:8
    else if constexpr (STAGE == 4) return bpermute_d(give, lane ^ 16);
    else return bpermute_d(give, lane ^ 32);
}

template <int STAGE, int HELD, int M>
__device__ __forceinline__ void wave_sum_stage(double (&v)[M], int lane)
{
    if constexpr (STAGE < 6) {
        constexpr int BIT[6] = {2, 0, 1, 3, 4, 5};
        if constexpr (HELD > 1) {
            constexpr int H = HELD / 2;
            const bool up = (lane >> BIT[STAGE]) & 1;
#pragma unroll
            for (int j = 0; j < H; ++j) {
                const double keep = up ? v[j + H] : v[j], give = up ? v[j] : v[j + H];
                v[j] = keep + wave_sum_exchange<STAGE>(give, lane);
            }
            wave_sum_stage<STAGE + 1, H, M>(v, lane);
        } else {
            v[0] += wave_sum_exchange<STAGE>(v[0], lane);
            wave_sum_stage<STAGE + 1, 1, M>(v, lane);
        }
    }
}

template <int N, int M>
__device__ __forceinline__ void wave_sum_many_f64(double (&v)[M], int lane)
{
    static_assert((N == 8 || N == 16 || N == 32) && N <= M, "8, 16 or 32 of the array's values");
    wave_sum_stage<0, N, M>(v, lane);
}

// Round-to-nearest-even conversion of a double to binary16 as if done in one step.  Two hardware conversions
// (fp64 -> fp32 -> fp16) would round twice; rounding the first one TO ODD instead (truncate toward zero, then set the
// last bit if anything was lost) keeps in fp32's 24 bits everything the second, nearest-even rounding to 11 bits or
// fewer needs.  The truncation is recovered from the nearest-even conversion: where that one moved away from zero,
// the neighbour toward zero is the fp32 pattern minus one.  NaN maps to a quiet NaN.
__device__ __forceinline__ uint16_t f64_to_f16_rne(double d)
{
    const float t = (float)d;
    const double r = (double)t;
    uint32_t tb = __builtin_bit_cast(uint32_t, t);
    if (r != d) {
        if (__builtin_fabs(r) > __builtin_fabs(d)) tb -= 1u;
        tb |= 1u;
    }
    const uint16_t h = __builtin_bit_cast(uint16_t, (_Float16)__builtin_bit_cast(float, tb));
    return d != d ? (uint16_t)(((uint64_t)__double_as_longlong(d) >> 48) & 0x8000u) | 0x7e00u : h;
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
