// Single-token expert FFN in one persistent launch: w1/w3 -> SiLU*mul -> grid barrier -> w2 -> combine
// -> residual.  At batch 1 the two GEMV launches are each only ~20 us long, so a fixed ~3.5 us of launch
// ramp and tail per kernel costs 15-25 % of HBM bandwidth; one launch with the HBM stream kept alive across
// the barrier (the first w2 rows are requested before waiting) pays it once, and the combine and residual
// need neither atomics nor a further kernel.
//
// Grid: one block of 16 waves per compute unit (all blocks resident at once, which the barrier needs).
// Phase 1: the grid's waves walk the (expert, row) pairs of w1/w3 exactly like k_w13.
// Phase 2: block b owns output rows [b*R, (b+1)*R); waves [e*CS, (e+1)*CS) own the column chunks of expert e.
#pragma once
#include "kernels_gemv.h"

namespace moe {

constexpr int FUSED_WAVES = 16;
constexpr uint32_t BARRIER_SPIN_LIMIT = 4000000;   // polls of ~100 ns: gives up after a fraction of a second

struct FusedArgs {
    const uint8_t *blob[2];         // the token's experts (n_exp of them)
    float w[2];                     // their combine weights
    int32_t n_exp;
    const uint16_t *h;              // [H] gate input of the token
    const uint16_t *x;              // [H] residual stream in
    uint16_t *x_out;                // [H]
    uint16_t *a;                    // [n_exp][F] scratch
    float *y;                       // [H] block output before the residual add (diagnostic copy)
    uint32_t *barrier;              // device counter, only ever incremented
    uint32_t barrier_target;        // value the counter reaches when every block of this launch has arrived
    uint32_t *error_flag;           // host-visible: set if the barrier gave up
    int32_t H, F, group;
    uint32_t stride13, meta13, stride2, meta2;
    uint64_t off_w2;
    int32_t rows_per_block;         // R
};

// All blocks of the grid meet here.  Bounded: a block that waits too long raises the error flag and goes
// on (its results are then invalid, which the host reports), so every wave always reaches the kernel's end.
__device__ __forceinline__ void grid_barrier(uint32_t *counter, uint32_t target, uint32_t *error_flag)
{
    __syncthreads();
    if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t spins = 0;
        while ((int32_t)(__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
            __builtin_amdgcn_s_sleep(4);
            if (++spins > BARRIER_SPIN_LIMIT) {
                __hip_atomic_store(error_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                break;
            }
        }
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

template <int BITS, int KCH, int G1, int G2>
__global__ __launch_bounds__(FUSED_WAVES *WAVE) void k_ffn_token(FusedArgs A)
{
    using F = Fmt<BITS>;
    __shared__ float red[2 * 8 * 64];                    // [expert][cs][row], rows_per_block <= 64
    const int lane = threadIdx.x & 63;
    const int wv = uniform(threadIdx.x >> 6);
    const int gw = uniform(blockIdx.x * FUSED_WAVES + wv), n_waves = gridDim.x * FUSED_WAVES;

    // ---------------- phase 1: a[e][r] = silu(W1_e h)[r] * (W3_e h)[r] ----------------
    {
        const int n_chunks = A.H / F::CODES;
        const RowGeom geo = row_geom<BITS>(A.meta13, A.H, A.group);
        int cidx[KCH];
        bool live[KCH];
#pragma unroll
        for (int k = 0; k < KCH; ++k) {
            live[k] = k * 64 + lane < n_chunks;
            cidx[k] = live[k] ? k * 64 + lane : 0;
        }
        struct RowPair { typename F::Row w1[KCH], w3[KCH]; };
        const int items = A.n_exp * A.F, last = items - 1;
        auto load_item = [&](RowPair &rb, int item) {
            const int e = item >= A.F ? 1 : 0, r = item - e * A.F;
            const uint8_t *r1 = A.blob[e] + (size_t)(2 * r) * A.stride13, *r3 = r1 + A.stride13;
#pragma unroll
            for (int k = 0; k < KCH; ++k) {
                F::load(rb.w1[k], r1, geo, cidx[k]);
                F::load(rb.w3[k], r3, geo, cidx[k]);
            }
        };
        const int iters = (items + n_waves - 1) / n_waves;
        RowPair ring[G1];
#pragma unroll
        for (int s = 0; s < G1; ++s) load_item(ring[s], min(gw + s * n_waves, last));
        typename F::Act hc[KCH];
#pragma unroll
        for (int k = 0; k < KCH; ++k) F::load_act(hc[k], A.h, cidx[k], live[k]);
        for (int it = 0; it < iters; it += G1) {
#pragma unroll
            for (int s = 0; s < G1; ++s) {
                const int item = gw + (it + s) * n_waves;
                float u = 0.f, v = 0.f;
#pragma unroll
                for (int k = 0; k < KCH; ++k) {
                    u += F::contrib(ring[s].w1[k], hc[k], live[k]);
                    v += F::contrib(ring[s].w3[k], hc[k], live[k]);
                }
                load_item(ring[s], min(item + G1 * n_waves, last));
                const float us = wave_sum_l63(u), vs = wave_sum_l63(v);
                if (lane == 63 && item < items) {
                    const _Float16 av = (_Float16)silu_mul(us, vs);
                    A.a[item] = __builtin_bit_cast(uint16_t, av);     // a is [n_exp][F], item = e*F + r
                }
            }
        }
    }

    // ---------------- phase 2: y[r] = sum_e w_e (W2_e a_e)[r];  x_out = fp16(x + y) ----------------
    const int n_chunks2 = A.F / F::CODES;
    const int CS = (n_chunks2 + 63) / 64;
    const int e2 = wv / CS, cs = wv - e2 * CS;
    const bool active = e2 < A.n_exp;
    const int c = cs * 64 + lane;
    const bool live2 = active && c < n_chunks2;
    const int cc = live2 ? c : 0;
    const RowGeom geo2 = row_geom<BITS>(A.meta2, A.F, A.group);
    const int R = A.rows_per_block;
    const int row0 = blockIdx.x * R;
    const int row_end = min(row0 + R, A.H);
    const int last2 = max(row_end - 1, 0);
    const uint8_t *base2 = A.blob[active ? e2 : 0] + A.off_w2;
    typename F::Row ring2[G2];
    // request the first rows of w2 before the barrier: they do not depend on a
#pragma unroll
    for (int s = 0; s < G2; ++s) F::load(ring2[s], base2 + (size_t)min(row0 + s, last2) * A.stride2, geo2, cc);

    grid_barrier(A.barrier, A.barrier_target, A.error_flag);

    typename F::Act ac;
    F::load_act(ac, A.a + (size_t)(active ? e2 : 0) * A.F, cc, live2);
    for (int rbase = row0; rbase < row_end; rbase += G2) {
#pragma unroll
        for (int s = 0; s < G2; ++s) {
            const int row = rbase + s;
            const float part = F::contrib(ring2[s], ac, live2);
            F::load(ring2[s], base2 + (size_t)min(row + G2, last2) * A.stride2, geo2, cc);
            const float p = wave_sum_l63(part);
            if (lane == 63 && active && row < row_end) red[(e2 * 8 + cs) * 64 + (row - row0)] = p;
        }
    }
    __syncthreads();
    const int rr = threadIdx.x;
    if (rr < row_end - row0) {
        float y = 0.f;
        for (int e = 0; e < A.n_exp; ++e) {
            float s = 0.f;
            for (int k = 0; k < CS; ++k) s += red[(e * 8 + k) * 64 + rr];
            y += A.w[e] * s;
        }
        const int row = row0 + rr;
        A.y[row] = y;
        const float v = (float)__builtin_bit_cast(_Float16, A.x[row]) + y;
        A.x_out[row] = __builtin_bit_cast(uint16_t, (_Float16)v);
    }
}

}  // namespace moe
