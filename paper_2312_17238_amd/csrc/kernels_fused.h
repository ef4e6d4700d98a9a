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
// 1 (default): after the grid barrier the activations a are read back with agent-scope loads, which no stale line in
// a die's L2 can serve -- correct by the memory model.  0: plain loads (a timing variant only: a block may then hit
// a line of a that its own die cached before the other dies' stores arrived).
#ifndef MOE_FUSED_COHERENT_A
#define MOE_FUSED_COHERENT_A 1
#endif


namespace moe {

constexpr int FUSED_WAVES = 16;
constexpr int FUSED_MAX_ITEMS = 64;                // (expert, row) pairs of w1/w3 per wave
constexpr uint32_t BARRIER_SPIN_LIMIT = 2000000;   // polls of ~200 ns: gives up after a fraction of a second

struct FusedArgs {
    const uint8_t *blob[2];         // the token's experts (n_exp of them)
    float w[2];                     // their combine weights
    int32_t a_row[2];               // row of the scratch a[.][F] each expert's activations live in
    int32_t n_exp;
    const uint16_t *h;              // [H] gate input of the token
    const uint16_t *x;              // [H] residual stream in
    uint16_t *x_out;                // [H]
    uint16_t *a;                    // [n_exp][F] scratch
    float *y;                       // [H] block output before the residual add (diagnostic copy)
    uint32_t *barrier;              // device flags, one per block: the epoch of the last launch the block arrived in
    uint32_t barrier_target;        // this launch's epoch (increases by one per launch)
    uint32_t *error_flag;           // host-visible: set if the barrier gave up
    int32_t H, F, group, scale_group;
    uint32_t stride13, meta13, stride2, meta2;
    uint64_t off_w2;
    int32_t rows_per_block;         // R
    // Device-side routing (k_w2_token only): expert e of the step is route_idx[e], its combine weight route_w[e], its
    // weights table[route_idx[e]], as the gate kernel of the same step left them.  Null: blob[] and w[] above.
    const int32_t *route_idx;
    const float *route_w;
    const uint8_t *table[16];
};

// All blocks of the grid meet here.  Bounded: a block that waits too long raises the error flag and goes
// on (its results are then invalid, which the host reports), so every wave always reaches the kernel's end.
//
// Visibility of the activations a across the barrier does not use agent-scope fences (on this multi-die part
// they write back and invalidate whole L2 slices, once per executing wave): a is written with agent-scope
// stores (write-through) and read back with agent-scope loads (no stale copy in a die's L2 can be hit); a
// wave only has to wait for its own stores to be acknowledged before its block arrives.
//
// The barrier itself avoids read-modify-write atomics (device-scope atomics are executed at the memory side
// and 256 of them on one address serialise for ~10 us): block b publishes flags[b] = epoch with one store,
// and every block polls all flags, one flag per thread, until none is behind the epoch.
__device__ __forceinline__ void grid_barrier(uint32_t *flags, uint32_t epoch, uint32_t *error_flag)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // this wave's stores are complete
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(flags + blockIdx.x, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (uint32_t spins = 0;; ++spins) {
        int ok = 1;
        for (uint32_t i = threadIdx.x; i < gridDim.x; i += blockDim.x)
            ok &= (int32_t)(__hip_atomic_load(flags + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch) >= 0;
        if (__syncthreads_and(ok)) break;
        if (spins > BARRIER_SPIN_LIMIT) {
            if (threadIdx.x == 0) __hip_atomic_store(error_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            break;
        }
        __builtin_amdgcn_s_sleep(2);
    }
}

// the fused kernel's own activation loader: the same Act as Fmt::load_act, read with agent-scope loads
template <int BITS>
__device__ __forceinline__ void load_act_coherent(typename Fmt<BITS>::Act &a, const uint16_t *vec, int c, bool live)
{
    constexpr int N8 = Fmt<BITS>::CODES / 4;              // 8-byte words per chunk
    __attribute__((aligned(16))) uint16_t tmp[Fmt<BITS>::CODES];
    const uint64_t *p = reinterpret_cast<const uint64_t *>(vec + (size_t)c * Fmt<BITS>::CODES);
#pragma unroll
    for (int i = 0; i < N8; ++i)
        reinterpret_cast<uint64_t *>(tmp)[i] = __hip_atomic_load(p + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    Fmt<BITS>::load_act(a, tmp, 0, live);
}

// y[r] = sum_e w_e (W2_e a_e)[r];  x_out = fp16(x + y), for the rows of this block.  Waves [e*CS, (e+1)*CS)
// own the column chunks of expert e; BARRIER: wait for the whole grid between requesting the first rows of
// w2 (which do not depend on a) and reading a.
template <int BITS, int G2, bool BARRIER>
__device__ __forceinline__ void token_w2_phase(const FusedArgs &A, float *red, int wv, int lane)
{
    using F = Fmt<BITS>;
    const int n_chunks2 = A.F / F::CODES;
    const int CS = (n_chunks2 + 63) / 64;
    const int e2 = wv / CS, cs = wv - e2 * CS;
    const bool active = e2 < A.n_exp;
    const int c = cs * 64 + lane;
    const bool live2 = active && c < n_chunks2;
    const int cc = live2 ? c : 0;
    const RowGeom geo2 = row_geom<BITS>(A.meta2, A.F, A.group, A.scale_group);
    const int R = A.rows_per_block;
    const int row0 = blockIdx.x * R;
    const int row_end = min(row0 + R, A.H);
    const int last2 = max(row_end - 1, 0);
    auto row_of = [&](int j) { return min(j, last2); };
    const uint8_t *blob2 = A.route_idx ? A.table[uniform(A.route_idx[active ? e2 : 0]) & 15] : A.blob[active ? e2 : 0];
    const uint8_t *base2 = blob2 + A.off_w2;
    typename F::Row ring2[G2];
#pragma unroll
    for (int s = 0; s < G2; ++s) F::load(ring2[s], base2 + (size_t)row_of(row0 + s) * A.stride2, geo2, cc);

    if (BARRIER) grid_barrier(A.barrier, A.barrier_target, A.error_flag);

    typename F::Act ac;
    // a written by an earlier launch is visible to plain loads; a written inside this launch by other dies is not
    if constexpr (BARRIER && MOE_FUSED_COHERENT_A) load_act_coherent<BITS>(ac, A.a + (size_t)A.a_row[active ? e2 : 0] * A.F, cc, live2);
    else F::load_act(ac, A.a + (size_t)A.a_row[active ? e2 : 0] * A.F, cc, live2);
    for (int rbase = row0; rbase < row_end; rbase += G2) {
#pragma unroll
        for (int s = 0; s < G2; ++s) {
            const int row = rbase + s;
            const float part = F::contrib(ring2[s], ac, live2);
            F::load(ring2[s], base2 + (size_t)row_of(row + G2) * A.stride2, geo2, cc);
            const float p = wave_sum_l63(part);
            if (lane == 63 && active && row < row_end) red[(e2 * 8 + cs) * 64 + (row - row0)] = p;
        }
    }
    __syncthreads();
    const int rr = threadIdx.x;
    if (rr < row_end - row0) {
        // The experts are added in ascending id, the order the host puts them in: with device-side routing the
        // entries are in selection order, so two of them may have to swap.
        const bool swap = A.route_idx && A.n_exp == 2 && A.route_idx[0] > A.route_idx[1];
        float y = 0.f;
        for (int i = 0; i < A.n_exp; ++i) {
            const int e = swap ? 1 - i : i;
            float s = 0.f;
            for (int k = 0; k < CS; ++k) s += red[(e * 8 + k) * 64 + rr];
            y += (A.route_idx ? A.route_w[e] : A.w[e]) * s;
        }
        const int row = row0 + rr;
        A.y[row] = y;
        const float v = (float)__builtin_bit_cast(_Float16, A.x[row]) + y;
        A.x_out[row] = __builtin_bit_cast(uint16_t, (_Float16)v);
    }
}

template <int BITS, int KCH, int G1, int G2>
__global__ __launch_bounds__(FUSED_WAVES *WAVE) void k_ffn_token(FusedArgs A)
{
    using F = Fmt<BITS>;
    __shared__ float red[2 * 8 * 64];                    // [expert][cs][row], rows_per_block <= 64
    __shared__ uint16_t a_stage[FUSED_WAVES][FUSED_MAX_ITEMS];   // a wave's outputs until the end of phase 1
    const int lane = threadIdx.x & 63;
    const int wv = uniform(threadIdx.x >> 6);
    const int gw = uniform(blockIdx.x * FUSED_WAVES + wv), n_waves = gridDim.x * FUSED_WAVES;

    // ---------------- phase 1: a[e][r] = silu(W1_e h)[r] * (W3_e h)[r] ----------------
    {
        const int n_chunks = A.H / F::CODES;
        const RowGeom geo = row_geom<BITS>(A.meta13, A.H, A.group, A.scale_group);
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
                // Results wait in LDS: a global store here would sit between the loads in the in-order
                // vmcnt queue, and an agent-scope (write-through) store is slow to be acknowledged.
                if (lane == 63) a_stage[wv][it + s] = __builtin_bit_cast(uint16_t, (_Float16)silu_mul(us, vs));
            }
        }
        // item = e*F + r goes to a[a_row[e]][r]; written with agent scope so that other dies see it after the barrier
        const int item = gw + lane * n_waves;
        if (lane < iters && item < items) {
            const int e = item >= A.F ? 1 : 0;
            __hip_atomic_store(A.a + (size_t)A.a_row[e] * A.F + (item - e * A.F), a_stage[wv][lane], __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    token_w2_phase<BITS, G2, true>(A, red, wv, lane);
}

// ---------------------------------------------------------------------------------------------
// One launch, expert after expert: w1/w3 of expert 0, w1/w3 of expert 1, w2 of expert 0, w2 of expert 1.
//
// k_ffn_token above meets at ONE barrier between all of w1/w3 and all of w2, and every block waits there for the
// slowest wave of the chip (waves of one launch finish their equal shares several microseconds apart).  Here the
// dependencies are per expert -- w2 of expert e needs the activations a of expert e only -- and the phases are
// ordered so that a whole phase of other work lies between producing an a and consuming it: by the time a wave asks
// whether expert 0's a is complete it has streamed expert 1's w1/w3 rows, and before it asks for expert 1's it has
// done expert 0's w2 rows.  The waits therefore find the flags already set (or nearly), the weight stream never
// stops at a phase boundary (the first rows of the next phase are requested before the wait), and the launch pays
// one ramp and one tail instead of two.  Blocks have 8 waves (two per SIMD, 256 registers per lane, the shape
// k_w13 runs best in), one block per compute unit, all resident at once.
//
// Visibility across the dies' L2s as in k_ffn_token: a is written with agent-scope stores, the block waits for their
// acknowledgement, then publishes flags[e][block] = epoch with an agent-scope store; a consumer polls the flags of
// all blocks with agent-scope loads and then reads a with agent-scope loads.  Every wait is bounded.
// ---------------------------------------------------------------------------------------------

constexpr int SEQ_WAVES = 8;
constexpr int SEQ_MAX_ROWS = 64;                   // rows of one expert's w1/w3 per wave
constexpr int SEQ_FLAG_STRIDE = 1024;              // flags[e * SEQ_FLAG_STRIDE + block]

// true when every block has published `epoch` (or a later one) for this expert; polled by one wave for itself
__device__ __forceinline__ bool seq_arrived(const uint32_t *flags, uint32_t epoch, int lane)
{
    int ok = 1;
    for (uint32_t i = lane; i < gridDim.x; i += 64)
        ok &= (int32_t)(__hip_atomic_load(flags + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch) >= 0;
    return __builtin_amdgcn_ballot_w64(!ok) == 0;
}

template <int BITS, int KCH, int G1, int G2>
__global__ __launch_bounds__(SEQ_WAVES *WAVE) void k_ffn_seq(FusedArgs A)
{
    using F = Fmt<BITS>;
    __shared__ float red[2 * 8 * 64];                     // [expert][cs][row]
    __shared__ uint16_t a_stage[SEQ_WAVES][SEQ_MAX_ROWS]; // a wave's outputs of the expert it is working on
    const int lane = threadIdx.x & 63;
    const int wv = uniform(threadIdx.x >> 6);
    const int gw = uniform(blockIdx.x * SEQ_WAVES + wv), n_waves = gridDim.x * SEQ_WAVES;
    auto blob_of = [&](int e) { return A.route_idx ? A.table[uniform(A.route_idx[e]) & 15] : A.blob[e]; };

    // ---------------- w1/w3: a[e][r] = silu(W1_e h)[r] * (W3_e h)[r], expert after expert ----------------
    {
        const int n_chunks = A.H / F::CODES;
        const RowGeom geo = row_geom<BITS>(A.meta13, A.H, A.group, A.scale_group);
        int cidx[KCH];
        bool live[KCH];
#pragma unroll
        for (int k = 0; k < KCH; ++k) {
            live[k] = k * 64 + lane < n_chunks;
            cidx[k] = live[k] ? k * 64 + lane : 0;
        }
        struct RowPair { typename F::Row w1[KCH], w3[KCH]; };
        const int rpw = (A.F + n_waves - 1) / n_waves;      // this wave's rows of every expert: [r0, r0 + rpw)
        const int r0 = gw * rpw;
        const int last_row = A.F - 1;
        // the ring runs over (expert, row) in order; past the end it re-reads the last row (cached, unused)
        auto load_at = [&](RowPair &rb, int e, int j) {
            const int ee = min(e, A.n_exp - 1);
            const uint8_t *r1 = blob_of(ee) + (size_t)(2 * min(r0 + j, last_row)) * A.stride13, *r3 = r1 + A.stride13;
#pragma unroll
            for (int k = 0; k < KCH; ++k) {
                F::load(rb.w1[k], r1, geo, cidx[k]);
                F::load(rb.w3[k], r3, geo, cidx[k]);
            }
        };
        RowPair ring[G1];
        int le = 0, lj = 0;                                  // the next (expert, row) to request
        auto advance = [&](int &e, int &j) { if (++j == rpw) { j = 0; ++e; } };
#pragma unroll
        for (int s = 0; s < G1; ++s) { load_at(ring[s], le, lj); advance(le, lj); }
        typename F::Act hc[KCH];
#pragma unroll
        for (int k = 0; k < KCH; ++k) F::load_act(hc[k], A.h, cidx[k], live[k]);
        const int total = A.n_exp * rpw, trips = (total + G1 - 1) / G1;
        int ce = 0, cj = 0;                                  // the (expert, row) being computed
        for (int it = 0; it < trips; ++it) {
#pragma unroll
            for (int s = 0; s < G1; ++s) {
                float u = 0.f, v = 0.f;
#pragma unroll
                for (int k = 0; k < KCH; ++k) {
                    u += F::contrib(ring[s].w1[k], hc[k], live[k]);
                    v += F::contrib(ring[s].w3[k], hc[k], live[k]);
                }
                load_at(ring[s], le, lj);
                advance(le, lj);
                const float us = wave_sum_l63(u), vs = wave_sum_l63(v);
                if (lane == 63 && ce < A.n_exp) a_stage[wv][cj] = __builtin_bit_cast(uint16_t, (_Float16)silu_mul(us, vs));
                const bool expert_done = ce < A.n_exp && cj == rpw - 1;
                advance(ce, cj);
                if (expert_done) {
                    // this wave's rows of expert ce-1 are complete: store them, wait for the stores (and, with them,
                    // for the ring's loads, which the next trips need anyway), and let the block publish
                    const int e = ce - 1;
                    if (lane < rpw && r0 + lane < A.F)
                        __hip_atomic_store(A.a + (size_t)A.a_row[e] * A.F + r0 + lane, a_stage[wv][lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                    __syncthreads();
                    if (threadIdx.x == 0)
                        __hip_atomic_store(A.barrier + e * SEQ_FLAG_STRIDE + blockIdx.x, A.barrier_target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }

    // ---------------- w2: rows [b*R, (b+1)*R) of this block, expert after expert; combine; residual ----------------
    {
        const int n_chunks2 = A.F / F::CODES;
        const int CS = (n_chunks2 + 63) / 64;               // waves that own a column chunk; the others only wait
        const int cs = wv;
        const bool owner = cs < CS;
        const int c = cs * 64 + lane;
        const bool live2 = owner && c < n_chunks2;
        const int cc = live2 ? c : 0;
        const RowGeom geo2 = row_geom<BITS>(A.meta2, A.F, A.group, A.scale_group);
        const int R = A.rows_per_block;                      // a multiple of G2
        const int row0 = blockIdx.x * R;
        const int row_end = min(row0 + R, A.H);
        const int last2 = max(row_end - 1, 0);
        const bool has_rows = row0 < A.H;
        typename F::Row ring2[G2];
        auto load2 = [&](typename F::Row &rw, int e, int j) {
            const int ee = min(e, A.n_exp - 1);
            F::load(rw, blob_of(ee) + A.off_w2 + (size_t)min(row0 + j, last2) * A.stride2, geo2, cc);
        };
        int le = 0, lj = 0;
        auto advance2 = [&](int &e, int &j) { if (++j == R) { j = 0; ++e; } };
        if (owner && has_rows) {                             // the other waves have no column chunk (or no rows) and go straight to the end
#pragma unroll
        for (int s = 0; s < G2; ++s) { load2(ring2[s], le, lj); advance2(le, lj); }
        typename F::Act ac;
        for (int e = 0; e < A.n_exp; ++e) {
            // expert e's activations must be complete on every block before any of them is read
            const uint32_t *flags = A.barrier + e * SEQ_FLAG_STRIDE;
            uint32_t spins = 0;
            while (!seq_arrived(flags, A.barrier_target, lane)) {
                if (++spins > BARRIER_SPIN_LIMIT) {
                    if (lane == 0) __hip_atomic_store(A.error_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
            }
            load_act_coherent<BITS>(ac, A.a + (size_t)A.a_row[e] * A.F, cc, live2);
            for (int jb = 0; jb < R; jb += G2) {
#pragma unroll
                for (int s = 0; s < G2; ++s) {
                    const int j = jb + s;
                    const float part = F::contrib(ring2[s], ac, live2);
                    load2(ring2[s], le, lj);
                    advance2(le, lj);
                    const float p = wave_sum_l63(part);
                    if (lane == 63 && row0 + j < row_end) red[(e * 8 + cs) * 64 + j] = p;
                }
            }
        }
        }
        __syncthreads();
        const int rr = threadIdx.x;
        if (has_rows && rr < row_end - row0) {
            const bool swap = A.route_idx && A.n_exp == 2 && A.route_idx[0] > A.route_idx[1];   // ascending expert id, as the host orders them
            float y = 0.f;
            for (int i = 0; i < A.n_exp; ++i) {
                const int e = swap ? 1 - i : i;
                float s = 0.f;
                for (int k = 0; k < CS; ++k) s += red[(e * 8 + k) * 64 + rr];
                y += (A.route_idx ? A.route_w[e] : A.w[e]) * s;
            }
            const int row = row0 + rr;
            A.y[row] = y;
            const float v = (float)__builtin_bit_cast(_Float16, A.x[row]) + y;
            A.x_out[row] = __builtin_bit_cast(uint16_t, (_Float16)v);
        }
    }
}

// The w2 half on its own (after k_w13): same combine and residual without atomics or a further kernel.
// grid = ceil(H / rows_per_block) blocks of n_exp * CS waves.
template <int BITS, int G2>
__global__ __launch_bounds__(FUSED_WAVES *WAVE) void k_w2_token(FusedArgs A)
{
    __shared__ float red[2 * 8 * 64];
    token_w2_phase<BITS, G2, false>(A, red, uniform(threadIdx.x >> 6), threadIdx.x & 63);
}

}  // namespace moe
