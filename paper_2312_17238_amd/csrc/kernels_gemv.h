// Fused dequantize+GEMV kernels of the expert FFN for 4-bit, 3-bit and 2-bit group-quantized weights
// (formats of Sec. 4.2 with fp16 scale and zero per group: Fmt<4>, Fmt<3>, Fmt<2>; or with 8-bit scale and zero
// codes per group and an fp16 quad per run of groups, its "scale group size": Fmt<48>, Fmt<38>, Fmt<28>).
//
// Dequantization is never materialised.  With W^ = (q - z) s per group,
//     sum_i W^_i h_i = s * (sum_i q_i h_i - z * sum_i h_i),
// and sum_i q_i h_i comes from fp16 bit tricks: OR-ing a code field into the mantissa of a power of two
// whose ulp equals the weight of the field's lowest bit gives the fp16 number bias+q exactly; two such
// numbers are multiplied with two activations and accumulated in fp32 by one v_dot2_f32_f16.  The biases
// are removed by starting the accumulator at -sum_i bias_i h_i, a per-lane constant.
//
// A lane owns a fixed chunk of columns of every row its wave visits; the activations of that chunk stay in
// registers for the whole kernel; each wave keeps a ring of G rows in flight and the loop body has no branch
// around a load, so the compiler waits (exact vmcnt) for the oldest row only and HBM never drains.
#pragma once
#include "kernels_common.h"

namespace moe {

struct FfnEntry {
    const uint8_t *blob;            // device buffer holding the expert
    int32_t n_tok;                  // 1..MAX_NT tokens routed to this expert in this entry
    int32_t tok[MAX_NT];            // token (batch row) of each
    int32_t pair[MAX_NT];           // row of the activation scratch a[pair][F] (= b*K + j)
    float w[MAX_NT];                // combine weight of each
};

struct FfnArgs {
    FfnEntry e[MAX_ENTRIES];
    const uint16_t *h;              // [B][H] fp16 gate input
    uint16_t *a;                    // [B*K][F] fp16 SwiGLU activations
    float *ypart;                   // [B*K][H] fp32: row `pair` receives w * (W2^ a[pair]); k_combine adds a token's rows
    uint32_t *ytab;                 // [B*K]: where k_combine finds the rows of each pair (y_rows below)
    int32_t H, F, group;
    int32_t scale_group;            // two-level metadata: groups per run of the second level (0: fp16 pairs)
    uint32_t stride13, meta13;      // w1/w3 row: stride and offset of the (scale, zero) pairs
    uint32_t stride2, meta2;        // w2 row
    uint64_t off_w2;
    int32_t rows_per_block;         // w2 kernel
    // Device-side routing: entry j serves the j-th selected expert, whose id the gate kernel of the same step left in
    // route_idx[j]; its weights are in table[id].  Null: the entries carry their blob pointers themselves.
    const int32_t *route_idx;
    const uint8_t *table[16];       // device buffer of every expert of the layer (all resident)
};

// Geometry of one matrix row as the format policies see it.
struct RowGeom {
    uint32_t meta_off;   // byte offset of the (scale, zero) pairs (4-bit, 3-bit)
    uint32_t b_off;      // byte offset of region B (3-bit)
    int32_t gshift;      // 4-bit: log2(group / 32)
    uint32_t meta2_off;  // two-level metadata: byte offset of the per-run fp16 quads
    int32_t run_shift;   // ... log2(groups per run); 31 when the row is one run
};

// sum over one 32-bit word of 4-bit fields (8 codes) times 8 activations, biases 1024 / 64 alternating
__device__ __forceinline__ float dot_word4(uint32_t w, const h2_t *h, float d)
{
    const uint32_t hi = w >> 8;
    d = __builtin_amdgcn_fdot2(as_h2(and_or(w, 0x000F000Fu, 0x64006400u)), h[0], d, false);
    d = __builtin_amdgcn_fdot2(as_h2(and_or(w, 0x00F000F0u, 0x54005400u)), h[1], d, false);
    d = __builtin_amdgcn_fdot2(as_h2(and_or(hi, 0x000F000Fu, 0x64006400u)), h[2], d, false);
    d = __builtin_amdgcn_fdot2(as_h2(and_or(hi, 0x00F000F0u, 0x54005400u)), h[3], d, false);
    return d;
}

// ---------------------------------------------------------------------------------------------
// format policies: CODES = codes per lane chunk; Row = what a lane loads per row and chunk;
// Act = the lane's activations for the chunk plus the constants of the factorisation
// ---------------------------------------------------------------------------------------------

template <int BITS>
struct Fmt;

// 4-bit, group 32/64/128: chunk = 32 codes = one uint4; one (scale, zero) pair per chunk (shared by
// group/32 neighbouring chunks).  Field bias: 1024 for bits 0..3, 64 for bits 4..7 of each half-word.
template <>
struct Fmt<4> {
    static constexpr int CODES = 32;
    struct Row { uint4 q; uint32_t m; };
    struct Act { h2_t h[16]; float bias_dot, hsum; };
    static __device__ __forceinline__ void load(Row &r, const uint8_t *row, const RowGeom &g, int c)
    {
        r.q = ldw4(row, c);
        r.m = ldw1(row + g.meta_off, c >> g.gshift);
    }
    static __device__ __forceinline__ void load_act(Act &a, const uint16_t *vec, int c, bool live)
    {
        const uint4 *p = reinterpret_cast<const uint4 *>(vec + (size_t)c * CODES);
        float bd = 0.f, hs = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 v = live ? p[i] : make_uint4(0, 0, 0, 0);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                a.h[4 * i + j] = as_h2(w[j]);
                const float s = (float)a.h[4 * i + j].x + (float)a.h[4 * i + j].y;
                hs += s;
                bd += ((j & 1) ? 64.f : 1024.f) * s;
            }
        }
        a.bias_dot = bd;
        a.hsum = hs;
    }
    static __device__ __forceinline__ float contrib(const Row &r, const Act &a, bool live)
    {
        float d = -a.bias_dot;
        d = dot_word4(r.q.x, a.h + 0, d);
        d = dot_word4(r.q.y, a.h + 4, d);
        d = dot_word4(r.q.z, a.h + 8, d);
        d = dot_word4(r.q.w, a.h + 12, d);
        const float s = live ? lo_half(r.m) : 0.f;
        return s * fmaf(-hi_half(r.m), a.hsum, d);
    }
};

// 4-bit with two-level metadata (Sec. 4.2 "scale group size"): per group a (scale code, zero code) byte pair, per run
// of groups an fp16 quad (scale step, scale zero, zero step, zero zero); scale = (code - zero) * step for both.
// The codes and the activations are those of Fmt<4>; only where a chunk's scale and zero come from differs.
template <>
struct Fmt<48> {
    static constexpr int CODES = 32;
    struct Row { uint4 q; uint32_t m; uint2 quad; };
    using Act = Fmt<4>::Act;
    static __device__ __forceinline__ void load(Row &r, const uint8_t *row, const RowGeom &g, int c)
    {
        const int grp = c >> g.gshift;
        r.q = ldw4(row, c);
        r.m = *reinterpret_cast<const uint16_t *>(row + g.meta_off + 2 * grp);
        r.quad = *reinterpret_cast<const uint2 *>(row + g.meta2_off + 8 * (grp >> g.run_shift));   // shared by the row's lanes: plain load
    }
    static __device__ __forceinline__ void load_act(Act &a, const uint16_t *vec, int c, bool live) { Fmt<4>::load_act(a, vec, c, live); }
    static __device__ __forceinline__ float contrib(const Row &r, const Act &a, bool live)
    {
        float d = -a.bias_dot;
        d = dot_word4(r.q.x, a.h + 0, d);
        d = dot_word4(r.q.y, a.h + 4, d);
        d = dot_word4(r.q.z, a.h + 8, d);
        d = dot_word4(r.q.w, a.h + 12, d);
        const float s = ((float)(r.m & 0xffu) - hi_half(r.quad.x)) * lo_half(r.quad.x);
        const float z = ((float)(r.m >> 8) - hi_half(r.quad.y)) * lo_half(r.quad.y);
        return (live ? s : 0.f) * fmaf(-z, a.hsum, d);
    }
};

// 2-bit, group 16: chunk = 32 codes = two groups, each a word of 16 codes followed by its pair (one uint4).
// Field n of a half-word (bits 2n..2n+1): direct for n < 5 with bias 1024 / 4^n, after >> 10 for n = 5..7.
template <>
struct Fmt<2> {
    static constexpr int CODES = 32;
    struct Row { uint4 q; };
    struct Act { h2_t h[16]; float bias_dot[2], hsum[2]; };
    static __device__ __forceinline__ float bias_of(int n)
    {
        return n == 0 || n == 5 ? 1024.f : (n == 1 || n == 6 ? 256.f : (n == 2 || n == 7 ? 64.f : (n == 3 ? 16.f : 4.f)));
    }
    static __device__ __forceinline__ void load(Row &r, const uint8_t *row, const RowGeom &, int c) { r.q = ldw4(row, c); }
    static __device__ __forceinline__ void load_act(Act &a, const uint16_t *vec, int c, bool live)
    {
        const uint4 *p = reinterpret_cast<const uint4 *>(vec + (size_t)c * CODES);
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            float bd = 0.f, hs = 0.f;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint4 v = live ? p[2 * g + i] : make_uint4(0, 0, 0, 0);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int n = 4 * i + j;
                    a.h[8 * g + n] = as_h2(w[j]);
                    const float s = (float)a.h[8 * g + n].x + (float)a.h[8 * g + n].y;
                    hs += s;
                    bd += bias_of(n) * s;
                }
            }
            a.bias_dot[g] = bd;
            a.hsum[g] = hs;
        }
    }
    static __device__ __forceinline__ float dot_word2(uint32_t w, const h2_t *h, float d)
    {
        const uint32_t hi = w >> 10;
        d = __builtin_amdgcn_fdot2(as_h2(and_or(w, 0x00030003u, 0x64006400u)), h[0], d, false);
        d = __builtin_amdgcn_fdot2(as_h2(and_or(w, 0x000C000Cu, 0x5C005C00u)), h[1], d, false);
        d = __builtin_amdgcn_fdot2(as_h2(and_or(w, 0x00300030u, 0x54005400u)), h[2], d, false);
        d = __builtin_amdgcn_fdot2(as_h2(and_or(w, 0x00C000C0u, 0x4C004C00u)), h[3], d, false);
        d = __builtin_amdgcn_fdot2(as_h2(and_or(w, 0x03000300u, 0x44004400u)), h[4], d, false);
        d = __builtin_amdgcn_fdot2(as_h2(and_or(hi, 0x00030003u, 0x64006400u)), h[5], d, false);
        d = __builtin_amdgcn_fdot2(as_h2(and_or(hi, 0x000C000Cu, 0x5C005C00u)), h[6], d, false);
        d = __builtin_amdgcn_fdot2(as_h2(and_or(hi, 0x00300030u, 0x54005400u)), h[7], d, false);
        return d;
    }
    static __device__ __forceinline__ float contrib(const Row &r, const Act &a, bool live)
    {
        const float d0 = dot_word2(r.q.x, a.h + 0, -a.bias_dot[0]);
        const float d1 = dot_word2(r.q.z, a.h + 8, -a.bias_dot[1]);
        const float s0 = live ? lo_half(r.q.y) : 0.f, s1 = live ? lo_half(r.q.w) : 0.f;
        return fmaf(s0, fmaf(-hi_half(r.q.y), a.hsum[0], d0), s1 * fmaf(-hi_half(r.q.w), a.hsum[1], d1));
    }
};

// 3-bit, group 64: chunk = 64 codes = one group: 16 B of region A (low two bits of eight 4-bit-layout
// words, two per word), 8 B of region B (third bits, four words per word), one pair.  The eight words are
// rebuilt with three bit operations each and fed to the 4-bit arithmetic.
template <>
struct Fmt<3> {
    static constexpr int CODES = 64;
    struct Row { uint4 a; uint2 b; uint32_t m; };
    struct Act { h2_t h[32]; float bias_dot, hsum; };
    static __device__ __forceinline__ void load(Row &r, const uint8_t *row, const RowGeom &g, int c)
    {
        r.a = ldw4(row, c);
        r.b = ldw2(row + g.b_off, c);
        r.m = ldw1(row + g.meta_off, c);
    }
    static __device__ __forceinline__ void load_act(Act &a, const uint16_t *vec, int c, bool live)
    {
        const uint4 *p = reinterpret_cast<const uint4 *>(vec + (size_t)c * CODES);
        float bd = 0.f, hs = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint4 v = live ? p[i] : make_uint4(0, 0, 0, 0);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                a.h[4 * i + j] = as_h2(w[j]);
                const float s = (float)a.h[4 * i + j].x + (float)a.h[4 * i + j].y;
                hs += s;
                bd += ((j & 1) ? 64.f : 1024.f) * s;
            }
        }
        a.bias_dot = bd;
        a.hsum = hs;
    }
    // sum of code * activation over the group, the field biases already taken off
    static __device__ __forceinline__ float code_dot(const uint4 &ra, const uint2 &rb, const Act &a)
    {
        const uint32_t A[4] = {ra.x, ra.y, ra.z, ra.w};
        const uint32_t B[2] = {rb.x, rb.y};
        float d = -a.bias_dot;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t lo = (j & 1) ? (A[j / 2] >> 2) : A[j / 2];
            const uint32_t bsrc = B[j / 4];
            const uint32_t hb = (j % 4) == 0 ? (bsrc << 2) : ((j % 4) == 1 ? (bsrc << 1) : ((j % 4) == 2 ? bsrc : (bsrc >> 1)));
            const uint32_t t = and_or(lo, 0x33333333u, hb & 0x44444444u);
            d = dot_word4(t, a.h + 4 * j, d);
        }
        return d;
    }
    static __device__ __forceinline__ float contrib(const Row &r, const Act &a, bool live)
    {
        const float d = code_dot(r.a, r.b, a);
        const float s = live ? lo_half(r.m) : 0.f;
        return s * fmaf(-hi_half(r.m), a.hsum, d);
    }
};

// Scale and zero of one group from its byte pair (scale code in the low byte) and its run's quad.
__device__ __forceinline__ void decode_meta8(uint32_t pair, const uint2 &quad, float &s, float &z)
{
    s = ((float)(pair & 0xffu) - hi_half(quad.x)) * lo_half(quad.x);
    z = ((float)((pair >> 8) & 0xffu) - hi_half(quad.y)) * lo_half(quad.y);
}

// 3-bit with two-level metadata: the codes and activations of Fmt<3>, scale and zero as in Fmt<48>.
template <>
struct Fmt<38> {
    static constexpr int CODES = 64;
    struct Row { uint4 a; uint2 b; uint32_t m; uint2 quad; };
    using Act = Fmt<3>::Act;
    static __device__ __forceinline__ void load(Row &r, const uint8_t *row, const RowGeom &g, int c)
    {
        r.a = ldw4(row, c);
        r.b = ldw2(row + g.b_off, c);
        r.m = *reinterpret_cast<const uint16_t *>(row + g.meta_off + 2 * c);
        r.quad = *reinterpret_cast<const uint2 *>(row + g.meta2_off + 8 * (c >> g.run_shift));
    }
    static __device__ __forceinline__ void load_act(Act &a, const uint16_t *vec, int c, bool live) { Fmt<3>::load_act(a, vec, c, live); }
    static __device__ __forceinline__ float contrib(const Row &r, const Act &a, bool live)
    {
        const float d = Fmt<3>::code_dot(r.a, r.b, a);
        float s, z;
        decode_meta8(r.m, r.quad, s, z);
        return (live ? s : 0.f) * fmaf(-z, a.hsum, d);
    }
};

// 2-bit with two-level metadata: chunk = 64 codes = four groups = one uint4 of code words (no longer interleaved
// with metadata), four byte pairs (one uint2) and the quad of the run the four groups lie in.
template <>
struct Fmt<28> {
    static constexpr int CODES = 64;
    struct Row { uint4 q; uint2 m; uint2 quad; };
    struct Act { h2_t h[32]; float bias_dot[4], hsum[4]; };
    static __device__ __forceinline__ void load(Row &r, const uint8_t *row, const RowGeom &g, int c)
    {
        r.q = ldw4(row, c);
        r.m = ldw2(row + g.meta_off, c);
        r.quad = *reinterpret_cast<const uint2 *>(row + g.meta2_off + 8 * ((4 * c) >> g.run_shift));
    }
    static __device__ __forceinline__ void load_act(Act &a, const uint16_t *vec, int c, bool live)
    {
        const uint4 *p = reinterpret_cast<const uint4 *>(vec + (size_t)c * CODES);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float bd = 0.f, hs = 0.f;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint4 v = live ? p[2 * g + i] : make_uint4(0, 0, 0, 0);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int n = 4 * i + j;
                    a.h[8 * g + n] = as_h2(w[j]);
                    const float s = (float)a.h[8 * g + n].x + (float)a.h[8 * g + n].y;
                    hs += s;
                    bd += Fmt<2>::bias_of(n) * s;
                }
            }
            a.bias_dot[g] = bd;
            a.hsum[g] = hs;
        }
    }
    static __device__ __forceinline__ float contrib(const Row &r, const Act &a, bool live)
    {
        const uint32_t w[4] = {r.q.x, r.q.y, r.q.z, r.q.w};
        const uint32_t pr[4] = {r.m.x, r.m.x >> 16, r.m.y, r.m.y >> 16};
        float acc = 0.f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float d = Fmt<2>::dot_word2(w[g], a.h + 8 * g, -a.bias_dot[g]);
            float s, z;
            decode_meta8(pr[g], r.quad, s, z);
            acc = fmaf(s, fmaf(-z, a.hsum[g], d), acc);
        }
        return live ? acc : 0.f;
    }
};

template <int BITS>
__device__ __forceinline__ RowGeom row_geom(uint32_t meta_off, int cols, int group, int scale_group)
{
    RowGeom g;
    g.meta_off = meta_off;
    g.b_off = (BITS == 3 || BITS == 38) ? (uint32_t)(cols / 64) * 16u : 0u;
    g.gshift = (group == 32) ? 0 : (group == 64 ? 1 : 2);
    const int groups = cols / group;
    g.meta2_off = (meta_off + 2u * groups + 7u) & ~7u;
    g.run_shift = (scale_group <= 0 || groups <= scale_group) ? 31 : __builtin_ctz((unsigned)scale_group);
    return g;
}

// K2: a[pair][r] = silu(W1^ h)[r] * (W3^ h)[r].  grid = (row blocks, entries), WAVES waves per block; a wave
// walks rows r = wave_id, wave_id + n_waves, ... with G of them in flight; KCH = chunks per lane per row.
template <int BITS, int KCH, int NT, int G, int WAVES>
__global__ __launch_bounds__(WAVES *WAVE) void k_w13(FfnArgs A)
{
    using F = Fmt<BITS>;
    const FfnEntry &en = A.e[blockIdx.y];
    const int lane = threadIdx.x & 63;
    const int wave = uniform(blockIdx.x * WAVES + (threadIdx.x >> 6)), n_waves = gridDim.x * WAVES;
    const int n_chunks = A.H / F::CODES;
    const RowGeom geo = row_geom<BITS>(A.meta13, A.H, A.group, A.scale_group);
    const uint8_t *base = A.route_idx ? A.table[uniform(A.route_idx[blockIdx.y]) & 15] : en.blob;

    int cidx[KCH];
    bool live[KCH];
#pragma unroll
    for (int k = 0; k < KCH; ++k) {
        live[k] = k * 64 + lane < n_chunks;
        cidx[k] = live[k] ? k * 64 + lane : 0;
    }
    struct RowPair { typename F::Row w1[KCH], w3[KCH]; };
    auto load_row = [&](RowPair &rb, int r) {
        const uint8_t *r1 = base + (size_t)(2 * r) * A.stride13, *r3 = r1 + A.stride13;
#pragma unroll
        for (int k = 0; k < KCH; ++k) {
            F::load(rb.w1[k], r1, geo, cidx[k]);
            F::load(rb.w3[k], r3, geo, cidx[k]);
        }
    };
    // Rows past the end are clamped to the last row (a redundant, cached read) and not stored.
    const int last = A.F - 1;
    const int iters = (A.F + n_waves - 1) / n_waves;
    RowPair ring[G];                      // weights first (HBM latency), then the activations (L2)
#pragma unroll
    for (int s = 0; s < G; ++s) load_row(ring[s], min(wave + s * n_waves, last));

    typename F::Act hc[NT][KCH];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tok = en.tok[t < en.n_tok ? t : 0];
#pragma unroll
        for (int k = 0; k < KCH; ++k) F::load_act(hc[t][k], A.h + (size_t)tok * A.H, cidx[k], live[k]);
    }

    for (int it = 0; it < iters; it += G) {
#pragma unroll
        for (int s = 0; s < G; ++s) {
            const int r = wave + (it + s) * n_waves;
            float u[NT], v[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) { u[t] = 0.f; v[t] = 0.f; }
#pragma unroll
            for (int k = 0; k < KCH; ++k)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    u[t] += F::contrib(ring[s].w1[k], hc[t][k], live[k]);
                    v[t] += F::contrib(ring[s].w3[k], hc[t][k], live[k]);
                }
            load_row(ring[s], min(r + G * n_waves, last));
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float us = wave_sum_l63(u[t]), vs = wave_sum_l63(v[t]);
                if (lane == 63 && t < en.n_tok && r < A.F) {
                    const _Float16 av = (_Float16)silu_mul(us, vs);
                    A.a[(size_t)en.pair[t] * A.F + r] = __builtin_bit_cast(uint16_t, av);
                }
            }
        }
    }
}

// Entry of the table that tells k_combine where the contribution of one (token, expert) pair lies: `parts`
// consecutive rows of the partial-output buffer starting at `row` (several when the contraction was split over blocks).
__host__ __device__ __forceinline__ uint32_t y_rows(uint32_t row, uint32_t parts) { return row | (parts << 24); }

// K3: ypart[pair][r] = w * (W2^ a[pair])[r].  grid = (row blocks, entries); block = CS waves, wave cs owns
// column chunk cs*64 + lane of every row of the block (G rows in flight); partial sums meet in LDS.  No atomics:
// every element of ypart has one writer, and k_combine adds the rows of a token in a fixed order.
template <int BITS, int NT, int G>
__global__ __launch_bounds__(512) void k_w2(FfnArgs A)
{
    using F = Fmt<BITS>;
    extern __shared__ float red[];                       // [rows_per_block][NT][CS]
    const FfnEntry &en = A.e[blockIdx.y];
    const int lane = threadIdx.x & 63, cs = uniform(threadIdx.x >> 6), CS = blockDim.x >> 6;
    const int n_chunks = A.F / F::CODES;
    const int c = cs * 64 + lane;
    const bool live = c < n_chunks;
    const int cc = live ? c : 0;
    const RowGeom geo = row_geom<BITS>(A.meta2, A.F, A.group, A.scale_group);
    const int R = A.rows_per_block;
    const int row0 = blockIdx.x * R;
    const int row_end = min(row0 + R, A.H);
    const uint8_t *base = en.blob + A.off_w2;

    const int last = row_end - 1;                        // rows past the block's end: clamped, results dropped
    typename F::Row ring[G];
#pragma unroll
    for (int s = 0; s < G; ++s) F::load(ring[s], base + (size_t)min(row0 + s, last) * A.stride2, geo, cc);

    typename F::Act ac[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) F::load_act(ac[t], A.a + (size_t)en.pair[t < en.n_tok ? t : 0] * A.F, cc, live);

    for (int rbase = row0; rbase < row_end; rbase += G) {
#pragma unroll
        for (int s = 0; s < G; ++s) {
            const int row = rbase + s;
            float part[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) part[t] = F::contrib(ring[s], ac[t], live);
            F::load(ring[s], base + (size_t)min(row + G, last) * A.stride2, geo, cc);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float p = wave_sum_l63(part[t]);
                if (lane == 63 && row < row_end) red[((row - row0) * NT + t) * CS + cs] = p;
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < (row_end - row0) * NT; i += blockDim.x) {
        const int rr = i / NT, t = i % NT;
        if (t < en.n_tok) {
            float s = 0.f;
            for (int k = 0; k < CS; ++k) s += red[i * CS + k];
            A.ypart[(size_t)en.pair[t] * A.H + row0 + rr] = en.w[t] * s;
        }
    }
    if (blockIdx.x == 0 && (int)threadIdx.x < en.n_tok) A.ytab[en.pair[threadIdx.x]] = y_rows((uint32_t)en.pair[threadIdx.x], 1u);
}

// S7 for steps that do not finish inside a w2 kernel: y[b] = sum over the token's K pairs, in selection order, of the
// pair's rows of ypart (parts of a split contraction in ascending order); x_out = fp16(x + y); y is kept (fp32) for
// diagnostics.  One thread per four elements; the order of the additions is fixed, so the result is reproducible
// bit for bit whatever order the w2 blocks finished in.
__global__ __launch_bounds__(256) void k_combine(const uint16_t *x, const float *ypart, const uint32_t *ytab, float *y, uint16_t *x_out,
                                                 int H, int K, uint32_t cap_rows)
{
    const int b = blockIdx.y, i = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= H) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < K; ++j) {
        const uint32_t t = ytab[b * K + j];
        const uint32_t row = t & 0xffffffu, parts = t >> 24;
        if (parts == 0 || row + parts > cap_rows) continue;      // an entry no kernel of this step wrote: never read outside the buffer
        float4 s = *reinterpret_cast<const float4 *>(ypart + (size_t)row * H + i);
        for (uint32_t p = 1; p < parts; ++p) {
            const float4 v = *reinterpret_cast<const float4 *>(ypart + (size_t)(row + p) * H + i);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        acc.x += s.x; acc.y += s.y; acc.z += s.z; acc.w += s.w;
    }
    *reinterpret_cast<float4 *>(y + (size_t)b * H + i) = acc;
    const uint2 xv = *reinterpret_cast<const uint2 *>(x + (size_t)b * H + i);
    const _Float16 o0 = (_Float16)(lo_half(xv.x) + acc.x), o1 = (_Float16)(hi_half(xv.x) + acc.y);
    const _Float16 o2 = (_Float16)(lo_half(xv.y) + acc.z), o3 = (_Float16)(hi_half(xv.y) + acc.w);
    const uint2 ov = make_uint2((uint32_t)__builtin_bit_cast(uint16_t, o0) | (uint32_t)__builtin_bit_cast(uint16_t, o1) << 16,
                                (uint32_t)__builtin_bit_cast(uint16_t, o2) | (uint32_t)__builtin_bit_cast(uint16_t, o3) << 16);
    *reinterpret_cast<uint2 *>(x_out + (size_t)b * H + i) = ov;
}

// ---------------------------------------------------------------------------------------------
// calibration probes: plain streaming read and plain copy of a device buffer
// ---------------------------------------------------------------------------------------------

// Every thread reads uint4s grid-strided, 8 in flight; the xor of everything lands in out[block] so the
// loads cannot be dropped.  n16 = number of 16-byte words.
__global__ __launch_bounds__(256) void k_probe_read(const uint4 *src, size_t n16, uint32_t *out)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t acc = 0;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        uint4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = ldw4(src + i + j * stride, 0);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u) out[blockIdx.x] = acc;      // practically never: keeps the loads alive without a store stream
}

__global__ __launch_bounds__(256) void k_probe_copy(const uint4 *src, uint4 *dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace moe
