// Grouped dequantize+GEMM on the matrix cores, streaming form: persistent blocks built so that the weights
// cross HBM once in long coalesced reads, every load is issued a whole step before its use, and the vector
// unit does the minimum of work per weight.
//
// Work item  = 128 consecutive MEMORY rows of one matrix of one (expert, token tile) entry, over one part of K
//              (w1/w3, whose rows are interleaved in the blob, always take all of K: their epilogue needs the
//              complete sums; w2 may split K: every part writes a row of partial sums of its own, and k_combine adds
//              the parts in ascending order, so no atomics and a result that does not depend on timing).
// Step       = one segment of 8 groups (512 codes) of a work item: 128 rows x (256 B codes + 32 B pairs) = 36 KB.
// Block      = 4 waves, two blocks per compute unit (their phases drift apart, so one block's loads overlap the
//              other's arithmetic), each walking its items (blockIdx.x, +gridDim.x, ...) as one sequence of
//              steps.  During step s every wave requests what step s+1 needs -- its own A operands
//              (activations of up to 32 tokens, from L2) and its share of the 36 KB of weights (from HBM, into
//              registers) -- in eight pieces, one beside each (group, tile) unit it multiplies out of one of two LDS
//              buffers (a wave that issues its whole share at once stalls on the full queues of the memory pipeline;
//              what depends on the item alone -- expert, token rows -- is looked up once per item), then stores the
//              arrived weights to the other buffer; one barrier per step.  Memory loads return in order per wave, so
//              nothing inside the multiply may wait for a load of the same step: the A operands travel a full step
//              ahead.
// Wave w     = groups w and w+4 of the step for all four 32-row tiles: A operand once per group, reused by the four
//              tiles; B operand from LDS as codes (read one tile ahead), dequantised to fp16 in registers,
//              w = (q - z) s computed as (q - rint(z)) s + (rint(z) - z) s with one rounding, and the MFMA
//              accumulates across all groups of the item (Sec. 4.2 runs the experts on dequantised fp16
//              weights; the GEMV kernels keep more).  At the end of an item the waves add their partial
//              sums through the LDS buffer just consumed, two tiles at a time, in a fixed order.
//
// R1 (default when the second level of metadata is absent): the exact subtraction above is left out.  The codes
//              enter as 1024+q or 64+q (the and_or patterns) and ONE fused multiply-add per pair of weights gives
//              (bias+q) s - e with e = fp16((bias+z) s): the bias cancels inside the fma, the result is rounded once,
//              as before.  What the rounding of e leaves, d = e - (bias+z) s (one number per row, group and bias, at
//              most half an ulp of e), multiplies every activation that meets a code of that bias; the sums of
//              those activations per (token, group, half of the group, bias) are taken from the A operands the lane already holds
//              (sixteen two-way dot products with ones per group, shared by the four tiles), and one more MFMA
//              per (tile, wave, step) adds sum d * (partial sum) back: 16 K-slots = 2 halves x 2 groups x 2 biases
//              (the rest zero).  The term is ~8 % of the result, so fp16 factors suffice.  A third fewer vector
//              instructions in the dequantisation.
//
// MFMA layouts (v_mfma_f32_32x32x16_f16): A lane l = row (token) l%32, k-slot l/32; B lane l = column (memory
// row) l%32, k-slot l/32; D lane l, register i = row 8*(i/4) + 4*(l/32) + i%4, column l%32.
#pragma once
#include "kernels_mfma.h"

namespace moe {

#ifndef MOE_TL_WAVES
#define MOE_TL_WAVES 4
#define MOE_TL_BLOCKS_PER_CU 2
#define MOE_TL_SG 8
#endif
constexpr int TL_WAVES = MOE_TL_WAVES;
constexpr int TL_BLOCKS_PER_CU = MOE_TL_BLOCKS_PER_CU;
constexpr int TL_THREADS = TL_WAVES * WAVE;
constexpr int TL_RT = 4;                                 // 32-row tiles per item
constexpr int TL_ROWS = TL_RT * 32;
constexpr int TL_SG = MOE_TL_SG;                         // groups per step
constexpr int TL_GPW = TL_SG / TL_WAVES;                 // groups per wave and step (2)
constexpr int TL_CODE_PITCH = TL_SG * 32 + 16;           // bytes per staged row of codes (+16: bank spread)
constexpr int TL_META_PITCH = TL_SG + 1;                 // words per staged row of pairs (odd: bank spread)
constexpr int TL_BUF_BYTES = TL_ROWS * TL_CODE_PITCH + TL_ROWS * TL_META_PITCH * 4;
constexpr int TL_TABLE_BYTES = MF_MAX_PAIRS * 6;         // token, pair (bytes) and combine weight (float) of every pair
constexpr int TL_LDS_BYTES = 2 * TL_BUF_BYTES + TL_TABLE_BYTES;
constexpr int TL_CPR = TL_SG * 2, TL_MPR = TL_SG / 4;    // 16-byte code / pair pieces per staged row
constexpr int TL_CP = TL_ROWS * TL_CPR / TL_THREADS;     // code pieces per thread and step (8)
constexpr int TL_MP = TL_ROWS * TL_MPR / TL_THREADS;     // pair pieces per thread and step (1)
constexpr int TL_NI = 2 * 16 / TL_WAVES;                 // accumulator registers a wave finishes per reduction round
static_assert(TL_WAVES * 2 * 16 * 64 * 4 <= TL_BUF_BYTES, "one reduction round (two tiles of every wave) must fit a staging buffer");
static_assert(TL_CP * TL_THREADS == TL_ROWS * TL_CPR && TL_MP * TL_THREADS == TL_ROWS * TL_MPR, "pieces must divide evenly");
static_assert(TL_SG % 4 == 0 && (TL_CPR & (TL_CPR - 1)) == 0 && (TL_MPR & (TL_MPR - 1)) == 0, "pieces per row must be powers of two");

struct TileArgs {
    MfmaEntry e[32];                         // (expert, token tile) entries
    uint8_t tok[MF_MAX_PAIRS];
    uint8_t pair[MF_MAX_PAIRS];
    float w[MF_MAX_PAIRS];
    const uint16_t *act;                     // w1/w3: h [B][H];   w2: a [B*K][F]
    uint16_t *a;                             // w1/w3 output
    float *ypart;                            // w2 output: fp32 rows of H, one per pair (and per part of a split contraction)
    uint32_t *ytab;                          // [pairs of the window]: where k_combine finds each pair's rows
    int32_t part_base;                       // k_parts > 1: pair i of the launch (its index in tok[]/pair[]) owns rows part_base + i * k_parts + part
    int32_t row_bias;                        // added to a row before it goes into ytab (ypart and ytab point at the window's first pair)
    int32_t K, N;                            // contraction length, output rows of the matrix
    uint32_t stride, meta_off;
    uint32_t meta2_off;                      // two-level metadata: byte offset of the per-run fp16 quads inside a row
    int32_t run_shift;                       // ... log2(groups per run), 31 when a row is one run
    uint64_t mat_off;
    int32_t row_blocks, k_parts, seg_per_part, n_items;   // item = ((entry * row_blocks) + row block) * k_parts + part
};

struct TileStep { int it, seg, seg_hi, rb, e; bool valid; };

// eight codes -> eight fp16 weights: exact integer q - rint(z) first, then one fused multiply-add
__device__ __forceinline__ h8_t codes_to_w8(uint32_t w, h2_t b1024, h2_t b64, h2_t s2, h2_t c2)
{
    const uint32_t hi = w >> 8;
    const h2_t t0 = __builtin_elementwise_fma(as_h2(and_or(w, 0x000F000Fu, 0x64006400u)) + b1024, s2, c2);
    const h2_t t1 = __builtin_elementwise_fma(as_h2(and_or(w, 0x00F000F0u, 0x54005400u)) + b64, s2, c2);
    const h2_t t2 = __builtin_elementwise_fma(as_h2(and_or(hi, 0x000F000Fu, 0x64006400u)) + b1024, s2, c2);
    const h2_t t3 = __builtin_elementwise_fma(as_h2(and_or(hi, 0x00F000F0u, 0x54005400u)) + b64, s2, c2);
    h8_t r;
    r[0] = t0.x; r[1] = t0.y; r[2] = t1.x; r[3] = t1.y; r[4] = t2.x; r[5] = t2.y; r[6] = t3.x; r[7] = t3.y;
    return r;
}

// R1: eight codes -> eight fp16 weights with one fused multiply-add per pair: (bias + q) s - e
__device__ __forceinline__ h8_t codes_to_w8_r1(uint32_t w, h2_t s2, h2_t ne1024, h2_t ne64)
{
    const uint32_t hi = w >> 8;
    const h2_t t0 = __builtin_elementwise_fma(as_h2(and_or(w, 0x000F000Fu, 0x64006400u)), s2, ne1024);
    const h2_t t1 = __builtin_elementwise_fma(as_h2(and_or(w, 0x00F000F0u, 0x54005400u)), s2, ne64);
    const h2_t t2 = __builtin_elementwise_fma(as_h2(and_or(hi, 0x000F000Fu, 0x64006400u)), s2, ne1024);
    const h2_t t3 = __builtin_elementwise_fma(as_h2(and_or(hi, 0x00F000F0u, 0x54005400u)), s2, ne64);
    h8_t r;
    r[0] = t0.x; r[1] = t0.y; r[2] = t1.x; r[3] = t1.y; r[4] = t2.x; r[5] = t2.y; r[6] = t3.x; r[7] = t3.y;
    return r;
}

// R1: the lane's 32 activations of one group half (A operand layout) -> fp16 pair (sum of those at positions 0,1,4,5
// mod 8: they meet the codes that decode with bias 1024; sum of those at 2,3,6,7 mod 8: bias 64), summed in fp32
__device__ __forceinline__ uint32_t half_sums(const h8_t (&a)[4])
{
    const h2_t ones = {(_Float16)1.f, (_Float16)1.f};
    float s1024 = 0.f, s64 = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const u32x4_t u = __builtin_bit_cast(u32x4_t, a[q]);
        s1024 = __builtin_amdgcn_fdot2(as_h2(u[0]), ones, s1024, false);
        s64 = __builtin_amdgcn_fdot2(as_h2(u[1]), ones, s64, false);
        s1024 = __builtin_amdgcn_fdot2(as_h2(u[2]), ones, s1024, false);
        s64 = __builtin_amdgcn_fdot2(as_h2(u[3]), ones, s64, false);
    }
    const h2_t r = {(_Float16)s1024, (_Float16)s64};
    return __builtin_bit_cast(uint32_t, r);
}

// META8: two-level metadata (Sec. 4.2 "scale group size").  A step then stages, per row, 16 bytes of (scale code, zero
// code) byte pairs and the run's fp16 quad instead of 32 bytes of fp16 pairs, and a unit decodes scale and zero in fp32
// before the same fp16 dequantisation.
template <bool W13, bool META8, bool R1 = false>
__global__ __launch_bounds__(TL_THREADS, TL_BLOCKS_PER_CU) void k_mfma_stream_q4(TileArgs A)
{
    static_assert(!(META8 && R1), "the rank-1 form reads fp16 (scale, zero) pairs");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wv = uniform(tid >> 6);
    const int col = lane & 31, kh = lane >> 5;
    const int n_rows = W13 ? 2 * A.N : A.N;
    const int groups = A.K / 64, n_seg = (groups + TL_SG - 1) / TL_SG;

    auto first_step = [&](int it) -> TileStep {
        TileStep s;
        s.it = it;
        s.valid = it < A.n_items;
        const int part = it % A.k_parts, t = it / A.k_parts;
        s.rb = t % A.row_blocks;
        s.e = s.valid ? t / A.row_blocks : 0;
        s.seg = part * A.seg_per_part;
        s.seg_hi = min(n_seg, s.seg + A.seg_per_part);
        return s;
    };
    auto next = [&](const TileStep &s) -> TileStep {
        if (s.seg + 1 < s.seg_hi) { TileStep n = s; n.seg++; return n; }
        return first_step(s.it + (int)gridDim.x);
    };
    auto seg_groups = [&](const TileStep &s) { return min(TL_SG, groups - s.seg * TL_SG); };

    TileStep cur = first_step(blockIdx.x);
    if (!cur.valid) return;                                          // whole block, before any barrier
    // the pair tables move from the kernel arguments to LDS once: the steps look them up with per-lane indices
    float *l_w = reinterpret_cast<float *>(lds + 2 * TL_BUF_BYTES);
    uint8_t *l_tok = reinterpret_cast<uint8_t *>(l_w + MF_MAX_PAIRS), *l_pair = l_tok + MF_MAX_PAIRS;
    if (tid < MF_MAX_PAIRS) {
        l_w[tid] = A.w[tid];
        l_tok[tid] = A.tok[tid];
        l_pair[tid] = A.pair[tid];
    }
    __syncthreads();
    TileStep nxt = next(cur);
    int buf = 0;

    // ---------------- addresses ----------------
    // What depends on the item alone -- its expert's matrix, this lane's token row of the activations (a lookup in the
    // LDS tables) -- is worked out when the sequence of loads enters the item; a step then adds only uniform terms
    // (segment, 16-row slab), which stay in scalar registers, to per-thread offsets that never change.
    int addr_it = -1;
    const uint8_t *mat_base = nullptr;
    uint32_t act_off = 0;                                            // bytes: token row of act + this lane's half of a group
    auto token_index = [&](const TileStep &s) -> int {               // row of act; lanes past the last token read the first again
        const MfmaEntry &en = A.e[s.e];
        const int tk = col < en.n_tok ? col : 0;
        return W13 ? l_tok[en.first + tk] : l_pair[en.first + tk];
    };
    auto enter_item = [&](const TileStep &s) {
        if (s.it == addr_it) return;
        addr_it = s.it;
        mat_base = A.e[s.e].blob + A.mat_off;
        act_off = (uint32_t)token_index(s) * (uint32_t)A.K * 2u + (uint32_t)kh * 64u;
    };

    // ---------------- weights: HBM -> registers -> LDS ----------------
    // The loads of a step go out in pieces, one between every two units of the multiply (below): a wave that issues
    // its whole share at once finds the memory pipeline's queues full and stalls where it could be computing.
    uint4 st_c[TL_CP], st_m[TL_MP];
    struct FetchCtx { const uint8_t *seg; uint32_t voff; int row0, slab, g0, sg; bool live; };
    constexpr int SLAB = TL_THREADS / TL_CPR;                        // rows that one piece index covers (16)
    static_assert(TL_THREADS % TL_CPR == 0 && 64 % SLAB == 0, "a slab of rows lies wholly inside or outside a matrix of 64 k rows");
    // live = false (after a block's last step there is nothing to fetch): the loads stay in the instruction stream,
    // so that no branch surrounds them, but every lane of every piece reads the same 16 bytes
    auto fetch_begin = [&](const TileStep &s, bool live) -> FetchCtx {
        enter_item(s);
        FetchCtx f;
        f.live = live;
        f.g0 = s.seg * TL_SG; f.sg = seg_groups(s);
        f.row0 = live ? s.rb * TL_ROWS : 0;
        f.slab = live ? SLAB : 0;
        const uint32_t c = tid % TL_CPR;
        f.voff = live ? (uint32_t)(tid / TL_CPR) * A.stride + ((int)c < 2 * f.sg ? c : 0u) * 16u : 0u;
        f.seg = mat_base + (size_t)f.g0 * 32;
        return f;
    };
    auto fetch_codes = [&](const FetchCtx &f, int i) {
        // a slab past the end of the matrix reads the last one instead: a redundant, cached read nobody uses
        st_c[i] = ldw4(f.seg + (size_t)min(f.row0 + i * f.slab, n_rows - SLAB) * A.stride + f.voff, 0);
    };
    auto fetch_meta = [&](const FetchCtx &f) {
        const int g0 = f.g0, sg = f.sg, row0 = f.row0;
#pragma unroll
        for (int i = 0; i < TL_MP; ++i) {
            const int p = tid + i * TL_THREADS, r = f.live ? p / TL_MPR : 0, c = p % TL_MPR;
            // a step takes 32 B of a row's pairs, its neighbours in the cache line belong to the next steps: a
            // plain load, so that L2 keeps the line (the streaming hint would fetch it from HBM once per step)
            const uint8_t *rowp = mat_base + (size_t)min(row0 + r, n_rows - 1) * A.stride;
            if constexpr (META8) {            // piece 0: the step's 8 byte pairs; piece 1: the fp16 quad of its run
                static_assert(TL_SG == 8 && TL_MPR == 2, "two-level staging is laid out for steps of 8 groups");
                if (c == 0) {
                    st_m[i] = reinterpret_cast<const uint4 *>(rowp + A.meta_off)[g0 / 8];
                } else {
                    const uint2 quad = *reinterpret_cast<const uint2 *>(rowp + A.meta2_off + 8 * (g0 >> A.run_shift));
                    st_m[i] = make_uint4(quad.x, quad.y, 0u, 0u);
                }
            } else {
                st_m[i] = reinterpret_cast<const uint4 *>(rowp + A.meta_off)[g0 / 4 + (c < (sg + 3) / 4 ? c : 0)];
            }
        }
    };
    auto commit = [&](int b) {                                       // pieces past a short segment hold copies nobody reads
        uint8_t *codes = lds + b * TL_BUF_BYTES;
        uint32_t *meta = reinterpret_cast<uint32_t *>(codes + TL_ROWS * TL_CODE_PITCH);
#pragma unroll
        for (int i = 0; i < TL_CP; ++i) {
            const int p = tid + i * TL_THREADS, r = p / TL_CPR, c = p % TL_CPR;
            *reinterpret_cast<uint4 *>(codes + r * TL_CODE_PITCH + c * 16) = st_c[i];
        }
#pragma unroll
        for (int i = 0; i < TL_MP; ++i) {
            const int p = tid + i * TL_THREADS, r = p / TL_MPR, c = p % TL_MPR;
            uint32_t *d = meta + r * TL_META_PITCH + c * 4;
            d[0] = st_m[i].x; d[1] = st_m[i].y; d[2] = st_m[i].z; d[3] = st_m[i].w;
        }
    };

    // ---------------- multiply ----------------
    f32x16_t acc[TL_RT];
#pragma unroll
    for (int rt = 0; rt < TL_RT; ++rt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[rt][i] = 0.f;
    auto load_a_piece = [&](h8_t (&dst)[TL_GPW][4], const TileStep &s, int j, int q) {   // one MFMA's A operand of step s
        const int g = s.seg * TL_SG + min(wv + TL_WAVES * j, seg_groups(s) - 1);
        const uint8_t *grp = reinterpret_cast<const uint8_t *>(A.act) + (size_t)g * 128;
        dst[j][q] = __builtin_bit_cast(h8_t, *reinterpret_cast<const uint4 *>(grp + act_off + q * 16));
    };
    // piece u of the loads of step s: unit u = (group j, tile rt) of the multiply runs beside it
    static_assert(TL_CP == TL_GPW * TL_RT && TL_RT == 4, "one piece of codes and one A operand per unit");
    // the A operand goes first: the codes then are the last load of a step, and the wait for them before they are
    // stored to LDS leaves nothing in flight for the next step's multiply to wait for
    auto load_piece = [&](const FetchCtx &f, h8_t (&a_dst)[TL_GPW][4], const TileStep &s, int u) {
        load_a_piece(a_dst, s, u / TL_RT, u % TL_RT);
        if (u == 0) fetch_meta(f);
        fetch_codes(f, u);
    };
    // One unit = one group of one 32-row tile; its codes and pair are read from LDS one unit ahead of their use.
    struct UnitMeta { uint32_t m, quad0, quad1; };                   // one-level: m = (scale, zero) fp16; two-level: byte pair + the run's quad
    auto unit_load = [&](int b, int gl, int rt, uint4 &q, UnitMeta &um) {
        const uint8_t *codes = lds + b * TL_BUF_BYTES;
        const uint32_t *meta = reinterpret_cast<const uint32_t *>(codes + TL_ROWS * TL_CODE_PITCH);
        const int r = rt * 32 + col;
        q = *reinterpret_cast<const uint4 *>(codes + r * TL_CODE_PITCH + gl * 32 + kh * 16);
        if constexpr (META8) {
            um.m = (meta[r * TL_META_PITCH + (gl >> 1)] >> (16 * (gl & 1))) & 0xffffu;
            um.quad0 = meta[r * TL_META_PITCH + 4];
            um.quad1 = meta[r * TL_META_PITCH + 5];
        } else {
            um.m = meta[r * TL_META_PITCH + gl];
        }
    };
    uint32_t rho[TL_RT][TL_GPW] = {};                               // R1: what the rounding of e left, per tile and group of the step
    auto unit_multiply = [&](const h8_t (&a)[4], const uint4 &q, const UnitMeta &um, int rt, int j) {
        if constexpr (R1) {
            const h2_t m2 = as_h2(um.m);                                 // (scale, zero)
            const h2_t s2 = __builtin_shufflevector(m2, m2, 0, 0), z2 = __builtin_shufflevector(m2, m2, 1, 1);
            const h2_t bias = {(_Float16)1024.f, (_Float16)64.f};
            const h2_t sb = s2 * bias;                                   // bias * s, exact
            const h2_t e = __builtin_elementwise_fma(z2, s2, sb);        // fp16((bias + z) s), both biases
            const h2_t t = e - sb;                                       // exact (the two are within 2 % of each other)
            const h2_t d = __builtin_elementwise_fma(-z2, s2, t);        // e - (bias + z) s, the fma exact before its rounding
            rho[rt][j] = __builtin_bit_cast(uint32_t, d);
            const h2_t ne = -e;
            const h2_t ne1024 = __builtin_shufflevector(ne, ne, 0, 0), ne64 = __builtin_shufflevector(ne, ne, 1, 1);
            h8_t b[4];
            b[0] = codes_to_w8_r1(q.x, s2, ne1024, ne64); b[1] = codes_to_w8_r1(q.y, s2, ne1024, ne64);
            b[2] = codes_to_w8_r1(q.z, s2, ne1024, ne64); b[3] = codes_to_w8_r1(q.w, s2, ne1024, ne64);
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[k], b[k], acc[rt], 0, 0, 0);
            return;
        }
        _Float16 s16, zi, c16;
        if constexpr (META8) {              // scale = (code - m1) m0, zero = (code - m3) m2, in fp32; then as below
            const float sc = ((float)(um.m & 0xffu) - hi_half(um.quad0)) * lo_half(um.quad0);
            const float ze = ((float)(um.m >> 8) - hi_half(um.quad1)) * lo_half(um.quad1);
            const float zr = rintf(ze);
            s16 = (_Float16)sc; zi = (_Float16)zr; c16 = (_Float16)((zr - ze) * sc);
        } else {
            s16 = __builtin_bit_cast(_Float16, (uint16_t)(um.m & 0xffff));
            const _Float16 z16 = __builtin_bit_cast(_Float16, (uint16_t)(um.m >> 16));
            zi = __builtin_rintf16(z16);
            c16 = (zi - z16) * s16;
        }
        const _Float16 k1024 = (_Float16)-1024.f - zi, k64 = (_Float16)-64.f - zi;
        const h2_t s2 = {s16, s16}, c2 = {c16, c16}, b1024 = {k1024, k1024}, b64 = {k64, k64};
        h8_t b[4];
        b[0] = codes_to_w8(q.x, b1024, b64, s2, c2); b[1] = codes_to_w8(q.y, b1024, b64, s2, c2);
        b[2] = codes_to_w8(q.z, b1024, b64, s2, c2); b[3] = codes_to_w8(q.w, b1024, b64, s2, c2);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[j], b[j], acc[rt], 0, 0, 0);
    };
    uint4 q_next = make_uint4(0, 0, 0, 0);
    UnitMeta m_next = {0u, 0u, 0u};
    auto group_multiply = [&](const h8_t (&a)[4], int b, int gl, int sg, int j, auto &&beside) {   // q_next/m_next hold tile 0 of group gl
#pragma unroll
        for (int rt = 0; rt < TL_RT; ++rt) {
            const uint4 q = q_next;
            const UnitMeta m = m_next;
            if (rt + 1 < TL_RT) unit_load(b, gl, rt + 1, q_next, m_next);
            else if (gl + TL_WAVES < sg) unit_load(b, gl + TL_WAVES, 0, q_next, m_next);
            beside(j * TL_RT + rt);
            unit_multiply(a, q, m, rt, j);
        }
    };
    // R1: add sum over (group, bias, half) of d * (partial activation sum): slots 0..3 of each half of the K dimension
    auto rank1_correct = [&](const h8_t (&a)[TL_GPW][4]) {
        static_assert(TL_GPW == 2, "the correction packs two groups per wave and step");
        const u32x4_t av = {half_sums(a[0]), half_sums(a[1]), 0u, 0u};
#pragma unroll
        for (int rt = 0; rt < TL_RT; ++rt) {
            const u32x4_t bv = {rho[rt][0], rho[rt][1], 0u, 0u};
            acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8_t, av), __builtin_bit_cast(h8_t, bv), acc[rt], 0, 0, 0);
        }
    };

    // ---------------- end of an item: add the eight waves' partial sums, finish, store ----------------
    // Rounds of two tiles each through LDS buffer b (free: every wave is past its last read of it).  In a round
    // the waves share the 2 x 16 accumulator registers evenly: wave v owns TL_NI consecutive ones of one tile.
    auto finish_item = [&](const TileStep &s, int b) {
        float *red = reinterpret_cast<float *>(lds + b * TL_BUF_BYTES);   // [wave][tile of the round][16][64]
        const MfmaEntry &en = A.e[s.e];
        const int t = wv / (TL_WAVES / 2), i0 = (wv % (TL_WAVES / 2)) * TL_NI;   // tile of the round, first register
        int dst[TL_NI];
        float wgt[TL_NI];
        const int part = s.it % A.k_parts;
#pragma unroll
        for (int ii = 0; ii < TL_NI; ++ii) {
            const int i = i0 + ii;
            const int tk = en.first + min(8 * (i / 4) + 4 * kh + (i % 4), en.n_tok - 1);
            // w1/w3: row of a; w2: row of ypart -- the pair's own, or its part's row when the contraction is split
            dst[ii] = W13 ? l_pair[tk] : (A.k_parts == 1 ? (int)l_pair[tk] : A.part_base + tk * A.k_parts + part);
            wgt[ii] = W13 ? 0.f : l_w[tk];
        }
        if (!W13 && s.rb == 0 && part == 0 && tid < en.n_tok) {      // one block per entry tells k_combine where the rows are
            const int tk = en.first + tid;
            const int row = A.k_parts == 1 ? (int)l_pair[tk] : A.part_base + tk * A.k_parts;
            A.ytab[l_pair[tk]] = y_rows((uint32_t)(row + A.row_bias), (uint32_t)A.k_parts);
        }
#pragma unroll
        for (int round = 0; round < TL_RT / 2; ++round) {
            __syncthreads();                                         // buffer free (first round) / previous round read
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    red[((wv * 2 + t) * 16 + i) * 64 + lane] = acc[round * 2 + t][i];
                    acc[round * 2 + t][i] = 0.f;
                }
            __syncthreads();
            const int mrow = s.rb * TL_ROWS + (round * 2 + t) * 32 + col;
#pragma unroll
            for (int ii = 0; ii < TL_NI; ++ii) {
                const int i = i0 + ii;
                float v = 0.f;
#pragma unroll
                for (int w = 0; w < TL_WAVES; ++w) v += red[((w * 2 + t) * 16 + i) * 64 + lane];
                const int tok = 8 * (i / 4) + 4 * kh + (i % 4);
                if (W13) {
                    const float other = dpp_f<0xB1>(v);              // neighbouring column: v of the pair for even lanes
                    if ((lane & 1) == 0 && tok < en.n_tok && mrow < n_rows)
                        A.a[(size_t)dst[ii] * A.N + (mrow >> 1)] = __builtin_bit_cast(uint16_t, (_Float16)silu_mul(v, other));
                } else if (tok < en.n_tok && mrow < n_rows) {
                    A.ypart[(size_t)dst[ii] * A.N + mrow] = wgt[ii] * v;
                }
            }
        }
    };

    // ---------------- one step; true when it was the block's last ----------------
    auto step = [&](const h8_t (&a_use)[TL_GPW][4], h8_t (&a_load)[TL_GPW][4]) -> bool {
        const bool item_ends = !nxt.valid || nxt.it != cur.it;
        const TileStep &ld = nxt.valid ? nxt : cur;                  // past the last step: 16 bytes re-read, never used
        const FetchCtx f = fetch_begin(ld, nxt.valid);
        auto beside = [&](int u) { load_piece(f, a_load, ld, u); };
        const int sg = seg_groups(cur);
        if (wv < sg) {
            unit_load(buf, wv, 0, q_next, m_next);
            group_multiply(a_use[0], buf, wv, sg, 0, beside);
        } else {
#pragma unroll
            for (int u = 0; u < TL_RT; ++u) beside(u);
        }
        if (wv + TL_WAVES < sg) {
            group_multiply(a_use[1], buf, wv + TL_WAVES, sg, 1, beside);
        } else {
#pragma unroll
            for (int u = TL_RT; u < 2 * TL_RT; ++u) beside(u);
            if constexpr (R1) {
#pragma unroll
                for (int rt = 0; rt < TL_RT; ++rt) rho[rt][1] = 0u;  // no second group in a short step
            }
        }
        if constexpr (R1) {
            if (wv < sg) rank1_correct(a_use);
        }
        if (item_ends) finish_item(cur, buf);
        // unconditional (after the last step it stores a copy nobody reads): the wait for the loads above
        // then sits on every path, and the next step starts with nothing in flight as far as the compiler can tell
        commit(buf ^ 1);
        __syncthreads();                                             // next buffer filled, this one free again
        if (!nxt.valid) return true;
        cur = nxt;
        nxt = next(cur);
        buf ^= 1;
        return false;
    };

    h8_t a0[TL_GPW][4], a1[TL_GPW][4];
    {
        const FetchCtx f = fetch_begin(cur, true);
#pragma unroll
        for (int u = 0; u < TL_CP; ++u) load_piece(f, a0, cur, u);
    }
    commit(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);                              // vmcnt(0): the loop starts with nothing in flight
    __syncthreads();
    while (true) {
        if (step(a0, a1)) break;
        if (step(a1, a0)) break;
    }
}

}  // namespace moe
