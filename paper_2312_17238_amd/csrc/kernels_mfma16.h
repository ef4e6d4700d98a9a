// Grouped dequantize+GEMM on the matrix cores for FEW tokens per expert: the streaming kernel of
// kernels_mfma_stream.h with the token side of the tile cut from 32 to 16 (v_mfma_f32_16x16x32_f16).
//
// At batch 16 with top-2 an expert sees four tokens on average: a 32-token tile is seven eighths padding, costs 64
// accumulator registers per wave and two 16-byte A-operand loads per token row and group that touch 32 cache lines
// each.  Here the tile is MT x 16 tokens (MT = 1 while no expert of the launch has more than 16 tokens, else 2):
// 8 x MT x 4 accumulator registers for the same 128 memory rows of an item, one A operand of 16 bytes per lane,
// k-step and token tile (lanes of one token read 64 consecutive bytes), and half the matrix instructions' work.
//
// Items, steps of 8 groups, the two LDS buffers, the fixed-order reduction of the waves' partial sums through the
// buffer just consumed and the epilogues are the streaming kernel's.  The weights are dequantised as in its form 2
// (exact q - rint(z), one fused multiply-add, one rounding to fp16; fp16 (scale, zero) pairs) unless GS is set.
//
// Loads: two steps of weights are on their way at any time.  While step n is multiplied out of one LDS buffer, step
// n + 1 sits in (or is still arriving in) the staging registers; beside the (group, tile) units of step n's multiply
// it is written to the other buffer piece by piece, each register taking a piece of step n + 2 as soon as it is free
// (staged all at once after the multiply, the waves of a compute unit queue for its one path to memory for as long as
// the multiply took).  A step's loads so have a whole step to arrive and a block never has less than a step's bytes
// in flight.  That fits 128 registers because an address is a buffer descriptor and an offset in scalar registers
// plus ONE 32-bit vector register, and because nothing is read ahead from LDS.  The loop has ONE body, the A operands
// of the next step handed over by register copies at its end: with two alternating copies of the body the compiler's
// placement of the waits for loads merges the paths through both and makes every second step wait for everything in
// flight; for the same reason no load sits behind a branch (an offset past the buffer's end makes one a no-op).
//
// GS ("group-scaled"): the weights are not dequantised at all.  The codes enter the matrix cores as the fp16 numbers
// 1024 + q and 64 + q that the bit patterns 0x6400 | q and 0x5400 | q << 4 spell (one v_and_or_b32 per pair, nothing
// else per weight).  Per group and token tile, four matrix instructions against constant B operands give, in fp32 and
// already in the accumulators' layout, X = the sum of the group's activations per token (B all ones) and
// -P = -(1024 X_a + 64 X_b), X_a and X_b the sums over the k-slots that meet a code with bias 1024 and 64 (B = -1024
// and -64 in those slots).  A (sub-tile, group) product then starts from -P instead of zero, which takes the biases out
// again, and two fp32 multiply-adds per accumulator register finish it: total += s (product - z X).  No weight is
// rounded to fp16, nothing depends on the size of the activations (every sum is an fp32 one), 18 vector instructions
// per (sub-tile, group) instead of 42.  With two-level metadata (META8) scale and zero are decoded in fp32 right there.
//
// MFMA layouts (v_mfma_f32_16x16x32_f16): A lane l = row (token) l%16, k-slots 8*(l/16)..+7; B lane l = column (memory
// row) l%16, k-slots 8*(l/16)..+7; D lane l, register i = row 4*(l/16) + i, column l%16.
#pragma once
#include "kernels_mfma_stream.h"

namespace moe {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int T16_ST = TL_ROWS / 16;                     // 16-row sub-tiles per item (8)

// The masks and exponent patterns of the code -> fp16 trick as values the compiler cannot see through: with the mask
// in a scalar and the pattern in a vector register it then selects one v_and_or_b32 per pair by itself.  The inline
// assembly of and_or() must not feed a matrix instruction directly: the compiler does not know that it writes a
// vector register and leaves out the two wait states that such a write needs before a matrix instruction reads it.
struct BiasPatterns { uint32_t m_lo, m_hi, k1024, k64; };
__device__ __forceinline__ BiasPatterns bias_patterns()
{
    BiasPatterns p = {0x000F000Fu, 0x00F000F0u, 0x64006400u, 0x54005400u};
    asm("" : "+s"(p.m_lo), "+s"(p.m_hi), "+v"(p.k1024), "+v"(p.k64));
    return p;
}

// eight codes as the fp16 numbers bias + q: slots 0, 1, 4, 5 with bias 1024, slots 2, 3, 6, 7 with bias 64
__device__ __forceinline__ h8_t codes_biased(uint32_t w, const BiasPatterns &p)
{
    const uint32_t hi = w >> 8;
    const u32x4_t r = {(w & p.m_lo) | p.k1024, (w & p.m_hi) | p.k64, (hi & p.m_lo) | p.k1024, (hi & p.m_hi) | p.k64};
    return __builtin_bit_cast(h8_t, r);
}

// WAVES: 4 (a wave multiplies two groups of a step) or 8 (one group; half the staging and A-operand registers per
// lane, so that two blocks of 8 waves fit a compute unit: four waves per SIMD, which is the second launch bound).
// META8 (GS only): two-level metadata (Sec. 4.2 "scale group size").  A step then stages, per row, 16 bytes of (scale
// code, zero code) byte pairs and the fp16 quad of the run the step lies in, and a unit decodes scale and zero in fp32
// -- which is where the group-scaled arithmetic wants them anyway.
template <bool W13, int MT, int WAVES, bool GS = false, bool META8 = false>
__global__ __launch_bounds__(WAVES *WAVE, (WAVES == 8 && MT == 1 ? 4 : 2)) void k_mfma_stream16_q4(TileArgs A)
{
    static_assert(GS || !META8, "two-level metadata is decoded in fp32: group-scaled arithmetic only");
    static_assert(MT == 1 || MT == 2, "one or two token tiles of 16");
    static_assert(WAVES == 4 || WAVES == 8, "four or eight waves per block");
    constexpr int THREADS = WAVES * WAVE;
    constexpr int GPW = TL_SG / WAVES;                               // groups per wave and step
    constexpr int CP = TL_ROWS * TL_CPR / THREADS;                   // code pieces per thread and step
    static_assert(GPW * WAVES == TL_SG && CP == GPW * TL_RT, "pieces and units must pair up");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wv = uniform(tid >> 6);
    const int col = lane & 15, kb = lane >> 4;           // memory row (B) / token (A) of the tile; block of 8 k-slots
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
    int addr_it = -1;
    // the item's matrix as a buffer: a load's address is this scalar descriptor, a scalar offset and ONE 32-bit vector
    // register, instead of 64-bit arithmetic in vector registers per load (a matrix is far below 4 GB)
    __amdgpu_buffer_rsrc_t mat_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(A.e[0].blob), 0, 0, 0x00020000);
    // The activations as a buffer too: a lane whose token does not exist carries an offset past the buffer's end, for
    // which the hardware returns zeros without a request -- at four tokens per expert three quarters of the A operand's
    // lanes, whose 16 bytes each would otherwise cross the compute unit's path to memory like any others.
    constexpr uint32_t ACT_RANGE = 0x7fffff00u, ACT_NONE = 0x80000000u;       // no offset of a load wraps around
    const __amdgpu_buffer_rsrc_t act_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(A.act), 0, (int)ACT_RANGE, 0x00020000);
    uint32_t act_off[MT];                                            // bytes: token row of act + this lane's block of 8 k-slots
    auto enter_item = [&](const TileStep &s) {
        if (s.it == addr_it) return;
        addr_it = s.it;
        const MfmaEntry &en = A.e[s.e];
        mat_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(en.blob + A.mat_off), 0, n_rows * (int)A.stride, 0x00020000);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const bool live = mt * 16 + col < en.n_tok;
            const int tk = live ? mt * 16 + col : 0;
            const int row = W13 ? l_tok[en.first + tk] : l_pair[en.first + tk];
            act_off[mt] = live ? (uint32_t)row * (uint32_t)A.K * 2u + (uint32_t)kb * 16u : ACT_NONE;
        }
    };

    // ---------------- weights: HBM -> registers -> LDS (as in the streaming kernel) ----------------
    uint4 st_c[CP], st_m;
    struct FetchCtx { uint32_t voff; int row0, slab, g0, sg; bool live; };
    constexpr int SLAB = THREADS / TL_CPR;
    static_assert(THREADS % TL_CPR == 0 && 64 % SLAB == 0, "a slab of rows lies wholly inside or outside a matrix of 64 k rows");
    auto fetch_begin = [&](const TileStep &s, bool live) -> FetchCtx {
        enter_item(s);
        FetchCtx f;
        f.live = live;
        f.g0 = s.seg * TL_SG; f.sg = seg_groups(s);
        f.row0 = live ? s.rb * TL_ROWS : 0;
        f.slab = live ? SLAB : 0;
        const uint32_t c = tid % TL_CPR;
        f.voff = live ? (uint32_t)(tid / TL_CPR) * A.stride + ((int)c < 2 * f.sg ? c : 0u) * 16u : 0u;
        return f;
    };
    auto fetch_codes = [&](const FetchCtx &f, int i) {
        const int soff = f.g0 * 32 + min(f.row0 + i * f.slab, n_rows - SLAB) * (int)A.stride;
        const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(mat_rsrc, (int)f.voff, soff, 2);     // 2: non-temporal
        st_c[i] = make_uint4(v.x, v.y, v.z, v.w);
    };
    auto commit_codes = [&](int b, int i) {
        uint8_t *codes = lds + b * TL_BUF_BYTES;
        const int p = tid + i * THREADS, r = p / TL_CPR, c = p % TL_CPR;
        *reinterpret_cast<uint4 *>(codes + r * TL_CODE_PITCH + c * 16) = st_c[i];
    };
    // pairs: 32 bytes per row and step, shared evenly by the block's threads (8 bytes each with 8 waves, 16 with 4);
    // pieces past the row's last group repeat the step's first
    constexpr int MW = TL_ROWS * TL_SG / THREADS;                    // words per thread: 2 or 4
    static_assert(MW == 2 || MW == 4, "a thread holds 8 or 16 bytes of pairs");
    auto fetch_meta = [&](const FetchCtx &f) {
        const int r = f.live ? tid / (TL_SG / MW) : 0, c = tid % (TL_SG / MW);
        int voff = min(f.row0 + r, n_rows - 1) * (int)A.stride, soff;
        if constexpr (META8) {
            // words 0..3 of the staged row: the step's 8 byte pairs; words 4, 5: the quad of its run; the rest is not read
            static_assert(TL_SG == 8, "two-level staging is laid out for steps of 8 groups");
            const int quad = (int)A.meta2_off + 8 * (f.g0 >> A.run_shift), pairs = (int)A.meta_off + f.g0 * 2;
            if constexpr (MW == 2) voff = c == 3 ? (int)0x80000000u : voff + (c == 2 ? quad : pairs + c * 8);
            else voff += c == 1 ? quad : pairs;
            soff = 0;
        } else {
            voff += (c * MW < f.sg ? c : 0) * (MW * 4);
            soff = (int)A.meta_off + f.g0 * 4;
        }
        if constexpr (MW == 2) {
            const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(mat_rsrc, voff, soff, 0);
            st_m.x = v.x; st_m.y = v.y;
        } else {
            const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(mat_rsrc, voff, soff, 0);
            st_m = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    auto commit_meta = [&](int b) {
        uint32_t *meta = reinterpret_cast<uint32_t *>(lds + b * TL_BUF_BYTES + TL_ROWS * TL_CODE_PITCH);
        uint32_t *d = meta + (tid / (TL_SG / MW)) * TL_META_PITCH + (tid % (TL_SG / MW)) * MW;
        d[0] = st_m.x; d[1] = st_m.y;
        if constexpr (MW == 4) { d[2] = st_m.z; d[3] = st_m.w; }
    };

    // ---------------- multiply ----------------
    f32x4_t acc[T16_ST][MT];
#pragma unroll
    for (int st = 0; st < T16_ST; ++st)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[st][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // A operands of one group: [token tile][k-step]; piece q = mt * 2 + kk
    auto load_a_piece = [&](h8_t (&dst)[GPW][2 * MT], const TileStep &s, int j, int q) {
        const int g = s.seg * TL_SG + min(wv + WAVES * j, seg_groups(s) - 1);
        dst[j][q] = __builtin_bit_cast(h8_t, __builtin_amdgcn_raw_buffer_load_b128(act_rsrc, (int)act_off[q >> 1], g * 128 + (q & 1) * 64, 0));
    };
    static_assert(TL_RT == 4, "four 32-row tiles per item");
    // One unit = one group of one 32-row tile = two 16-row sub-tiles; its code words (two per sub-tile: this lane's
    // block of 8 k-slots in each half of the group) and pairs are read from LDS one unit ahead of their use.
    struct UnitRegs { uint32_t q[2][2], m[2], quad[2][2]; };         // m: the (scale, zero) pair, fp16 or (META8) bytes; quad: META8 only
    auto unit_load = [&](int b, int gl, int rt, UnitRegs &u) {
        const uint8_t *codes = lds + b * TL_BUF_BYTES;
        const uint32_t *meta = reinterpret_cast<const uint32_t *>(codes + TL_ROWS * TL_CODE_PITCH);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int r = rt * 32 + h * 16 + col;
            const uint32_t *w = reinterpret_cast<const uint32_t *>(codes + r * TL_CODE_PITCH + gl * 32);
            u.q[h][0] = w[kb];
            u.q[h][1] = w[4 + kb];
            if constexpr (META8) {
                u.m[h] = (meta[r * TL_META_PITCH + (gl >> 1)] >> (16 * (gl & 1))) & 0xffffu;
                u.quad[h][0] = meta[r * TL_META_PITCH + 4];
                u.quad[h][1] = meta[r * TL_META_PITCH + 5];
            } else {
                u.m[h] = meta[r * TL_META_PITCH + gl];
            }
        }
    };
    // GS: per token of the lane's accumulator rows, the group's activation sum and minus the biases' share
    f32x4_t g_x[MT], g_negp[MT];
    const BiasPatterns bp = bias_patterns();
    auto group_sums = [&](const h8_t (&a)[2 * MT]) {
        const u32x4_t ones = {0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};       // 1, 1, ...
        const u32x4_t negb = {0xE400E400u, 0xD400D400u, 0xE400E400u, 0xD400D400u};       // -1024, -1024, -64, -64, ...
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
            g_x[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt * 2], __builtin_bit_cast(h8_t, ones), zero, 0, 0, 0);
            g_x[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt * 2 + 1], __builtin_bit_cast(h8_t, ones), g_x[mt], 0, 0, 0);
            g_negp[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt * 2], __builtin_bit_cast(h8_t, negb), zero, 0, 0, 0);
            g_negp[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt * 2 + 1], __builtin_bit_cast(h8_t, negb), g_negp[mt], 0, 0, 0);
        }
    };
    auto unit_multiply = [&](const h8_t (&a)[2 * MT], const UnitRegs &u, int rt) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if constexpr (GS) {
                float s32, nz32;
                if constexpr (META8) {          // scale = (code - m1) m0, zero = (code - m3) m2, in fp32
                    s32 = ((float)(u.m[h] & 0xffu) - hi_half(u.quad[h][0])) * lo_half(u.quad[h][0]);
                    nz32 = (hi_half(u.quad[h][1]) - (float)(u.m[h] >> 8)) * lo_half(u.quad[h][1]);
                } else {
                    s32 = (float)__builtin_bit_cast(_Float16, (uint16_t)(u.m[h] & 0xffff));
                    nz32 = -(float)__builtin_bit_cast(_Float16, (uint16_t)(u.m[h] >> 16));
                }
                const h8_t b0 = codes_biased(u.q[h][0], bp), b1 = codes_biased(u.q[h][1], bp);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    f32x4_t g = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt * 2], b0, g_negp[mt], 0, 0, 0);
                    g = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt * 2 + 1], b1, g, 0, 0, 0);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        acc[rt * 2 + h][mt][i] = __builtin_fmaf(s32, __builtin_fmaf(nz32, g_x[mt][i], g[i]), acc[rt * 2 + h][mt][i]);
                }
                continue;
            }
            const _Float16 s16 = __builtin_bit_cast(_Float16, (uint16_t)(u.m[h] & 0xffff));
            const _Float16 z16 = __builtin_bit_cast(_Float16, (uint16_t)(u.m[h] >> 16));
            const _Float16 zi = __builtin_rintf16(z16);
            const _Float16 c16 = (zi - z16) * s16;
            const _Float16 k1024 = (_Float16)-1024.f - zi, k64 = (_Float16)-64.f - zi;
            const h2_t s2 = {s16, s16}, c2 = {c16, c16}, b1024 = {k1024, k1024}, b64 = {k64, k64};
            const h8_t b0 = codes_to_w8(u.q[h][0], b1024, b64, s2, c2), b1 = codes_to_w8(u.q[h][1], b1024, b64, s2, c2);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc[rt * 2 + h][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt * 2], b0, acc[rt * 2 + h][mt], 0, 0, 0);
                acc[rt * 2 + h][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt * 2 + 1], b1, acc[rt * 2 + h][mt], 0, 0, 0);
            }
        }
    };
    auto group_multiply = [&](const h8_t (&a)[2 * MT], int b, int gl, int j, auto &&beside) {
        if constexpr (GS) group_sums(a);
#pragma unroll
        for (int rt = 0; rt < TL_RT; ++rt) {
            UnitRegs u;
            unit_load(b, gl, rt, u);
            beside(j * TL_RT + rt);
            unit_multiply(a, u, rt);
        }
    };

    // ---------------- end of an item: add the four waves' partial sums, finish, store ----------------
    // Rounds through LDS buffer b (free: every wave is past its last read of it).  A round takes RS sub-tiles of one
    // token tile: every wave writes its RS x 4 registers of them, then the RS x 4 registers are shared evenly among
    // the waves, wave v adding all waves' values of NI consecutive ones, always in the order of the waves.
    constexpr int RS = WAVES == 4 ? T16_ST : T16_ST / 2;             // sub-tiles per round
    constexpr int NI = RS * 4 / WAVES;                               // registers a wave finishes per round (8 or 2)
    static_assert(WAVES * RS * 4 * 64 * 4 <= TL_BUF_BYTES && NI * WAVES == RS * 4 && 4 % (NI < 4 ? NI : 4) == 0, "one reduction round must fit a staging buffer");
    auto finish_item = [&](const TileStep &s, int b) {
        float *red = reinterpret_cast<float *>(lds + b * TL_BUF_BYTES);   // [wave][sub-tile of the round][4][64]
        const MfmaEntry &en = A.e[s.e];
        const int part = s.it % A.k_parts;
        if (!W13 && s.rb == 0 && part == 0 && tid < en.n_tok) {      // one block per entry tells k_combine where the rows are
            const int tk = en.first + tid;
            const int row = A.k_parts == 1 ? (int)l_pair[tk] : A.part_base + tk * A.k_parts;
            A.ytab[l_pair[tk]] = y_rows((uint32_t)(row + A.row_bias), (uint32_t)A.k_parts);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r0 = 0; r0 < T16_ST; r0 += RS) {
                __syncthreads();                                     // buffer free (first round) / previous round read
#pragma unroll
                for (int sl = 0; sl < RS; ++sl)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        red[((wv * RS + sl) * 4 + i) * 64 + lane] = acc[r0 + sl][mt][i];
                        acc[r0 + sl][mt][i] = 0.f;
                    }
                __syncthreads();
#pragma unroll
                for (int ii = 0; ii < NI; ++ii) {
                    const int flat = wv * NI + ii, sl = flat / 4, i = flat % 4;
                    const int mrow = s.rb * TL_ROWS + (r0 + sl) * 16 + col;
                    float v = 0.f;
#pragma unroll
                    for (int w = 0; w < WAVES; ++w) v += red[((w * RS + sl) * 4 + i) * 64 + lane];
                    const int tok = mt * 16 + 4 * kb + i;            // token of the entry this register belongs to
                    const int tk = en.first + min(tok, en.n_tok - 1);
                    if (W13) {
                        const float other = dpp_f<0xB1>(v);          // neighbouring column: v of the pair for even lanes
                        if ((lane & 1) == 0 && tok < en.n_tok && mrow < n_rows)
                            A.a[(size_t)l_pair[tk] * A.N + (mrow >> 1)] = __builtin_bit_cast(uint16_t, (_Float16)silu_mul(v, other));
                    } else if (tok < en.n_tok && mrow < n_rows) {
                        const int dst = A.k_parts == 1 ? (int)l_pair[tk] : A.part_base + tk * A.k_parts + part;
                        A.ypart[(size_t)dst * A.N + mrow] = l_w[tk] * v;
                    }
                }
            }
    };

    // ---------------- the steps ----------------
    h8_t a0[GPW][2 * MT], a1[GPW][2 * MT];                           // this step's A operands, the next step's
    auto load_a = [&](h8_t (&dst)[GPW][2 * MT], const TileStep &s) {
#pragma unroll
        for (int j = 0; j < GPW; ++j)
#pragma unroll
            for (int q = 0; q < 2 * MT; ++q) load_a_piece(dst, s, j, q);
    };
    TileStep nxt2 = next(nxt);
    {
        const FetchCtx f = fetch_begin(cur, true);
        fetch_meta(f);
#pragma unroll
        for (int i = 0; i < CP; ++i) fetch_codes(f, i);
        load_a(a0, cur);
    }
#pragma unroll
    for (int i = 0; i < CP; ++i) commit_codes(0, i);
    commit_meta(0);
    // Everything of step 0 has arrived before step 1 is requested: the compiler places the waits inside the loop from
    // the order in which loads can be outstanding on ANY path into it.
    __builtin_amdgcn_s_waitcnt(0x0F70);                              // vmcnt(0)
    {
        const TileStep &ld = nxt.valid ? nxt : cur;                  // past the last step: 16 bytes re-read, never used
        const FetchCtx f = fetch_begin(ld, nxt.valid);
        fetch_meta(f);
#pragma unroll
        for (int i = 0; i < CP; ++i) fetch_codes(f, i);
        load_a(a1, ld);
    }
    __syncthreads();
    while (true) {
        const bool item_ends = !nxt.valid || nxt.it != cur.it;
        const int sg = seg_groups(cur);
        // step n + 1 from the registers into the other buffer, step n + 2 into the registers
        const TileStep &ld = nxt2.valid ? nxt2 : cur;                // past the last step: 16 bytes re-read, never used
        const FetchCtx f = fetch_begin(ld, nxt2.valid);
        auto beside = [&](int u) {                                   // one piece beside each (group, tile) unit of the multiply
            if (u == 0) {
                commit_meta(buf ^ 1);
                fetch_meta(f);
            }
            commit_codes(buf ^ 1, u);
            fetch_codes(f, u);
        };
#pragma unroll
        for (int j = 0; j < GPW; ++j) {
            if (wv + WAVES * j < sg) {
                group_multiply(a0[j], buf, wv + WAVES * j, j, beside);
            } else {
#pragma unroll
                for (int u = j * TL_RT; u < (j + 1) * TL_RT; ++u) beside(u);
            }
        }
        if (item_ends) finish_item(cur, buf);
#pragma unroll
        for (int j = 0; j < GPW; ++j)
#pragma unroll
            for (int q = 0; q < 2 * MT; ++q) {
                a0[j][q] = a1[j][q];
                // the copy is made HERE, before its source takes a new load: left to itself the compiler loads into
                // fresh registers and copies at the top of the next step, behind a wait for the newest load
                asm volatile("" : "+v"(a0[j][q]));
            }
        load_a(a1, ld);
        __syncthreads();                                             // next buffer filled, this one free again
        if (!nxt.valid) break;
        cur = nxt;
        nxt = nxt2;
        nxt2 = next(nxt2);
        buf ^= 1;
    }
}

}  // namespace moe
