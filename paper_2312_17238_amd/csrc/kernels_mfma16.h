// Grouped dequantize+GEMM on the matrix cores for FEW tokens per expert: the streaming kernel of
// kernels_mfma_stream.h with the token side of the tile cut from 32 to 16 (v_mfma_f32_16x16x32_f16).
//
// At batch 16 with top-2 an expert sees four tokens on average: a 32-token tile is seven eighths padding, costs 64
// accumulator registers per wave and two 16-byte A-operand loads per token row and group that touch 32 cache lines
// each.  Here the tile is MT x 16 tokens (MT = 1 while no expert of the launch has more than 16 tokens, else 2):
// 8 x MT x 4 accumulator registers for the same 128 memory rows of an item, one A operand of 16 bytes per lane,
// k-step and token tile (lanes of one token read 64 consecutive bytes), and half the matrix instructions' work.
//
// Everything around the multiply is the streaming kernel's: items, steps of 8 groups, HBM -> registers -> LDS copies in
// eight pieces beside the units of the multiply, one barrier per step, partial sums of the four waves added through
// the LDS buffer just consumed in a fixed order, the same epilogues.  The weights are dequantised as in its form 2
// (exact q - rint(z), one fused multiply-add, one rounding to fp16; fp16 (scale, zero) pairs).
//
// MFMA layouts (v_mfma_f32_16x16x32_f16): A lane l = row (token) l%16, k-slots 8*(l/16)..+7; B lane l = column (memory
// row) l%16, k-slots 8*(l/16)..+7; D lane l, register i = row 4*(l/16) + i, column l%16.
#pragma once
#include "kernels_mfma_stream.h"

namespace moe {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int T16_ST = TL_ROWS / 16;                     // 16-row sub-tiles per item (8)

// WAVES: 4 (a wave multiplies two groups of a step) or 8 (one group; half the staging and A-operand registers per
// lane, so that two blocks of 8 waves fit a compute unit: four waves per SIMD).
template <bool W13, int MT, int WAVES>
__global__ __launch_bounds__(WAVES *WAVE, TL_BLOCKS_PER_CU) void k_mfma_stream16_q4(TileArgs A)
{
    static_assert(MT == 1 || MT == 2, "one or two token tiles of 16");
    static_assert(WAVES == 4 || WAVES == 8, "four or eight waves per block");
    constexpr int THREADS = WAVES * WAVE;
    constexpr int GPW = TL_SG / WAVES;                               // groups per wave and step
    constexpr int CP = TL_ROWS * TL_CPR / THREADS;                   // code pieces per thread and step
    constexpr int MPIECES = TL_ROWS * TL_MPR;                        // pair pieces per step, at most one per thread
    static_assert(GPW * WAVES == TL_SG && CP == GPW * TL_RT && MPIECES <= THREADS, "pieces and units must pair up");
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
    const uint8_t *mat_base = nullptr;
    uint32_t act_off[MT];                                            // bytes: token row of act + this lane's block of 8 k-slots
    auto enter_item = [&](const TileStep &s) {
        if (s.it == addr_it) return;
        addr_it = s.it;
        const MfmaEntry &en = A.e[s.e];
        mat_base = en.blob + A.mat_off;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {                            // lanes past the last token read the first again
            const int tk = mt * 16 + col < en.n_tok ? mt * 16 + col : 0;
            const int row = W13 ? l_tok[en.first + tk] : l_pair[en.first + tk];
            act_off[mt] = (uint32_t)row * (uint32_t)A.K * 2u + (uint32_t)kb * 16u;
        }
    };

    // ---------------- weights: HBM -> registers -> LDS (as in the streaming kernel) ----------------
    uint4 st_c[CP], st_m;
    struct FetchCtx { const uint8_t *seg; uint32_t voff; int row0, slab, g0, sg; bool live; };
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
        f.seg = mat_base + (size_t)f.g0 * 32;
        return f;
    };
    auto fetch_codes = [&](const FetchCtx &f, int i) {
        st_c[i] = ldw4(f.seg + (size_t)min(f.row0 + i * f.slab, n_rows - SLAB) * A.stride + f.voff, 0);
    };
    auto fetch_meta = [&](const FetchCtx &f) {                       // threads past the last piece repeat the last row's
        const int p = min(tid, MPIECES - 1), r = f.live ? p / TL_MPR : 0, c = p % TL_MPR;
        const uint8_t *rowp = mat_base + (size_t)min(f.row0 + r, n_rows - 1) * A.stride;
        st_m = reinterpret_cast<const uint4 *>(rowp + A.meta_off)[f.g0 / 4 + (c < (f.sg + 3) / 4 ? c : 0)];
    };
    auto commit = [&](int b) {
        uint8_t *codes = lds + b * TL_BUF_BYTES;
        uint32_t *meta = reinterpret_cast<uint32_t *>(codes + TL_ROWS * TL_CODE_PITCH);
#pragma unroll
        for (int i = 0; i < CP; ++i) {
            const int p = tid + i * THREADS, r = p / TL_CPR, c = p % TL_CPR;
            *reinterpret_cast<uint4 *>(codes + r * TL_CODE_PITCH + c * 16) = st_c[i];
        }
        if (tid < MPIECES) {
            const int r = tid / TL_MPR, c = tid % TL_MPR;
            uint32_t *d = meta + r * TL_META_PITCH + c * 4;
            d[0] = st_m.x; d[1] = st_m.y; d[2] = st_m.z; d[3] = st_m.w;
        }
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
        const uint8_t *grp = reinterpret_cast<const uint8_t *>(A.act) + (size_t)g * 128 + (q & 1) * 64;
        dst[j][q] = __builtin_bit_cast(h8_t, *reinterpret_cast<const uint4 *>(grp + act_off[q >> 1]));
    };
    static_assert(TL_RT == 4, "four 32-row tiles per item");
    auto load_piece = [&](const FetchCtx &f, h8_t (&a_dst)[GPW][2 * MT], const TileStep &s, int u) {
        if (u % TL_RT < 2 * MT) load_a_piece(a_dst, s, u / TL_RT, u % TL_RT);
        if (u == 0) fetch_meta(f);
        fetch_codes(f, u);
    };
    // One unit = one group of one 32-row tile = two 16-row sub-tiles; its code words (two per sub-tile: this lane's
    // block of 8 k-slots in each half of the group) and pairs are read from LDS one unit ahead of their use.
    struct UnitRegs { uint32_t q[2][2], m[2]; };
    auto unit_load = [&](int b, int gl, int rt, UnitRegs &u) {
        const uint8_t *codes = lds + b * TL_BUF_BYTES;
        const uint32_t *meta = reinterpret_cast<const uint32_t *>(codes + TL_ROWS * TL_CODE_PITCH);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int r = rt * 32 + h * 16 + col;
            const uint32_t *w = reinterpret_cast<const uint32_t *>(codes + r * TL_CODE_PITCH + gl * 32);
            u.q[h][0] = w[kb];
            u.q[h][1] = w[4 + kb];
            u.m[h] = meta[r * TL_META_PITCH + gl];
        }
    };
    auto unit_multiply = [&](const h8_t (&a)[2 * MT], const UnitRegs &u, int rt) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
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
    UnitRegs u_next = {};
    auto group_multiply = [&](const h8_t (&a)[2 * MT], int b, int gl, int sg, int j, auto &&beside) {   // u_next holds tile 0 of group gl
#pragma unroll
        for (int rt = 0; rt < TL_RT; ++rt) {
            const UnitRegs u = u_next;
            if (rt + 1 < TL_RT) unit_load(b, gl, rt + 1, u_next);
            else if (j + 1 < GPW && gl + WAVES < sg) unit_load(b, gl + WAVES, 0, u_next);
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

    // ---------------- one step; true when it was the block's last ----------------
    auto step = [&](const h8_t (&a_use)[GPW][2 * MT], h8_t (&a_load)[GPW][2 * MT]) -> bool {
        const bool item_ends = !nxt.valid || nxt.it != cur.it;
        const TileStep &ld = nxt.valid ? nxt : cur;                  // past the last step: 16 bytes re-read, never used
        const FetchCtx f = fetch_begin(ld, nxt.valid);
        auto beside = [&](int u) { load_piece(f, a_load, ld, u); };
        const int sg = seg_groups(cur);
        if (wv < sg) unit_load(buf, wv, 0, u_next);
#pragma unroll
        for (int j = 0; j < GPW; ++j) {
            if (wv + WAVES * j < sg) {
                group_multiply(a_use[j], buf, wv + WAVES * j, sg, j, beside);
            } else {
#pragma unroll
                for (int u = j * TL_RT; u < (j + 1) * TL_RT; ++u) beside(u);
            }
        }
        if (item_ends) finish_item(cur, buf);
        commit(buf ^ 1);
        __syncthreads();                                             // next buffer filled, this one free again
        if (!nxt.valid) return true;
        cur = nxt;
        nxt = next(cur);
        buf ^= 1;
        return false;
    };

    h8_t a0[GPW][2 * MT], a1[GPW][2 * MT];
    {
        const FetchCtx f = fetch_begin(cur, true);
#pragma unroll
        for (int u = 0; u < CP; ++u) load_piece(f, a0, cur, u);
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
