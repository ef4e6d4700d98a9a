// Grouped dequantize+GEMM on the matrix cores for batched decode: when several tokens are routed to the same
// expert the step is a real contraction, U[t][r] = sum_k h[t][k] W^[r][k] over the tokens t of that expert.
// 4-bit codes with group 64 (the batched configuration); other formats stay on the GEMV kernels.
//
// This file: the shared argument types, the exact integer conversion of the codes, and the row-staging kernel
// that scales every group's product in fp32 (GEMV-path accuracy).  The default, faster kernel is in
// kernels_mfma_stream.h.
//
// D layout of the 32x32 MFMA: lane l, register i  ->  row (token) m = 8*(i/4) + 4*(l/32) + i%4, column l%32.
#pragma once
#include "kernels_gemv.h"

namespace moe {

typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int MF_MAX_PAIRS = 256;            // (token, expert) pairs per step: batch * top_k

struct MfmaEntry {
    const uint8_t *blob;
    int32_t n_tok;                           // tokens routed to this expert (<= 64)
    int32_t first;                           // its slice of the pair tables
};

struct MfmaArgs {
    MfmaEntry e[16];
    uint8_t tok[MF_MAX_PAIRS];               // token (batch row) of each pair, grouped by expert
    uint8_t pair[MF_MAX_PAIRS];              // row of a[.][F] of each pair (= b*K + j)
    float w[MF_MAX_PAIRS];                   // combine weight of each pair
    const uint16_t *act;                     // w1/w3: h [B][H];   w2: a [B*K][F]
    uint16_t *a;                             // w1/w3 output
    float *ypart;                            // w2 output: row `pair` of [B*K][H] fp32 (k_combine adds a token's rows)
    uint32_t *ytab;                          // [B*K]: y_rows(pair, 1) for every pair of the launch
    int32_t K, N;                            // contraction length, output rows of the matrix
    uint32_t stride, meta_off;               // row stride and offset of the (scale, zero) pairs
    uint64_t mat_off;                        // byte offset of the matrix inside the blob
};

// 8 codes of one word as 8 exact fp16 integers, in the order of the contraction index
__device__ __forceinline__ h8_t codes_to_h8(uint32_t w)
{
    const h2_t m1024 = {(_Float16)-1024.f, (_Float16)-1024.f}, m64 = {(_Float16)-64.f, (_Float16)-64.f};
    const uint32_t hi = w >> 8;
    const h2_t t0 = as_h2(and_or(w, 0x000F000Fu, 0x64006400u)) + m1024;
    const h2_t t1 = as_h2(and_or(w, 0x00F000F0u, 0x54005400u)) + m64;
    const h2_t t2 = as_h2(and_or(hi, 0x000F000Fu, 0x64006400u)) + m1024;
    const h2_t t3 = as_h2(and_or(hi, 0x00F000F0u, 0x54005400u)) + m64;
    h8_t r;
    r[0] = t0.x; r[1] = t0.y; r[2] = t1.x; r[3] = t1.y; r[4] = t2.x; r[5] = t2.y; r[6] = t3.x; r[7] = t3.y;
    return r;
}

// ---------------------------------------------------------------------------------------------
// Row-streaming form.  HBM wants long contiguous reads (the GEMV kernels read whole rows); feeding the
// weights straight into the MFMA lane layout touches 32 bytes per row and instruction.  Here a block owns 32
// consecutive MEMORY rows of a matrix -- for w1/w3, whose rows are interleaved in the blob, that is 16 rows
// of each, one contiguous 74 KB range -- and copies them through registers into LDS with fully coalesced
// 16-byte pieces (long rows in segments of SEG groups), then every wave takes every fourth group of the
// segment: B operand from LDS (row l%32, half l/32 of the group), A operand (16 bytes of one token's
// activations per lane and MFMA) from L2, and the per-(token, group) sums of the activations from one more
// MFMA against a B operand of ones, so no table and no extra kernel is needed.  Columns of D are memory rows:
// for w1/w3 even columns hold u and odd columns v of the same output row.
// grid = (ceil(memory rows / 32), entries), 4 waves; two blocks per compute unit overlap copy and multiply.
// ---------------------------------------------------------------------------------------------

constexpr int MF2_WAVES = 4;
constexpr int MF2_SEG = 64;                  // groups staged per pass (4096 codes): 32 rows * 64 * 36 B = 72 KB

template <bool W13, int MT>
__global__ __launch_bounds__(MF2_WAVES *WAVE) void k_mfma_rows_q4(MfmaArgs A)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const MfmaEntry &en = A.e[blockIdx.y];
    const int tid = threadIdx.x, lane = tid & 63, wv = uniform(tid >> 6);
    const int col = lane & 31, kh = lane >> 5;
    const int n_rows = W13 ? 2 * A.N : A.N;                           // memory rows of the matrix
    const int row0 = blockIdx.x * 32;
    const int groups = A.K / 64;
    const int seg_groups = min(groups, MF2_SEG);
    const int code_pitch = seg_groups * 32 + 16;                      // bytes per staged row of codes (+16: bank spread)
    uint8_t *lds_codes = lds;                                         // [32][code_pitch]
    const int meta_pitch = (seg_groups + 3) & ~3;                     // pairs per staged row, 16-byte aligned
    uint32_t *lds_meta = reinterpret_cast<uint32_t *>(lds + 32 * code_pitch);   // [32][meta_pitch]
    const uint8_t *mat = en.blob + A.mat_off;

    f32x16_t acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
    h8_t ones;
#pragma unroll
    for (int i = 0; i < 8; ++i) ones[i] = (_Float16)1.f;
    // activation rows of this lane's token (A operand: lane l feeds token l%32 of the tile); lanes past the
    // entry's last token read its first token again, their results are never stored
    const uint16_t *arow[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int tk = t * 32 + col < en.n_tok ? t * 32 + col : 0;
        arow[t] = A.act + (size_t)(W13 ? A.tok[en.first + tk] : A.pair[en.first + tk]) * A.K;
    }
    auto load_a = [&](h8_t (&av)[MT][4], int g) {                     // one group's A operands for this lane's token(s)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                av[t][j] = __builtin_bit_cast(h8_t, *reinterpret_cast<const uint4 *>(arow[t] + (size_t)g * 64 + kh * 32 + j * 8));
    };
    auto multiply = [&](const h8_t (&av)[MT][4], int g) {             // group g of the staged segment
        const uint4 q = *reinterpret_cast<const uint4 *>(lds_codes + col * code_pitch + g * 32 + kh * 16);
        const uint32_t m = lds_meta[col * meta_pitch + g];
        const float sc = lo_half(m), z = hi_half(m);
        h8_t b[4];
        {
            b[0] = codes_to_h8(q.x); b[1] = codes_to_h8(q.y); b[2] = codes_to_h8(q.z); b[3] = codes_to_h8(q.w);
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                f32x16_t cg, chs;
#pragma unroll
                for (int i = 0; i < 16; ++i) { cg[i] = 0.f; chs[i] = 0.f; }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    cg = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[t][j], b[j], cg, 0, 0, 0);
                    chs = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[t][j], ones, chs, 0, 0, 0);
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[t][i] = fmaf(sc, fmaf(-z, chs[i], cg[i]), acc[t][i]);
            }
        }
    };
    constexpr int THREADS = MF2_WAVES * WAVE;
    constexpr int CP = MF2_SEG * 2 * 32 / THREADS;                    // code pieces per thread of a full segment (16)
    constexpr int MP = (MF2_SEG / 4 * 32 + THREADS - 1) / THREADS;    // pair pieces per thread (2)

    for (int g0 = 0; g0 < groups; g0 += seg_groups) {
        const int sg = min(seg_groups, groups - g0);
        // ---- copy 32 rows x sg groups (codes, then pairs) into LDS in 16-byte pieces, coalesced along each row.
        // All loads are issued before the first LDS store, so one HBM latency is paid per segment, not per piece.
        const int ppr = sg * 2, mpr = (sg + 3) / 4;                   // code / pair pieces per row
        uint4 stage[CP], mstage[MP];
#pragma unroll
        for (int i = 0; i < CP; ++i) {
            const int p = tid + i * THREADS, pp = p < 32 * ppr ? p : 0;
            const int rr = pp / ppr, c = pp - rr * ppr;
            stage[i] = ldw4(mat + (size_t)min(row0 + rr, n_rows - 1) * A.stride, g0 * 2 + c);
        }
#pragma unroll
        for (int i = 0; i < MP; ++i) {
            const int p = tid + i * THREADS, pp = p < 32 * mpr ? p : 0;
            const int rr = pp / mpr, c = pp - rr * mpr;
            mstage[i] = ldw4(mat + (size_t)min(row0 + rr, n_rows - 1) * A.stride + A.meta_off, g0 / 4 + c);
        }
        h8_t a_even[MT][4], a_odd[MT][4];
        load_a(a_even, g0 + min(wv, sg - 1));                         // first A operands travel during the copy
#pragma unroll
        for (int i = 0; i < CP; ++i) {
            const int p = tid + i * THREADS;
            if (p < 32 * ppr) {
                const int rr = p / ppr, c = p - rr * ppr;
                *reinterpret_cast<uint4 *>(lds_codes + rr * code_pitch + c * 16) = stage[i];
            }
        }
#pragma unroll
        for (int i = 0; i < MP; ++i) {
            const int p = tid + i * THREADS;
            if (p < 32 * mpr) {
                const int rr = p / mpr, c = p - rr * mpr;
                *reinterpret_cast<uint4 *>(lds_meta + rr * meta_pitch + c * 4) = mstage[i];
            }
        }
        __syncthreads();
        // ---- multiply: wave wv takes groups wv, wv+4, ...; two per trip, each one's A operands requested while
        // the other is multiplied (past the end the last group is read again and not used)
        for (int g = wv; g < sg; g += 2 * MF2_WAVES) {
            load_a(a_odd, g0 + min(g + MF2_WAVES, sg - 1));
            multiply(a_even, g);
            load_a(a_even, g0 + min(g + 2 * MF2_WAVES, sg - 1));
            if (g + MF2_WAVES < sg) multiply(a_odd, g + MF2_WAVES);
        }
        __syncthreads();                                              // before the next segment overwrites LDS
    }
    // ---- add the four waves' partial sums (LDS reused), then the epilogue
    float *red = reinterpret_cast<float *>(lds);                      // [wave][MT][16][64]
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) red[((wv * MT + t) * 16 + i) * 64 + lane] = acc[t][i];
    __syncthreads();
    const int mrow = row0 + col;                                      // this lane's memory row
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) {
            const int i = wv * 4 + ii;                                // each wave finishes a quarter of the registers
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < MF2_WAVES; ++w) v += red[((w * MT + t) * 16 + i) * 64 + lane];
            const int tok = t * 32 + 8 * (i / 4) + 4 * kh + (i % 4);
            if (W13) {
                const float other = dpp_f<0xB1>(v);                   // the neighbouring column: v of the pair for even lanes
                if ((lane & 1) == 0 && tok < en.n_tok && mrow < n_rows) {
                    const _Float16 av = (_Float16)silu_mul(v, other);
                    A.a[(size_t)A.pair[en.first + tok] * A.N + (mrow >> 1)] = __builtin_bit_cast(uint16_t, av);
                }
            } else if (tok < en.n_tok && mrow < n_rows) {
                A.ypart[(size_t)A.pair[en.first + tok] * A.N + mrow] = A.w[en.first + tok] * v;
            }
        }
    if (!W13 && blockIdx.x == 0 && tid < en.n_tok) A.ytab[A.pair[en.first + tid]] = y_rows(A.pair[en.first + tid], 1u);
}

}  // namespace moe
