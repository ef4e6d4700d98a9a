// gfx950 device code of the decode step: gate (RMSNorm + linear gate + top-k + speculative gate),
// fused dequantize+GEMV for w1/w3 -> SiLU*mul and for w2 -> weighted accumulate, and the residual add.
//
// Wavefronts are 64 wide.  The GEMV kernels are bound by HBM bandwidth: every weight byte is read
// exactly once per step with 128-bit loads, a lane owns a fixed 32-code column chunk of every row its
// wave visits, the activations it needs for that chunk stay in registers for the whole kernel, and the
// only cross-lane traffic is one DPP reduction per output row.
//
// Dequantization is never materialised.  With W^ = (q - z) s per group (Sec. 4.2),
//     sum_i W^_i h_i = s * (sum_i q_i h_i - z * sum_i h_i),
// and sum_i q_i h_i comes from fp16 bit tricks: OR-ing a 4-bit code into the mantissa of 1024.0
// (bits 0..3) or 64.0 (bits 4..7) gives the fp16 numbers 1024+q and 64+q exactly; two of them are
// multiplied with two activations and accumulated in fp32 by one v_dot2_f32_f16.  The biases are
// removed by starting the accumulator at -sum_i bias_i h_i, a per-lane constant.
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

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over the 64 lanes; the total is returned in every lane.  Fixed order, so deterministic.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_f<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f<0x141>(v);   // row_half_mirror
    v += dpp_f<0x140>(v);   // row_mirror: every lane of a 16-lane row now holds the row's sum
    float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
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

// ---------------------------------------------------------------------------------------------
// K1: RMSNorm + gate + top-k (+ next layer's gate for speculative loading)
// ---------------------------------------------------------------------------------------------

struct GateHostOut {                // lives in host-mapped pinned memory; written by the kernel
    int32_t idx[64 * 4];            // [b*K + j]
    float w[64 * 4];
    double logits[64 * 16];         // [b*E + e]
    double spec_p[64 * 16];         // [b*E2 + e] next-layer gate probabilities per token
    uint32_t done;                  // incremented once per block, system scope, after its results
};

struct GateArgs {
    const uint16_t *x;              // [B][H] fp16
    const float *wg;                // [E][H] fp32 or null (speculative gate only)
    const float *wg2;               // [E2][H] fp32 or null
    const uint16_t *gamma;          // [H] fp16 or null (gain 1)
    uint16_t *h_out;                // [B][H] fp16 or null
    uint16_t *h_out2;               // optional second copy
    float *yacc;                    // [B][H] fp32 to clear, or null
    GateHostOut *out;
    double eps;                     // 0: no norm
    int32_t H, E, E2, K;
};

constexpr int GATE_THREADS = 256;

// One block per token.  All decisions are taken in fp64: the products fp32 x fp16 are exact in fp64
// and the sums only differ from any other fp64 summation order at the 1e-16 level, so routing equals
// an fp64 reference except on ties closer than that.
__global__ __launch_bounds__(GATE_THREADS) void k_gate(GateArgs a)
{
    extern __shared__ uint16_t sh_h[];                     // H fp16
    __shared__ double red[GATE_THREADS / WAVE][2 * 16 + 1];
    __shared__ double tot[2 * 16 + 1];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint16_t *x = a.x + (size_t)b * a.H;

    double scale = 1.0;
    if (a.eps > 0.0) {
        double ss = 0.0;
        for (int i = tid; i < a.H; i += GATE_THREADS) {
            double v = (double)__builtin_bit_cast(_Float16, x[i]);
            ss += v * v;
        }
        ss = wave_sum_f64(ss);
        if (lane == 0) red[wv][0] = ss;
        __syncthreads();
        if (tid == 0) {
            double t = 0.0;
            for (int w = 0; w < GATE_THREADS / WAVE; ++w) t += red[w][0];
            tot[0] = 1.0 / sqrt(t / (double)a.H + a.eps);
        }
        __syncthreads();
        scale = tot[0];
        __syncthreads();
    }
    for (int i = tid; i < a.H; i += GATE_THREADS) {
        uint16_t hv = x[i];
        if (a.eps > 0.0) {
            double g = a.gamma ? (double)__builtin_bit_cast(_Float16, a.gamma[i]) : 1.0;
            hv = f64_to_f16_rne((double)__builtin_bit_cast(_Float16, x[i]) * scale * g);
        }
        sh_h[i] = hv;
        if (a.h_out) a.h_out[(size_t)b * a.H + i] = hv;
        if (a.h_out2) a.h_out2[(size_t)b * a.H + i] = hv;
        if (a.yacc) a.yacc[(size_t)b * a.H + i] = 0.f;
    }
    __syncthreads();

    const int n1 = a.wg ? a.E : 0, n2 = a.wg2 ? a.E2 : 0, nt = n1 + n2;
    double acc[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) acc[e] = 0.0;
    for (int i = tid; i < a.H; i += GATE_THREADS) {
        const double hv = (double)__builtin_bit_cast(_Float16, sh_h[i]);
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (e < n1) acc[e] += (double)a.wg[(size_t)e * a.H + i] * hv;
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (e < n2) acc[16 + e] += (double)a.wg2[(size_t)e * a.H + i] * hv;
    }
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const bool live = (e < 16) ? (e < n1) : (e - 16 < n2);
        if (live) {
            double v = wave_sum_f64(acc[e]);
            if (lane == 0) red[wv][e] = v;
        }
    }
    __syncthreads();
    if (tid < 32) {
        const bool live = (tid < 16) ? (tid < n1) : (tid - 16 < n2);
        if (live) {
            double t = 0.0;
            for (int w = 0; w < GATE_THREADS / WAVE; ++w) t += red[w][tid];
            tot[tid] = t;
        }
    }
    __syncthreads();
    if (tid == 0) {
        GateHostOut *o = a.out;
        if (n1) {
            // top-K by (logit descending, index ascending)
            int chosen[4];
            for (int j = 0; j < a.K; ++j) {
                int best = -1;
                for (int e = 0; e < n1; ++e) {
                    bool used = false;
                    for (int q = 0; q < j; ++q) used |= (chosen[q] == e);
                    if (used) continue;
                    if (best < 0 || tot[e] > tot[best]) best = e;
                }
                chosen[j] = best;
            }
            // softmax over all experts, renormalised over the chosen ones == softmax over the chosen logits
            const double zmax = tot[chosen[0]];
            double p[4], ps = 0.0;
            for (int j = 0; j < a.K; ++j) { p[j] = exp(tot[chosen[j]] - zmax); ps += p[j]; }
            for (int j = 0; j < a.K; ++j) {
                o->idx[b * a.K + j] = chosen[j];
                o->w[b * a.K + j] = (float)(p[j] / ps);
            }
            for (int e = 0; e < n1; ++e) o->logits[b * n1 + e] = tot[e];
        }
        if (n2) {
            double zmax = tot[16];
            for (int e = 1; e < n2; ++e) zmax = tot[16 + e] > zmax ? tot[16 + e] : zmax;
            double pe[16], ps = 0.0;
            for (int e = 0; e < n2; ++e) { pe[e] = exp(tot[16 + e] - zmax); ps += pe[e]; }
            for (int e = 0; e < n2; ++e) o->spec_p[b * n2 + e] = pe[e] / ps;
        }
        __threadfence_system();
        __hip_atomic_fetch_add(&o->done, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// ---------------------------------------------------------------------------------------------
// fused dequant-GEMV, 4-bit codes
// ---------------------------------------------------------------------------------------------

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
    float *yacc;                    // [B][H] fp32 accumulators (cleared by the gate kernel)
    int32_t H, F, group;
    uint32_t stride13, meta13;      // w1/w3 row: stride and offset of the (scale, zero) pairs
    uint32_t stride2, meta2;        // w2 row
    uint64_t off_w2;
    int32_t rows_per_block;         // w2 kernel
};

// Per-lane activation state for one 32-code chunk: 16 half2 registers plus the two constants of the
// factorisation.  Element i of a word's 8 codes has bias 1024 if i%4 < 2, else 64.
struct Chunk {
    h2_t h[16];
    float bias_dot;   // sum_i bias_i * h_i
    float hsum;       // sum_i h_i
};

__device__ __forceinline__ void load_chunk(Chunk &c, const uint16_t *vec, int chunk, bool live)
{
    const uint4 *p = reinterpret_cast<const uint4 *>(vec + (size_t)chunk * 32);
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint4 v = live ? p[i] : make_uint4(0, 0, 0, 0);
        w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
    }
    float bd = 0.f, hs = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        c.h[i] = as_h2(w[i]);
        const float x0 = (float)c.h[i].x, x1 = (float)c.h[i].y;
        hs += x0 + x1;
        bd += ((i & 1) ? 64.f : 1024.f) * (x0 + x1);
    }
    c.bias_dot = bd;
    c.hsum = hs;
}

// sum_i q_i h_i over the 32 codes of one uint4 (bias already folded into `start`)
__device__ __forceinline__ float dot_q4(const uint4 &q, const Chunk &c, float start)
{
    float d = start;
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t lo = w[i], hi = w[i] >> 8;
        d = __builtin_amdgcn_fdot2(as_h2((lo & 0x000F000Fu) | 0x64006400u), c.h[4 * i + 0], d, false);
        d = __builtin_amdgcn_fdot2(as_h2((lo & 0x00F000F0u) | 0x54005400u), c.h[4 * i + 1], d, false);
        d = __builtin_amdgcn_fdot2(as_h2((hi & 0x000F000Fu) | 0x64006400u), c.h[4 * i + 2], d, false);
        d = __builtin_amdgcn_fdot2(as_h2((hi & 0x00F000F0u) | 0x54005400u), c.h[4 * i + 3], d, false);
    }
    return d;
}

__device__ __forceinline__ float silu_mul(float u, float v) { return u / (1.f + __expf(-u)) * v; }

constexpr int W13_WAVES = 4;

// K2: a[pair][r] = silu(W1^ h)[r] * (W3^ h)[r].  grid = (row blocks, entries); a wave walks rows
// r = wave_id, wave_id + n_waves, ...; KCH = ceil(H / 2048) chunks per lane per row.
template <int KCH, int NT>
__global__ __launch_bounds__(W13_WAVES *WAVE) void k_w13_q4(FfnArgs A)
{
    const FfnEntry &en = A.e[blockIdx.y];
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * W13_WAVES + (threadIdx.x >> 6), n_waves = gridDim.x * W13_WAVES;
    const int n_chunks = A.H / 32;

    Chunk hc[NT][KCH];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tok = en.tok[t < en.n_tok ? t : 0];
#pragma unroll
        for (int k = 0; k < KCH; ++k) load_chunk(hc[t][k], A.h + (size_t)tok * A.H, k * 64 + lane, k * 64 + lane < n_chunks);
    }
    const uint8_t *base = en.blob;
    const int groups_per_chunk_shift = (A.group == 32) ? 0 : (A.group == 64 ? 1 : 2);

    uint4 q1[KCH], q3[KCH];
    uint32_t m1[KCH], m3[KCH];
    auto load_row = [&](int r) {
        const uint8_t *r1 = base + (size_t)(2 * r) * A.stride13, *r3 = r1 + A.stride13;
#pragma unroll
        for (int k = 0; k < KCH; ++k) {
            const int c = k * 64 + lane;
            const bool live = c < n_chunks;
            const int cc = live ? c : 0;
            q1[k] = reinterpret_cast<const uint4 *>(r1)[cc];
            q3[k] = reinterpret_cast<const uint4 *>(r3)[cc];
            m1[k] = reinterpret_cast<const uint32_t *>(r1 + A.meta13)[cc >> groups_per_chunk_shift];
            m3[k] = reinterpret_cast<const uint32_t *>(r3 + A.meta13)[cc >> groups_per_chunk_shift];
        }
    };

    int r = wave;
    if (r < A.F) load_row(r);
    while (r < A.F) {
        uint4 c1[KCH], c3[KCH];
        uint32_t n1[KCH], n3[KCH];
#pragma unroll
        for (int k = 0; k < KCH; ++k) { c1[k] = q1[k]; c3[k] = q3[k]; n1[k] = m1[k]; n3[k] = m3[k]; }
        const int rn = r + n_waves;
        if (rn < A.F) load_row(rn);
        float u[NT], v[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) { u[t] = 0.f; v[t] = 0.f; }
#pragma unroll
        for (int k = 0; k < KCH; ++k) {
            const bool live = k * 64 + lane < n_chunks;
            const float s1 = live ? lo_half(n1[k]) : 0.f, z1 = hi_half(n1[k]);
            const float s3 = live ? lo_half(n3[k]) : 0.f, z3 = hi_half(n3[k]);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float d1 = dot_q4(c1[k], hc[t][k], -hc[t][k].bias_dot);
                const float d3 = dot_q4(c3[k], hc[t][k], -hc[t][k].bias_dot);
                u[t] = fmaf(s1, fmaf(-z1, hc[t][k].hsum, d1), u[t]);
                v[t] = fmaf(s3, fmaf(-z3, hc[t][k].hsum, d3), v[t]);
            }
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const float us = wave_sum(u[t]), vs = wave_sum(v[t]);
            if (lane == 0 && t < en.n_tok) {
                const _Float16 av = (_Float16)silu_mul(us, vs);
                A.a[(size_t)en.pair[t] * A.F + r] = __builtin_bit_cast(uint16_t, av);
            }
        }
        r = rn;
    }
}

// K3: yacc[tok][r] += w * (W2^ a[pair])[r].  grid = (row blocks, entries); block = CS waves, wave cs
// owns column chunk cs*64 + lane of every row of the block; partial sums meet in LDS.
template <int NT>
__global__ __launch_bounds__(1024) void k_w2_q4(FfnArgs A)
{
    extern __shared__ float red[];                       // [rows_per_block][NT][CS]
    const FfnEntry &en = A.e[blockIdx.y];
    const int lane = threadIdx.x & 63, cs = threadIdx.x >> 6, CS = blockDim.x >> 6;
    const int n_chunks = A.F / 32;
    const int c = cs * 64 + lane;
    const bool live = c < n_chunks;
    const int cc = live ? c : 0;
    const int gshift = (A.group == 32) ? 0 : (A.group == 64 ? 1 : 2);

    Chunk ac[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) load_chunk(ac[t], A.a + (size_t)en.pair[t < en.n_tok ? t : 0] * A.F, c, live);

    const int R = A.rows_per_block;
    const int row0 = blockIdx.x * R;
    const uint8_t *base = en.blob + A.off_w2;
    constexpr int UN = 8;
    for (int rr = 0; rr < R; rr += UN) {
        uint4 q[UN];
        uint32_t m[UN];
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            int row = row0 + rr + j;
            row = row < A.H ? row : A.H - 1;
            const uint8_t *rp = base + (size_t)row * A.stride2;
            q[j] = reinterpret_cast<const uint4 *>(rp)[cc];
            m[j] = reinterpret_cast<const uint32_t *>(rp + A.meta2)[cc >> gshift];
        }
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const float s = live ? lo_half(m[j]) : 0.f, z = hi_half(m[j]);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float d = dot_q4(q[j], ac[t], -ac[t].bias_dot);
                const float part = wave_sum(s * fmaf(-z, ac[t].hsum, d));
                if (lane == 0 && rr + j < R) red[((rr + j) * NT + t) * CS + cs] = part;
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < R * NT; i += blockDim.x) {
        const int rr = i / NT, t = i % NT, row = row0 + rr;
        if (row < A.H && t < en.n_tok) {
            float s = 0.f;
            for (int k = 0; k < CS; ++k) s += red[i * CS + k];
            atomicAdd(&A.yacc[(size_t)en.tok[t] * A.H + row], en.w[t] * s);
        }
    }
}

// x_out = fp16(x + yacc)
__global__ void k_residual(const uint16_t *x, const float *yacc, uint16_t *x_out, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const float v = (float)__builtin_bit_cast(_Float16, x[i]) + yacc[i];
        x_out[i] = __builtin_bit_cast(uint16_t, (_Float16)v);
    }
}

}  // namespace moe
