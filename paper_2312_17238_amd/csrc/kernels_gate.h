// Gate kernel: RMSNorm + linear gate + top-k, plus the next layer's gate for speculative loading
// (Sec. 2.1, Sec. 3.2), all decisions in fp64.
#pragma once
#include "kernels_common.h"

namespace moe {

// ---------------------------------------------------------------------------------------------
// K1: RMSNorm + gate + top-k (+ next layer's gate for speculative loading)
// ---------------------------------------------------------------------------------------------

constexpr int GATE_MAX_TOKENS = 1024;   // tokens per launch (the interface's batch limit)

struct GateHostOut {                // lives in host-mapped pinned memory; written by the kernel
    int32_t idx[GATE_MAX_TOKENS * 4];            // [b*K + j]
    float w[GATE_MAX_TOKENS * 4];
    double logits[GATE_MAX_TOKENS * 16];         // [b*E + e]
    double spec_p[GATE_MAX_TOKENS * 16];         // [b*E2 + e] next-layer gate probabilities per token
    uint32_t done[GATE_MAX_TOKENS];              // [b] = sequence number of the launch, stored by block b after its results
                                    // (system-scope release; one word per block: posted writes, no round trips)
    uint32_t ffn_error;             // set by the fused FFN kernel if its grid barrier gave up
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
    uint32_t seq;                   // value to publish in out->done[b]
    // Device-side routing (one token, every expert of the layer resident): the selection and the combine weights go
    // to device memory for the FFN kernels of the same step, the selection also to a log ring the host copies back
    // later for its bookkeeping; nothing is published in `out` and nobody waits for this launch.
    int32_t *route_idx;             // [K] device, or null
    float *route_w;                 // [K] device
    int32_t *route_log;             // [K] device: this step's slot of the log ring
};

constexpr int GATE_THREADS = 1024;
constexpr int GATE_WAVES = GATE_THREADS / WAVE;

// One block per token, 4 consecutive elements per thread and pass.  All decisions are taken in fp64:
// the products fp32 x fp16 are exact in fp64 and the sums differ from any other fp64 summation order
// only at the 1e-16 level, so routing equals an fp64 reference except on ties closer than that.
// SPEC: the launch also evaluates the next layer's gate (a.wg2).  Without it the accumulators of the second gate
// are not needed and the registers go to this thread's first slice of W_g instead, requested before the norm's
// reduction so that its memory latency overlaps the norm rather than following it (after the thread's slice of x:
// loads return in order, and the norm waits for x).
// After the one barrier that collects the waves' partial logits, wave 0 finishes alone: lane e holds logit e (lane
// 16 + e the next layer's), the selection runs on values read from those lanes, and the exponentials, divisions and
// stores of the K chosen experts (and of the next layer's probabilities) are one per lane.
template <bool SPEC>
__global__ __launch_bounds__(GATE_THREADS) void k_gate(GateArgs a)
{
    constexpr int NACC = SPEC ? 32 : 16;
    constexpr int NPRE = SPEC ? 0 : 8;                   // experts whose first slice is requested up front
    __shared__ double red[GATE_WAVES][32];
    __shared__ double inv_rms;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint16_t *x = a.x + (size_t)b * a.H;
    const int n1 = a.wg ? a.E : 0, n2 = (SPEC && a.wg2) ? a.E2 : 0;
    const bool normed = a.eps > 0.0;

    const int i0 = tid * 4;                              // the thread's first slice
    const uint2 ones = make_uint2(0x3c003c00u, 0x3c003c00u);
    const uint2 x0 = i0 < a.H ? *reinterpret_cast<const uint2 *>(x + i0) : make_uint2(0u, 0u);
    const uint2 g0 = (normed && a.gamma && i0 < a.H) ? *reinterpret_cast<const uint2 *>(a.gamma + i0) : ones;
    float4 wpre[NPRE > 0 ? NPRE : 1];
    if constexpr (NPRE > 0) {
#pragma unroll
        for (int e = 0; e < NPRE; ++e)
            wpre[e] = (e < n1 && i0 < a.H) ? *reinterpret_cast<const float4 *>(a.wg + (size_t)e * a.H + i0) : make_float4(0.f, 0.f, 0.f, 0.f);
    }

    double scale = 1.0;
    if (normed) {
        double ss = 0.0;
        for (int i = i0; i < a.H; i += GATE_THREADS * 4) {
            const uint2 p = i == i0 ? x0 : *reinterpret_cast<const uint2 *>(x + i);
            const double v0 = half_bits_to_f64(p.x & 0xffff), v1 = half_bits_to_f64(p.x >> 16);
            const double v2 = half_bits_to_f64(p.y & 0xffff), v3 = half_bits_to_f64(p.y >> 16);
            ss += v0 * v0; ss += v1 * v1; ss += v2 * v2; ss += v3 * v3;
        }
        ss = wave_sum_f64(ss);
        if (lane == 0) red[wv][0] = ss;
        __syncthreads();
        if (tid == 0) {
            double t = 0.0;
            for (int w = 0; w < GATE_WAVES; ++w) t += red[w][0];
            inv_rms = 1.0 / sqrt(t / (double)a.H + a.eps);
        }
        __syncthreads();
        scale = inv_rms;
    }

    double acc[NACC];
#pragma unroll
    for (int e = 0; e < NACC; ++e) acc[e] = 0.0;
    for (int i = i0; i < a.H; i += GATE_THREADS * 4) {
        const uint2 p = i == i0 ? x0 : *reinterpret_cast<const uint2 *>(x + i);
        uint16_t hv[4] = {(uint16_t)(p.x & 0xffff), (uint16_t)(p.x >> 16), (uint16_t)(p.y & 0xffff), (uint16_t)(p.y >> 16)};
        if (normed) {
            uint2 g = ones;
            if (a.gamma) g = i == i0 ? g0 : *reinterpret_cast<const uint2 *>(a.gamma + i);
            const uint16_t gv[4] = {(uint16_t)(g.x & 0xffff), (uint16_t)(g.x >> 16), (uint16_t)(g.y & 0xffff), (uint16_t)(g.y >> 16)};
#pragma unroll
            for (int j = 0; j < 4; ++j) hv[j] = f64_to_f16_rne(half_bits_to_f64(hv[j]) * scale * half_bits_to_f64(gv[j]));
        }
        const uint2 ho = make_uint2((uint32_t)hv[0] | (uint32_t)hv[1] << 16, (uint32_t)hv[2] | (uint32_t)hv[3] << 16);
        if (a.h_out) *reinterpret_cast<uint2 *>(a.h_out + (size_t)b * a.H + i) = ho;
        if (a.h_out2) *reinterpret_cast<uint2 *>(a.h_out2 + (size_t)b * a.H + i) = ho;
        if (a.yacc) *reinterpret_cast<float4 *>(a.yacc + (size_t)b * a.H + i) = make_float4(0.f, 0.f, 0.f, 0.f);
        const double h0 = half_bits_to_f64(hv[0]), h1 = half_bits_to_f64(hv[1]), h2 = half_bits_to_f64(hv[2]),
                     h3 = half_bits_to_f64(hv[3]);
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (e < n1) {
                float4 w;
                if (e < NPRE && i == i0) w = wpre[e < NPRE ? e : 0];
                else w = *reinterpret_cast<const float4 *>(a.wg + (size_t)e * a.H + i);
                acc[e] += (double)w.x * h0; acc[e] += (double)w.y * h1; acc[e] += (double)w.z * h2; acc[e] += (double)w.w * h3;
            }
        if constexpr (SPEC) {
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (e < n2) {
                    const float4 w = *reinterpret_cast<const float4 *>(a.wg2 + (size_t)e * a.H + i);
                    acc[16 + e] += (double)w.x * h0; acc[16 + e] += (double)w.y * h1; acc[16 + e] += (double)w.z * h2; acc[16 + e] += (double)w.w * h3;
                }
        }
    }
    // all logits' wave sums at once; accumulators of experts that do not exist hold zeros
    if constexpr (SPEC) {
        wave_sum_many_f64<32>(acc, lane);
        if (lane < 32) red[wv][wave_sum_index<32>(lane)] = acc[0];
    } else if (n1 <= 8) {
        wave_sum_many_f64<8>(acc, lane);
        if (lane < 8) red[wv][wave_sum_index<8>(lane)] = acc[0];
    } else {
        wave_sum_many_f64<16>(acc, lane);
        if (lane < 16) red[wv][wave_sum_index<16>(lane)] = acc[0];
    }
    __syncthreads();
    if (wv != 0) return;

    const bool live = lane < 16 ? lane < n1 : (lane < 32 && lane - 16 < n2);
    double t = 0.0;
    if (live)
        for (int w = 0; w < GATE_WAVES; ++w) t += red[w][lane];
    GateHostOut *o = a.out;
    if (n1) {
        // top-K by (logit descending, index ascending), the same for every lane: on the 16 logits read from their lanes
        double z[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) z[e] = readlane_d(t, e);
        int c[4] = {0, 0, 0, 0};
        double zc[4] = {0.0, 0.0, 0.0, 0.0};
        uint32_t used = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < a.K) {
                int best = -1;
                double zb = 0.0;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const bool take = e < n1 && !((used >> e) & 1u) && (best < 0 || z[e] > zb);
                    best = take ? e : best;
                    zb = take ? z[e] : zb;
                }
                c[j] = best;
                zc[j] = zb;
                used |= 1u << best;
            }
        // softmax over all experts, renormalised over the chosen ones == softmax over the chosen logits; lane j < K
        // takes choice j (the first holds the largest logit: exp(0) = 1)
        int mine = 0;
        double zmine = zc[0];
#pragma unroll
        for (int j = 1; j < 4; ++j)
            if (lane == j && j < a.K) { mine = c[j]; zmine = zc[j]; }
        if (lane == 0) mine = c[0];
        const double pe = exp(zmine - zc[0]);
        double ps = 0.0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < a.K) ps += readlane_d(pe, j);
        const float wgt = (float)(pe / ps);
        if (a.route_idx) {
            if (lane < a.K) {
                a.route_idx[lane] = mine;
                a.route_w[lane] = wgt;
                a.route_log[lane] = mine;
            }
            return;
        }
        if (lane < a.K) {
            o->idx[b * a.K + lane] = mine;
            o->w[b * a.K + lane] = wgt;
        }
        if (lane < n1) o->logits[b * n1 + lane] = t;
    }
    if constexpr (SPEC) {
        if (n2) {
            double zmax = readlane_d(t, 16);
#pragma unroll
            for (int e = 1; e < 16; ++e)
                if (e < n2) {
                    const double v = readlane_d(t, 16 + e);
                    zmax = v > zmax ? v : zmax;
                }
            const double se = exp(t - zmax);
            double ps = 0.0;
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (e < n2) ps += readlane_d(se, 16 + e);
            if (lane >= 16 && lane - 16 < n2) o->spec_p[b * n2 + lane - 16] = se / ps;
        }
    }
    if (lane == 0) __hip_atomic_store(&o->done[b], a.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

}  // namespace moe
