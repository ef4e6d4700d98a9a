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
// reduction so that its memory latency overlaps the norm rather than following it.
template <bool SPEC>
__global__ __launch_bounds__(GATE_THREADS) void k_gate(GateArgs a)
{
    constexpr int NACC = SPEC ? 32 : 16;
    constexpr int NPRE = SPEC ? 0 : 8;                   // experts whose first slice is requested up front
    __shared__ double red[GATE_WAVES][32];
    __shared__ double tot[33];
    __shared__ double prob[16];          // thread 0's small tables live in LDS: indexed at run time, they would
    __shared__ int chosen[4];            // otherwise be carved out of scratch memory for every lane of the launch
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint16_t *x = a.x + (size_t)b * a.H;
    const int n1 = a.wg ? a.E : 0, n2 = (SPEC && a.wg2) ? a.E2 : 0;

    float4 wpre[NPRE > 0 ? NPRE : 1];
    if constexpr (NPRE > 0) {
#pragma unroll
        for (int e = 0; e < NPRE; ++e)
            wpre[e] = (e < n1 && tid * 4 < a.H) ? *reinterpret_cast<const float4 *>(a.wg + (size_t)e * a.H + tid * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
    }

    double scale = 1.0;
    if (a.eps > 0.0) {
        double ss = 0.0;
        for (int i = tid * 4; i < a.H; i += GATE_THREADS * 4) {
            const uint2 p = *reinterpret_cast<const uint2 *>(x + i);
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
            tot[32] = 1.0 / sqrt(t / (double)a.H + a.eps);
        }
        __syncthreads();
        scale = tot[32];
    }

    double acc[NACC];
#pragma unroll
    for (int e = 0; e < NACC; ++e) acc[e] = 0.0;
    for (int i = tid * 4; i < a.H; i += GATE_THREADS * 4) {
        const uint2 p = *reinterpret_cast<const uint2 *>(x + i);
        uint16_t hv[4] = {(uint16_t)(p.x & 0xffff), (uint16_t)(p.x >> 16), (uint16_t)(p.y & 0xffff), (uint16_t)(p.y >> 16)};
        if (a.eps > 0.0) {
            uint2 g = make_uint2(0x3c003c00u, 0x3c003c00u);
            if (a.gamma) g = *reinterpret_cast<const uint2 *>(a.gamma + i);
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
                if (e < NPRE && i == tid * 4) w = wpre[e < NPRE ? e : 0];
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
    if (tid < 32) {
        const bool live = (tid < 16) ? (tid < n1) : (tid - 16 < n2);
        if (live) {
            double t = 0.0;
            for (int w = 0; w < GATE_WAVES; ++w) t += red[w][tid];
            tot[tid] = t;
        }
    }
    __syncthreads();
    // speculative gate: one thread per expert takes its exponential (thread 0 alone would take them one after another)
    __shared__ double spec_e[16];
    if constexpr (SPEC) {
        if (tid < n2) {
            double zmax = tot[16];
            for (int e = 1; e < n2; ++e) zmax = tot[16 + e] > zmax ? tot[16 + e] : zmax;
            spec_e[tid] = exp(tot[16 + tid] - zmax);
        }
        __syncthreads();
    }
    if (tid == 0) {
        GateHostOut *o = a.out;
        if (n1) {
            // top-K by (logit descending, index ascending).  The logits move to registers first (fixed indices): every
            // comparison out of LDS would otherwise be a dependent round trip of this one thread.
            double z[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) z[e] = e < n1 ? tot[e] : 0.0;
            uint32_t used = 0;
            for (int j = 0; j < a.K; ++j) {
                int best = -1;
                double zb = 0.0;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const bool take = e < n1 && !((used >> e) & 1u) && (best < 0 || z[e] > zb);
                    best = take ? e : best;
                    zb = take ? z[e] : zb;
                }
                chosen[j] = best;
                used |= 1u << best;
                prob[j] = zb;                // the chosen logit, until the softmax below replaces it
            }
            // softmax over all experts, renormalised over the chosen ones == softmax over the chosen logits
            const double zmax = prob[0];
            double ps;
            prob[0] = 1.0;                   // exp(0): the first choice holds the largest logit
            ps = 1.0;
            for (int j = 1; j < a.K; ++j) { prob[j] = exp(prob[j] - zmax); ps += prob[j]; }
            if (a.route_idx) {
                for (int j = 0; j < a.K; ++j) {
                    a.route_idx[j] = chosen[j];
                    a.route_w[j] = (float)(prob[j] / ps);
                    a.route_log[j] = chosen[j];
                }
                return;
            }
            for (int j = 0; j < a.K; ++j) {
                o->idx[b * a.K + j] = chosen[j];
                o->w[b * a.K + j] = (float)(prob[j] / ps);
            }
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (e < n1) o->logits[b * n1 + e] = z[e];
        }
        if (n2) {
            double ps = 0.0;
            for (int e = 0; e < n2; ++e) ps += spec_e[e];
            for (int e = 0; e < n2; ++e) o->spec_p[b * n2 + e] = spec_e[e] / ps;
        }
        __hip_atomic_store(&o->done[b], a.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

}  // namespace moe
