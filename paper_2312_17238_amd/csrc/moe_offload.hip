// C ABI of the MoE-offloading decode engine (see include/moe_offload.h for the contract).
//
// One decode step of one layer, as the paper orders it (Sec. 3.2, 3.3):
//   gate kernel (compute stream)  ->  host reads the routing from host-mapped memory
//   -> host resolves the LRU cache -> demand copies (copy stream) -> speculative copies for the next
//   layer (copy stream, right after the demand copies) -> compute stream waits on the events of the
//   buffers it is about to read -> fused dequant-GEMV kernels -> residual add.
// The call returns as soon as everything is enqueued.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "../../include/moe_offload.h"
#include "cache.h"
#include "kernels.h"
#include "layout.h"

using namespace moe;

static_assert(GATE_MAX_TOKENS == MOE_MAX_BATCH && MOE_MAX_TOPK == 4 && MOE_MAX_EXPERTS == 16, "the gate kernel's result arrays are sized for the interface limits");

// ---------------------------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------------------------

static thread_local char g_err[512] = "";
static thread_local int32_t g_hip_err = 0;

static int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIPCHK(expr)                                                                                   \
    do {                                                                                               \
        hipError_t e_ = (expr);                                                                        \
        if (e_ != hipSuccess) {                                                                        \
            g_hip_err = (int32_t)e_;                                                                   \
            return fail(MOE_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
        }                                                                                              \
    } while (0)

// The boundary lets no C++ exception through (allocation failures of the containers, thread creation): every exported
// function that can raise one is a function-try-block ending here.
static int32_t on_exception(const char *what) noexcept
{
    try {
        throw;
    } catch (const std::bad_alloc &) {
        return fail(MOE_ENOMEM, "%s: out of host memory", what);
    } catch (const std::exception &e) {
        return fail(MOE_ESTATE, "%s: %s", what, e.what());
    } catch (...) {
        return fail(MOE_ESTATE, "%s: unknown exception", what);
    }
}

extern "C" const char *moe_last_error(void) { return g_err; }
extern "C" int32_t moe_last_hip_error(void) { return g_hip_err; }

// ---------------------------------------------------------------------------------------------
// scratch of the entry point that allocates nothing
// ---------------------------------------------------------------------------------------------

// moe_layer_step_noalloc runs a step whose kernels keep their intermediate results (gate input h, SwiGLU
// activations a, the pairs' fp32 partial outputs and the block output y) in this file-scope device array instead of the context's arena, for steps of
// at most NOALLOC_MAX_BATCH tokens of layers no wider than the limits below.  Every GPU the library runs on holds its
// own copy until the process ends; all calls on one GPU share it.
constexpr int NOALLOC_MAX_BATCH = 4, NOALLOC_MAX_HIDDEN = 8192, NOALLOC_MAX_FFN = 16384, NOALLOC_MAX_TOPK = 4;
constexpr size_t NOALLOC_H_BYTES = (size_t)NOALLOC_MAX_BATCH * NOALLOC_MAX_HIDDEN * 2;                    //  64 KB
constexpr size_t NOALLOC_A_BYTES = (size_t)NOALLOC_MAX_BATCH * NOALLOC_MAX_TOPK * NOALLOC_MAX_FFN * 2;    // 512 KB
constexpr size_t NOALLOC_Y_BYTES = (size_t)NOALLOC_MAX_BATCH * NOALLOC_MAX_HIDDEN * 4;                    // 128 KB
constexpr size_t NOALLOC_YPART_BYTES = (size_t)NOALLOC_MAX_BATCH * NOALLOC_MAX_TOPK * NOALLOC_MAX_HIDDEN * 4;   // 512 KB: one row per (token, expert) pair
constexpr size_t NOALLOC_YTAB_BYTES = 256;
constexpr size_t NOALLOC_BYTES = NOALLOC_H_BYTES + NOALLOC_A_BYTES + NOALLOC_Y_BYTES + NOALLOC_YPART_BYTES + NOALLOC_YTAB_BYTES;
static __device__ __align__(256) uint8_t scratch[NOALLOC_BYTES];

// In host code the array's name is only a handle; its device address is asked for once per device, with that device
// current, and kept here.  Host code uses this pointer, never the name.
constexpr int NOALLOC_MAX_DEVICES = 64;
static uint8_t *g_scratch_ptr[NOALLOC_MAX_DEVICES] = {};

// ---------------------------------------------------------------------------------------------
// objects
// ---------------------------------------------------------------------------------------------

struct PoolBuf {
    uint8_t *ptr = nullptr;
    hipEvent_t ready = nullptr;   // recorded on the copy stream after the last copy into this buffer
    bool pending = false;         // a copy was recorded that the compute stream has not yet waited on
    uint64_t have = 0;            // staging use: bytes of the guessed expert requested so far (head of a speculative load)
    hipEvent_t drained = nullptr; // swap mode: recorded on the write-back stream after the evicted expert left this buffer
    bool draining = false;        // a write-back out of this buffer was recorded that no later copy into it has waited on
};

// Optional timing of the engine's own launches with HIP events recorded on the stream each launch goes to.
enum { PROF_GATE = 0, PROF_W13 = 1, PROF_W2 = 2, PROF_COPY = 3, PROF_FFN = 4, PROF_WRITEBACK = 5, PROF_KINDS = 6 };

struct ProfKind {
    std::vector<hipEvent_t> start, stop;   // created on demand, reused after a drain
    size_t used = 0;
    uint64_t launches = 0, bytes = 0;
    double ms = 0.0;
};

struct Profiler {
    bool on = false;
    hipEvent_t base = nullptr;                 // recorded on the compute stream when profiling is switched on: time zero of the timeline
    ProfKind kind[PROF_KINDS];
    static constexpr size_t RING = 65536;      // pairs per kind before a drain (which synchronises) is needed
    static constexpr size_t PREALLOC = 16384;  // pairs per kind created when profiling is switched on
    int32_t copy_stride = 1;                   // time every n-th transfer only: the two event records per copy cost the link ~1 %
    uint64_t copy_seq = 0;
};

constexpr uint32_t ROUTE_LOG_ENTRIES = 8192;      // device-routed steps whose bookkeeping may be pending at once

struct moe_ctx {
    moe_ctx_config_t cfg{};
    Profiler prof;
    bool host_only = false;
    hipStream_t compute = nullptr, copy = nullptr;
    hipStream_t writeback = nullptr;    // device -> host copies of evicted experts (layers with MOE_LAYER_SWAP); created on first use
    uint64_t buf_bytes = 0;
    std::vector<PoolBuf> bufs;          // [0, n_staging): staging; layers append their slots
    BufferPool pool;
    uint16_t *h_buf = nullptr, *a_buf = nullptr, *xbuf[2] = {nullptr, nullptr};
    float *yacc = nullptr;              // [B][H] fp32 block output of the last step (before the residual add)
    // Steps that do not finish inside a w2 kernel: every (token, expert) pair's weighted output goes to a row of its
    // own in ypart (rows [0, B*K): row = pair), k_combine adds a token's rows in selection order.  A matrix-core w2
    // launch that splits its contraction over blocks takes one row per (pair, part) from the rows behind those, as
    // long as they last; ytab[pair] tells k_combine where a pair's rows are.
    float *ypart = nullptr;
    uint32_t *ytab = nullptr;
    uint64_t ypart_extra_floats = 0;    // capacity behind the first B*K rows
    uint64_t ypart_extra_used = 0;      // floats of it taken by the launches of the current step
    std::vector<int32_t> w2_parts;      // per window of the current step: parts the matrix-core w2 launches split their contraction into
    std::vector<uint8_t> win_small;     // ... and whether no expert has more than 16 tokens of the window (the 16-token tile form fits)
    uint8_t *noalloc_scratch = nullptr; // this device's copy of the file-scope scratch array (moe_layer_step_noalloc)
    GateHostOut *gate_out = nullptr;    // host pointer
    GateHostOut *gate_out_dev = nullptr;// the same memory as the device sees it
    hipEvent_t ev_gate = nullptr, ev_compute = nullptr;
    int32_t n_layers = 0;
    int32_t w13_blocks = 256, w2_rows = 32;
    int32_t w2_token_rows = 0;          // rows per block of the single-token w2 kernel; 0: hidden / compute units
    uint32_t gate_seq = 0;              // sequence number of the last gate launch
    int32_t mfma_form = 0;              // matrix-core kernels: 0 the default (5); 5 streaming form with 16-token tiles (one per
                                        // expert while no expert of the window has more than 16 tokens, else two), codes multiplied as they are and
                                        // groups scaled in fp32; 4 the same with weights dequantised to fp16;
                                        // 3 streaming form, one fma per pair of weights plus a rank-1 correction;
                                        // 2 streaming form with an exact subtraction first; 1 row-staging form with fp32 group scaling
    int32_t mfma16_waves = 8;           // waves per block of the 16-token forms' single-tile kernels: 4 or 8 (two blocks per compute unit either
                                        // way; with two token tiles 8 waves need 194 registers, one block per unit, and measured 12 % slower)
    int32_t mfma_min_batch = 3;         // batches at least this large use the matrix-core kernels (4-bit g64): measured, all experts of a
                                        // Mixtral-shaped layer resident, they are 9 % faster than the GEMV kernels at 3 tokens and 82 % at 12
    int32_t staged_min_batch = 0;       // matrix-core batches larger than this: resident experts first, arriving ones one by one
    uint64_t spec_head_bytes = 0;       // 0: a speculative load moves the whole expert at once (as the paper describes);
                                        // > 0: only this many leading bytes, the rest when the guess is confirmed
    bool token_path = true;             // single-token steps: w2 kernel with in-kernel combine + residual (no atomics)
    int32_t fused = 0;                  // ... and w1/w3 + w2 as one persistent launch: 1 with a grid barrier between them, 2 expert after expert
    uint32_t *seq_flags = nullptr;      // device flags of the expert-after-expert kernel: [expert][block] = epoch of the last arrival
    int32_t n_cu = 0;                   // compute units: grid size of the persistent kernel
    uint32_t *barrier = nullptr;        // device counter of its grid barrier
    uint32_t barrier_count = 0;         // value it reaches after all launches enqueued so far
    bool sync_wait = false;
    // Device-side routing: steps of one token through a layer whose experts are all resident need no decision of the
    // host, so they are enqueued without waiting for the gate; the cache bookkeeping (recency stamps, counters) is
    // caught up from a log of the selections (a ring in device memory, copied back then) before anything reads or changes it.
    bool device_routing = true;
    int32_t *route_idx = nullptr;       // device: the current step's selection, written by its gate kernel
    float *route_w = nullptr;           // device: ... and combine weights
    int32_t *route_log = nullptr;       // pinned host copy of the ring below, refreshed when the bookkeeping catches up
    int32_t *route_log_dev = nullptr;   // device ring of ROUTE_LOG entries of MOE_MAX_TOPK selections, written by the gate kernel
    struct PendingStep { moe_layer *layer; uint32_t slot; };
    std::vector<PendingStep> pending;   // steps enqueued that way whose bookkeeping is still to be done, oldest first
    static constexpr uint32_t ROUTE_LOG = ROUTE_LOG_ENTRIES;
};

struct moe_layer {
    moe_ctx *ctx = nullptr;
    moe_layer_config_t cfg{};
    BlobLayout lay;
    LayerCache cache;
    Counters st;
    float *gate_w_dev = nullptr;
    uint16_t *gamma_dev = nullptr;
    uint8_t *host_blobs = nullptr;
    std::vector<uint32_t> loaded;       // bit m set: matrix m of the expert was loaded
    std::atomic<bool> wide_meta{false}; // a loaded (scale, zero) pair is too large for the rank-1 matrix-core form (below)
    std::vector<int32_t> own_bufs;      // the k pool buffers created for this layer
    // Where each expert's blob lives on the host: buffer index into host_blobs, or -1 while it is on the device
    // (swap mode only; otherwise expert e stays in buffer e for good).
    bool swap = false;
    std::vector<int32_t> host_buf_of;
    int32_t spare_host = -1;            // swap mode: the one host buffer holding no expert
    std::vector<int32_t> host_reader;   // per host buffer: pool buffer whose `ready` event covers its last read, or -1
    std::vector<int32_t> host_writer;   // per host buffer: pool buffer whose `drained` event covers its last write, or -1
    std::vector<std::vector<uint8_t>> pack_tmp;   // swap mode: experts 0..k-1 are packed here until they move to the device
    uint64_t steps_device_routed = 0;   // steps enqueued without waiting for their gate
    bool stepped = false;               // the layer has taken part in a step since it was created or reset: its blobs may be in flight
};

static int32_t fold_pending(moe_ctx *c);   // bookkeeping of device-routed steps; every reader of cache state calls it first

static int32_t n_host_bufs(const moe_layer_config_t &c)
{
    return (c.flags & MOE_LAYER_SWAP) ? c.n_experts - c.cache_slots + 1 : c.n_experts;
}

static uint64_t align_u64(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

static bool ctx_cfg_ok(const moe_ctx_config_t *c)
{
    return c && c->n_staging >= 0 && c->n_staging <= 64 && c->max_batch >= 1 && c->max_batch <= MOE_MAX_BATCH &&
           c->max_hidden >= 64 && c->max_hidden % 64 == 0 && c->max_hidden <= 8192 && c->max_ffn >= 64 &&
           c->max_ffn % 64 == 0 && c->max_ffn <= 16384 && c->max_top_k >= 1 && c->max_top_k <= MOE_MAX_TOPK &&
           c->max_expert_bytes > 0;
}

static bool layer_cfg_ok(const moe_layer_config_t *c)
{
    return c && c->n_experts >= 1 && c->n_experts <= MOE_MAX_EXPERTS && c->top_k >= 1 && c->top_k <= MOE_MAX_TOPK &&
           c->top_k <= c->n_experts && c->cache_slots >= c->top_k && c->cache_slots <= c->n_experts &&
           c->prefetch_m >= 0 && c->prefetch_m <= MOE_MAX_GUESS && c->rms_eps >= 0.f &&
           (c->init_policy == 0 || c->init_policy == 1) && (c->flags & ~(MOE_LAYER_NO_CACHE | MOE_LAYER_SWAP)) == 0 &&
           (!(c->flags & MOE_LAYER_SWAP) || (c->init_policy == 1 && !(c->flags & MOE_LAYER_NO_CACHE))) &&
           c->scale_group >= 0 && blob_layout(c->hidden, c->ffn, c->bits, c->group, c->scale_group).ok;
}

struct ScratchPlan { uint64_t staging, h, a, yacc, ypart, ytab, ypart_extra_floats, x0, x1, barrier, route, route_log, total; };

static ScratchPlan plan_scratch(const moe_ctx_config_t *c)
{
    ScratchPlan p{};
    const uint64_t buf = align_u64(c->max_expert_bytes, 4096);
    uint64_t off = 0;
    p.staging = off; off += buf * (uint64_t)c->n_staging;
    p.h = off;    off += align_u64((uint64_t)c->max_batch * c->max_hidden * 2, 256);
    p.a = off;    off += align_u64((uint64_t)c->max_batch * c->max_top_k * c->max_ffn * 2, 256);
    p.yacc = off; off += align_u64((uint64_t)c->max_batch * c->max_hidden * 4, 256);
    const uint64_t pairs = (uint64_t)c->max_batch * c->max_top_k;
    // rows for the partial sums of split contractions: sixteen parts for small batches, four for prompt-sized ones
    p.ypart_extra_floats = std::max(std::min<uint64_t>(2048, 16 * pairs), std::min<uint64_t>(16384, 4 * pairs)) * c->max_hidden;
    p.ypart = off; off += align_u64((pairs * c->max_hidden + p.ypart_extra_floats) * 4, 256);
    p.ytab = off; off += align_u64(pairs * 4, 256);
    p.x0 = off;   off += align_u64((uint64_t)c->max_batch * c->max_hidden * 2, 256);
    p.x1 = off;   off += align_u64((uint64_t)c->max_batch * c->max_hidden * 2, 256);
    p.barrier = off; off += 4096 + 2 * SEQ_FLAG_STRIDE * 4;     // one flag per block of the persistent kernels (at most 1024 compute units); then [2 experts][blocks]
    p.route = off; off += 256;        // device-side routing: MOE_MAX_TOPK selections and as many combine weights
    p.route_log = off; off += align_u64((uint64_t)ROUTE_LOG_ENTRIES * MOE_MAX_TOPK * sizeof(int32_t), 256);
    p.total = off;
    return p;
}

// ---------------------------------------------------------------------------------------------
// sizes
// ---------------------------------------------------------------------------------------------

extern "C" uint64_t moe_expert_blob_bytes(int32_t hidden, int32_t ffn, int32_t bits, int32_t group)
{
    BlobLayout b = blob_layout(hidden, ffn, bits, group);
    return b.ok ? b.total : 0;
}

extern "C" uint64_t moe_expert_blob_bytes_2level(int32_t hidden, int32_t ffn, int32_t bits, int32_t group, int32_t scale_group)
{
    BlobLayout b = blob_layout(hidden, ffn, bits, group, scale_group < 0 ? -1 : scale_group);
    return (scale_group >= 0 && b.ok) ? b.total : 0;
}

extern "C" uint64_t moe_ctx_dev_bytes(const moe_ctx_config_t *cfg)
{
    if (!ctx_cfg_ok(cfg)) return 0;
    return plan_scratch(cfg).total;
}

extern "C" uint64_t moe_layer_dev_bytes(const moe_ctx_t *ctx, const moe_layer_config_t *cfg)
{
    if (!ctx || !layer_cfg_ok(cfg)) return 0;
    return ctx->buf_bytes * (uint64_t)cfg->cache_slots + align_u64((uint64_t)cfg->n_experts * cfg->hidden * 4, 256) +
           align_u64((uint64_t)cfg->hidden * 2, 256);
}

extern "C" uint64_t moe_layer_host_bytes(const moe_layer_config_t *cfg)
{
    if (!layer_cfg_ok(cfg)) return 0;
    return blob_layout(cfg->hidden, cfg->ffn, cfg->bits, cfg->group, cfg->scale_group).total * (uint64_t)n_host_bufs(*cfg);
}

// ---------------------------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------------------------

extern "C" int32_t moe_ctx_create(const moe_ctx_config_t *cfg, void *dev_arena, uint64_t dev_arena_bytes,
                                  void *compute_stream, void *copy_stream, moe_ctx_t **out)
try {
    if (!out) return fail(MOE_EINVAL, "moe_ctx_create: out is null");
    *out = nullptr;
    if (!ctx_cfg_ok(cfg)) return fail(MOE_EINVAL, "moe_ctx_create: bad configuration");
    moe_ctx *c = new (std::nothrow) moe_ctx();
    if (!c) return fail(MOE_ENOMEM, "moe_ctx_create: out of host memory");
    std::unique_ptr<moe_ctx, int32_t (*)(moe_ctx *)> own(c, moe_ctx_destroy);   // released into *out on success
    c->cfg = *cfg;
    c->host_only = (cfg->flags & MOE_CTX_HOST_ONLY) != 0;
    c->buf_bytes = align_u64(cfg->max_expert_bytes, 4096);
    c->bufs.resize(cfg->n_staging);
    for (int i = 0; i < cfg->n_staging; ++i) c->pool.free_staging.push_back(i);
    if (c->host_only) {
        c->gate_out = static_cast<GateHostOut *>(calloc(1, sizeof(GateHostOut)));
        if (!c->gate_out) return fail(MOE_ENOMEM, "moe_ctx_create: out of host memory");
        *out = own.release();
        return MOE_OK;
    }
    const ScratchPlan p = plan_scratch(cfg);
    if (!dev_arena || ((uintptr_t)dev_arena & 255)) return fail(MOE_EINVAL, "moe_ctx_create: device arena null or not 256-byte aligned");
    if (dev_arena_bytes < p.total) return fail(MOE_ENOMEM, "moe_ctx_create: device arena has %llu bytes, %llu needed", (unsigned long long)dev_arena_bytes, (unsigned long long)p.total);
    if (compute_stream == copy_stream) return fail(MOE_EINVAL, "moe_ctx_create: compute and copy stream must differ");
    c->compute = static_cast<hipStream_t>(compute_stream);
    c->copy = static_cast<hipStream_t>(copy_stream);
    uint8_t *base = static_cast<uint8_t *>(dev_arena);
    for (int i = 0; i < cfg->n_staging; ++i) c->bufs[i].ptr = base + p.staging + c->buf_bytes * i;
    c->h_buf = reinterpret_cast<uint16_t *>(base + p.h);
    c->a_buf = reinterpret_cast<uint16_t *>(base + p.a);
    c->yacc = reinterpret_cast<float *>(base + p.yacc);
    c->ypart = reinterpret_cast<float *>(base + p.ypart);
    c->ytab = reinterpret_cast<uint32_t *>(base + p.ytab);
    c->ypart_extra_floats = p.ypart_extra_floats;
    c->xbuf[0] = reinterpret_cast<uint16_t *>(base + p.x0);
    c->xbuf[1] = reinterpret_cast<uint16_t *>(base + p.x1);
    c->barrier = reinterpret_cast<uint32_t *>(base + p.barrier);
    c->seq_flags = c->barrier + 1024;
    c->route_idx = reinterpret_cast<int32_t *>(base + p.route);
    c->route_w = reinterpret_cast<float *>(base + p.route + 128);
    c->route_log_dev = reinterpret_cast<int32_t *>(base + p.route_log);
    hipError_t e = hipMemset(c->barrier, 0, 4096 + 2 * SEQ_FLAG_STRIDE * 4);
    if (e == hipSuccess) {
        int dev = 0;
        hipDeviceProp_t prop;
        e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
        if (e == hipSuccess) c->n_cu = prop.multiProcessorCount;
        // the device address of the file-scope scratch array, once per device, with that device current
        if (e == hipSuccess && (dev < 0 || dev >= NOALLOC_MAX_DEVICES)) return fail(MOE_EINVAL, "moe_ctx_create: device ordinal %d out of range", dev);
        if (e == hipSuccess && !g_scratch_ptr[dev]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e == hipSuccess && !p) return fail(MOE_EHIP, "moe_ctx_create: the scratch array has no device address");
            if (e == hipSuccess) g_scratch_ptr[dev] = static_cast<uint8_t *>(p);
        }
        if (e == hipSuccess) c->noalloc_scratch = g_scratch_ptr[dev];
    }
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void **>(&c->gate_out), sizeof(GateHostOut), hipHostMallocMapped);
    if (e == hipSuccess) e = hipHostGetDevicePointer(reinterpret_cast<void **>(&c->gate_out_dev), c->gate_out, 0);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void **>(&c->route_log), (size_t)moe_ctx::ROUTE_LOG * MOE_MAX_TOPK * sizeof(int32_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_gate, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_compute, hipEventDisableTiming);
    for (int i = 0; i < cfg->n_staging && e == hipSuccess; ++i) {
        e = hipEventCreateWithFlags(&c->bufs[i].ready, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->bufs[i].drained, hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        g_hip_err = (int32_t)e;
        return fail(MOE_EHIP, "moe_ctx_create: HIP set-up failed: %s", hipGetErrorString(e));
    }
    memset(c->gate_out, 0, sizeof(GateHostOut));
    *out = own.release();
    return MOE_OK;
} catch (...) {
    return on_exception("moe_ctx_create");
}

extern "C" int32_t moe_ctx_destroy(moe_ctx_t *c)
try {
    if (!c) return MOE_OK;
    if (c->host_only) {
        free(c->gate_out);
    } else {
        if (c->compute) (void)hipStreamSynchronize(c->compute);
        if (c->copy) (void)hipStreamSynchronize(c->copy);
        if (c->writeback) { (void)hipStreamSynchronize(c->writeback); (void)hipStreamDestroy(c->writeback); }
        for (PoolBuf &b : c->bufs) {
            if (b.ready) (void)hipEventDestroy(b.ready);
            if (b.drained) (void)hipEventDestroy(b.drained);
        }
        for (int k = 0; k < PROF_KINDS; ++k) {
            for (hipEvent_t e : c->prof.kind[k].start) (void)hipEventDestroy(e);
            for (hipEvent_t e : c->prof.kind[k].stop) (void)hipEventDestroy(e);
        }
        if (c->prof.base) (void)hipEventDestroy(c->prof.base);
        if (c->ev_gate) (void)hipEventDestroy(c->ev_gate);
        if (c->ev_compute) (void)hipEventDestroy(c->ev_compute);
        if (c->gate_out) (void)hipHostFree(c->gate_out);
        if (c->route_log) (void)hipHostFree(c->route_log);
    }
    delete c;
    return MOE_OK;
} catch (...) {
    return on_exception("moe_ctx_destroy");
}

// ---------------------------------------------------------------------------------------------
// layer
// ---------------------------------------------------------------------------------------------

static void cache_init(moe_layer *l)
{
    LayerCache &c = l->cache;
    c.k = l->cfg.cache_slots;
    c.n_experts = l->cfg.n_experts;
    c.slot_expert.assign(c.k, -1);
    c.slot_stamp.assign(c.k, 0);
    c.slot_buf = l->own_bufs;
    c.staged.clear();
    l->st = Counters();
    l->steps_device_routed = 0;
}

extern "C" int32_t moe_layer_create(moe_ctx_t *ctx, const moe_layer_config_t *cfg, const float *gate_w_host,
                                    const uint16_t *rms_gamma_host, void *dev_mem, void *pinned_host_mem,
                                    moe_layer_t **out)
try {
    if (!out) return fail(MOE_EINVAL, "moe_layer_create: out is null");
    *out = nullptr;
    if (!ctx) return fail(MOE_EINVAL, "moe_layer_create: ctx is null");
    if (!layer_cfg_ok(cfg)) return fail(MOE_EINVAL, "moe_layer_create: bad or unsupported configuration");
    if (!gate_w_host || !pinned_host_mem) return fail(MOE_EINVAL, "moe_layer_create: null gate or host arena");
    BlobLayout lay = blob_layout(cfg->hidden, cfg->ffn, cfg->bits, cfg->group, cfg->scale_group);
    if (lay.total > ctx->buf_bytes) return fail(MOE_EINVAL, "moe_layer_create: expert blob (%llu B) exceeds the context's buffer size (%llu B)", (unsigned long long)lay.total, (unsigned long long)ctx->buf_bytes);
    if (cfg->hidden > ctx->cfg.max_hidden || cfg->ffn > ctx->cfg.max_ffn || cfg->top_k > ctx->cfg.max_top_k)
        return fail(MOE_EINVAL, "moe_layer_create: layer exceeds the context's maxima");
    if ((uintptr_t)pinned_host_mem & 63) return fail(MOE_EINVAL, "moe_layer_create: host arena not 64-byte aligned");
    moe_layer *l = new (std::nothrow) moe_layer();
    if (!l) return fail(MOE_ENOMEM, "moe_layer_create: out of host memory");
    std::unique_ptr<moe_layer> own(l);      // released into *out on success
    l->ctx = ctx;
    l->cfg = *cfg;
    l->lay = lay;
    l->host_blobs = static_cast<uint8_t *>(pinned_host_mem);
    l->loaded.assign(cfg->n_experts, 0);
    l->swap = (cfg->flags & MOE_LAYER_SWAP) != 0;
    l->host_buf_of.resize(cfg->n_experts);
    for (int e = 0; e < cfg->n_experts; ++e)            // swap: experts 0..k-1 start on the device, the rest fill the host buffers
        l->host_buf_of[e] = l->swap ? (e < cfg->cache_slots ? -1 : e - cfg->cache_slots) : e;
    l->spare_host = l->swap ? cfg->n_experts - cfg->cache_slots : -1;
    l->host_reader.assign(n_host_bufs(*cfg), -1);
    l->host_writer.assign(n_host_bufs(*cfg), -1);
    l->pack_tmp.resize(l->swap ? cfg->cache_slots : 0);
    const int first = (int)ctx->bufs.size();
    if (!ctx->host_only) {
        if (!dev_mem || ((uintptr_t)dev_mem & 255)) return fail(MOE_EINVAL, "moe_layer_create: device memory null or not 256-byte aligned");
        uint8_t *base = static_cast<uint8_t *>(dev_mem);
        const uint64_t gate_bytes = (uint64_t)cfg->n_experts * cfg->hidden * 4;
        l->gate_w_dev = reinterpret_cast<float *>(base + ctx->buf_bytes * cfg->cache_slots);
        l->gamma_dev = reinterpret_cast<uint16_t *>(reinterpret_cast<uint8_t *>(l->gate_w_dev) + align_u64(gate_bytes, 256));
        hipError_t e = hipMemcpy(l->gate_w_dev, gate_w_host, gate_bytes, hipMemcpyHostToDevice);
        std::vector<uint16_t> ones;
        if (e == hipSuccess) {
            const uint16_t *g = rms_gamma_host;
            if (!g) { ones.assign(cfg->hidden, 0x3c00); g = ones.data(); }
            e = hipMemcpy(l->gamma_dev, g, (size_t)cfg->hidden * 2, hipMemcpyHostToDevice);
        }
        std::vector<PoolBuf> fresh(cfg->cache_slots);
        for (int s = 0; s < cfg->cache_slots && e == hipSuccess; ++s) {
            fresh[s].ptr = base + ctx->buf_bytes * s;
            e = hipEventCreateWithFlags(&fresh[s].ready, hipEventDisableTiming);
            if (e == hipSuccess) e = hipEventCreateWithFlags(&fresh[s].drained, hipEventDisableTiming);
        }
        if (e == hipSuccess && (cfg->flags & MOE_LAYER_SWAP) && !ctx->writeback)
            e = hipStreamCreateWithFlags(&ctx->writeback, hipStreamNonBlocking);
        if (e != hipSuccess) {
            for (PoolBuf &b : fresh) { if (b.ready) (void)hipEventDestroy(b.ready); if (b.drained) (void)hipEventDestroy(b.drained); }
            g_hip_err = (int32_t)e;
            return fail(MOE_EHIP, "moe_layer_create: HIP set-up failed: %s", hipGetErrorString(e));
        }
        for (PoolBuf &b : fresh) ctx->bufs.push_back(b);
    } else {
        ctx->bufs.resize(first + cfg->cache_slots);
    }
    for (int s = 0; s < cfg->cache_slots; ++s) l->own_bufs.push_back(first + s);
    cache_init(l);
    ctx->n_layers++;
    *out = own.release();
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_create");
}

extern "C" int32_t moe_layer_destroy(moe_layer_t *l)
try {
    if (!l) return MOE_OK;
    (void)fold_pending(l->ctx);
    if (!l->ctx->host_only) {
        (void)hipStreamSynchronize(l->ctx->compute);
        (void)hipStreamSynchronize(l->ctx->copy);
        if (l->ctx->writeback) (void)hipStreamSynchronize(l->ctx->writeback);
    }
    l->ctx->n_layers--;
    delete l;   // pool buffers and their events stay with the context until it is destroyed
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_destroy");
}

static bool all_loaded(const moe_layer *l)
{
    for (uint32_t m : l->loaded)
        if (m != 7u) return false;
    return true;
}

// Host memory of expert e's blob: its host buffer, or, in swap mode while an expert that starts on the device is
// still being loaded, its packing area.  nullptr when the blob is on the device only.
static uint8_t *host_blob(moe_layer *l, int32_t e)
{
    if (l->host_buf_of[e] >= 0) return l->host_blobs + (uint64_t)l->host_buf_of[e] * l->lay.total;
    if (l->swap && e < (int32_t)l->pack_tmp.size() && !l->pack_tmp[e].empty()) return l->pack_tmp[e].data();
    return nullptr;
}

static int32_t warm_fill(moe_layer *l, int32_t e)
{
    // init_policy 1: expert e < k sits in slot e from the start
    LayerCache &c = l->cache;
    c.slot_expert[e] = e;
    c.slot_stamp[e] = ++l->ctx->pool.clock;
    if (!l->ctx->host_only) {
        PoolBuf &b = l->ctx->bufs[c.slot_buf[e]];
        HIPCHK(hipMemcpy(b.ptr, host_blob(l, e), l->lay.total, hipMemcpyHostToDevice));
    }
    if (l->swap) std::vector<uint8_t>().swap(l->pack_tmp[e]);    // the device copy is now the only one
    return MOE_OK;
}

// Common part of the two load entry points: checks, threading over rows, bookkeeping.  pack(r, dst) packs row r.
template <typename PackRow>
static int32_t load_matrix(moe_layer *l, int32_t expert, int32_t matrix, const uint8_t *codes, PackRow pack)
{
    if (expert < 0 || expert >= l->cfg.n_experts || matrix < 0 || matrix > 2)
        return fail(MOE_EINVAL, "moe_layer_load_expert: expert %d / matrix %d out of range", expert, matrix);
    // Once a layer has stepped, copies of its blobs may be in flight, resident copies would go stale, and in swap
    // mode an expert on the device has no host buffer to pack into: loading ends with the first step.
    if (l->stepped) return fail(MOE_ESTATE, "moe_layer_load_expert: the layer has already taken part in a step; experts are loaded before the first step (or after moe_layer_reset)");
    const BlobLayout &b = l->lay;
    const MatLayout &m = mat_of(b, matrix);
    if (l->swap && expert < l->cfg.cache_slots) {
        if (l->loaded[expert] == 7u) return fail(MOE_ESTATE, "moe_layer_load_expert: expert %d already moved to the device (swap mode)", expert);
        if (l->pack_tmp[expert].empty()) {
            try { l->pack_tmp[expert].resize(b.total); } catch (...) { return fail(MOE_ENOMEM, "moe_layer_load_expert: out of host memory"); }
        }
    }
    uint8_t *blob = host_blob(l, expert);
    if (!blob) return fail(MOE_ESTATE, "moe_layer_load_expert: expert %d has no host buffer to be packed into", expert);
    const uint32_t qmax = (1u << b.bits) - 1;
    const unsigned hw = std::max(1u, std::min(16u, std::thread::hardware_concurrency()));
    const unsigned nthreads = (uint64_t)m.rows * m.cols < (1u << 20) ? 1 : hw;
    std::atomic<int> bad{0};
    auto work = [&](uint32_t r0, uint32_t r1) {
        for (uint32_t r = r0; r < r1; ++r) {
            const uint8_t *cr = codes + (uint64_t)r * m.cols;
            uint32_t mx = 0;
            for (uint32_t i = 0; i < m.cols; ++i) mx |= cr[i];
            if (mx > qmax) { bad.store(1); return; }
            pack(r, blob + row_offset(b, matrix, r));
        }
    };
    if (nthreads == 1) {
        work(0, m.rows);
    } else {
        std::vector<std::thread> th;
        th.reserve(nthreads);
        const uint32_t per = (m.rows + nthreads - 1) / nthreads;
        for (unsigned t = 0; t < nthreads; ++t) {
            uint32_t r0 = t * per, r1 = std::min(m.rows, r0 + per);
            if (r0 >= r1) continue;
            // a thread that cannot be started (resource limits) leaves its share to this one: a joinable thread must
            // never be destroyed by an exception on its way out
            try { th.emplace_back(work, r0, r1); } catch (...) { work(r0, r1); }
        }
        for (std::thread &t : th) t.join();
    }
    if (bad.load()) return fail(MOE_EINVAL, "moe_layer_load_expert: a code exceeds %u", qmax);
    l->loaded[expert] |= 1u << matrix;
    if (l->loaded[expert] == 7u && l->cfg.init_policy == 1 && expert < l->cfg.cache_slots) return warm_fill(l, expert);
    return MOE_OK;
}

// binary16 bit pattern -> float (host side)
static float half_bits_to_float(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16, ex = (h >> 10) & 0x1fu, man = h & 0x3ffu;
    uint32_t bits;
    if (ex == 0x1fu) bits = sign | 0x7f800000u | (man << 13);
    else if (ex) bits = sign | ((ex + 112u) << 23) | (man << 13);
    else if (!man) bits = sign;
    else {
        int e = -1;
        uint32_t m = man;
        do { m <<= 1; ++e; } while (!(m & 0x400u));
        bits = sign | ((uint32_t)(112 - e) << 23) | ((m & 0x3ffu) << 13);
    }
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

// The rank-1 matrix-core form computes (1024 + z) * s in fp16: pairs for which that product (or anything else about
// them) leaves the comfortable part of the fp16 range make the layer fall back to the form that subtracts first.
static bool pair_fits_rank1(uint16_t scale, uint16_t zero)
{
    const float s = half_bits_to_float(scale), z = half_bits_to_float(zero);
    return std::isfinite(s) && std::isfinite(z) && (1024.f + std::fabs(z)) * std::fabs(s) <= 16384.f;
}

extern "C" int32_t moe_layer_load_expert(moe_layer_t *l, int32_t expert, int32_t matrix, const uint8_t *codes,
                                         const uint16_t *scale, const uint16_t *zero)
try {
    if (!l || !codes || !scale || !zero) return fail(MOE_EINVAL, "moe_layer_load_expert: null argument");
    if (l->lay.scale_group) return fail(MOE_ESTATE, "moe_layer_load_expert: the layer has two-level metadata; use moe_layer_load_expert_2level");
    if (matrix < 0 || matrix > 2) return fail(MOE_EINVAL, "moe_layer_load_expert: matrix %d out of range", matrix);
    const BlobLayout &b = l->lay;
    const MatLayout &m = mat_of(b, matrix);
    const uint32_t groups = m.cols / b.group;
    const bool watch = b.bits == 4 && b.group == 64;     // the formats the matrix cores take
    return load_matrix(l, expert, matrix, codes, [&](uint32_t r, uint8_t *dst) {
        const uint16_t *sr = scale + (uint64_t)r * groups, *zr = zero + (uint64_t)r * groups;
        if (watch && !l->wide_meta.load(std::memory_order_relaxed))
            for (uint32_t g = 0; g < groups; ++g)
                if (!pair_fits_rank1(sr[g], zr[g])) { l->wide_meta.store(true, std::memory_order_relaxed); break; }
        pack_row(b, m, codes + (uint64_t)r * m.cols, sr, zr, dst);
    });
} catch (...) {
    return on_exception("moe_layer_load_expert");
}

extern "C" int32_t moe_layer_load_expert_2level(moe_layer_t *l, int32_t expert, int32_t matrix, const uint8_t *codes,
                                                const uint8_t *scale_code, const uint8_t *zero_code, const uint16_t *run_meta)
try {
    if (!l || !codes || !scale_code || !zero_code || !run_meta) return fail(MOE_EINVAL, "moe_layer_load_expert_2level: null argument");
    if (!l->lay.scale_group) return fail(MOE_ESTATE, "moe_layer_load_expert_2level: the layer has one-level metadata; use moe_layer_load_expert");
    if (matrix < 0 || matrix > 2) return fail(MOE_EINVAL, "moe_layer_load_expert_2level: matrix %d out of range", matrix);
    const BlobLayout &b = l->lay;
    const MatLayout &m = mat_of(b, matrix);
    const uint32_t groups = m.cols / b.group, runs = (groups + m.run_len - 1) / m.run_len;
    return load_matrix(l, expert, matrix, codes, [&](uint32_t r, uint8_t *dst) {
        pack_row_meta8(b, m, codes + (uint64_t)r * m.cols, scale_code + (uint64_t)r * groups, zero_code + (uint64_t)r * groups,
                       run_meta + (uint64_t)r * runs * 4, dst);
    });
} catch (...) {
    return on_exception("moe_layer_load_expert_2level");
}

extern "C" int32_t moe_layer_peek_weight(const moe_layer_t *l, int32_t expert, int32_t matrix, int32_t row, int32_t col,
                                         uint8_t *code, uint16_t *scale, uint16_t *zero)
try {
    if (!l || !code || !scale || !zero) return fail(MOE_EINVAL, "moe_layer_peek_weight: null argument");
    if (expert < 0 || expert >= l->cfg.n_experts || matrix < 0 || matrix > 2)
        return fail(MOE_EINVAL, "moe_layer_peek_weight: expert or matrix out of range");
    const MatLayout &m = mat_of(l->lay, matrix);
    if (row < 0 || (uint32_t)row >= m.rows || col < 0 || (uint32_t)col >= m.cols)
        return fail(MOE_EINVAL, "moe_layer_peek_weight: row or column out of range");
    if (!(l->loaded[expert] & (1u << matrix))) return fail(MOE_ESTATE, "moe_layer_peek_weight: matrix not loaded");
    const uint8_t *blob = host_blob(const_cast<moe_layer *>(l), expert);
    if (!blob) return fail(MOE_ESTATE, "moe_layer_peek_weight: expert %d is on the device only (swap mode)", expert);
    if (l->lay.scale_group) {               // two-level metadata: the byte codes, widened
        uint8_t sc = 0, zc = 0;
        uint16_t quad[4];
        peek_row_meta8(l->lay, m, blob + row_offset(l->lay, matrix, row), col, code, &sc, &zc, quad);
        *scale = sc; *zero = zc;
        return MOE_OK;
    }
    peek_row(l->lay, m, blob + row_offset(l->lay, matrix, row), col, code, scale, zero);
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_peek_weight");
}

extern "C" int32_t moe_layer_peek_run_meta(const moe_layer_t *l, int32_t expert, int32_t matrix, int32_t row, int32_t col,
                                           uint16_t *run_meta)
try {
    if (!l || !run_meta) return fail(MOE_EINVAL, "moe_layer_peek_run_meta: null argument");
    if (!l->lay.scale_group) return fail(MOE_ESTATE, "moe_layer_peek_run_meta: the layer has one-level metadata");
    if (expert < 0 || expert >= l->cfg.n_experts || matrix < 0 || matrix > 2)
        return fail(MOE_EINVAL, "moe_layer_peek_run_meta: expert or matrix out of range");
    const MatLayout &m = mat_of(l->lay, matrix);
    if (row < 0 || (uint32_t)row >= m.rows || col < 0 || (uint32_t)col >= m.cols)
        return fail(MOE_EINVAL, "moe_layer_peek_run_meta: row or column out of range");
    if (!(l->loaded[expert] & (1u << matrix))) return fail(MOE_ESTATE, "moe_layer_peek_run_meta: matrix not loaded");
    const uint8_t *blob = host_blob(const_cast<moe_layer *>(l), expert);
    if (!blob) return fail(MOE_ESTATE, "moe_layer_peek_run_meta: expert %d is on the device only (swap mode)", expert);
    uint8_t c, sc, zc;
    peek_row_meta8(l->lay, m, blob + row_offset(l->lay, matrix, row), col, &c, &sc, &zc, run_meta);
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_peek_run_meta");
}

// ---------------------------------------------------------------------------------------------
// profiling
// ---------------------------------------------------------------------------------------------

static int32_t prof_drain(moe_ctx *c, int k)
{
    ProfKind &p = c->prof.kind[k];
    if (!p.used) return MOE_OK;
    HIPCHK(hipEventSynchronize(p.stop[p.used - 1]));
    for (size_t i = 0; i < p.used; ++i) {
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, p.start[i], p.stop[i]));
        p.ms += ms;
    }
    p.used = 0;
    return MOE_OK;
}

// Record the start event of a launch of kind k on stream s; *slot receives the ring index (or -1 when off).
static int32_t prof_begin(moe_ctx *c, int k, hipStream_t s, uint64_t bytes, int *slot)
{
    *slot = -1;
    if (!c->prof.on) return MOE_OK;
    ProfKind &p = c->prof.kind[k];
    if (p.used == Profiler::RING) { int32_t rc = prof_drain(c, k); if (rc) return rc; }
    if (p.used == p.start.size()) {
        hipEvent_t a, b;
        HIPCHK(hipEventCreate(&a));
        HIPCHK(hipEventCreate(&b));
        p.start.push_back(a);
        p.stop.push_back(b);
    }
    HIPCHK(hipEventRecord(p.start[p.used], s));
    *slot = (int)p.used;
    p.launches++;
    p.bytes += bytes;
    return MOE_OK;
}

static int32_t prof_end(moe_ctx *c, int k, hipStream_t s, int slot)
{
    if (slot < 0) return MOE_OK;
    ProfKind &p = c->prof.kind[k];
    HIPCHK(hipEventRecord(p.stop[slot], s));
    p.used = (size_t)slot + 1;
    return MOE_OK;
}

extern "C" int32_t moe_ctx_profile_enable(moe_ctx_t *c, int32_t on)
try {
    if (!c) return fail(MOE_EINVAL, "moe_ctx_profile_enable: ctx is null");
    if (c->host_only) return fail(MOE_ESTATE, "moe_ctx_profile_enable: host-only context");
    HIPCHK(hipStreamSynchronize(c->compute));
    HIPCHK(hipStreamSynchronize(c->copy));
    if (c->writeback) HIPCHK(hipStreamSynchronize(c->writeback));
    for (int k = 0; k < PROF_KINDS; ++k) {
        ProfKind &p = c->prof.kind[k];
        p.used = 0; p.launches = 0; p.bytes = 0; p.ms = 0.0;
        // create the events up front, so that no event is created inside a region the caller is timing
        while (on && p.start.size() < Profiler::PREALLOC) {
            hipEvent_t a, b;
            HIPCHK(hipEventCreate(&a));
            HIPCHK(hipEventCreate(&b));
            p.start.push_back(a);
            p.stop.push_back(b);
        }
    }
    if (on) {
        if (!c->prof.base) HIPCHK(hipEventCreate(&c->prof.base));
        HIPCHK(hipEventRecord(c->prof.base, c->compute));
        HIPCHK(hipEventSynchronize(c->prof.base));
    }
    c->prof.on = on != 0;
    return MOE_OK;
} catch (...) {
    return on_exception("moe_ctx_profile_enable");
}

extern "C" int32_t moe_ctx_profile_timeline(moe_ctx_t *c, int32_t kind, double *start_ms, double *stop_ms, int32_t cap, int32_t *n)
try {
    if (!c || !n || kind < 0 || kind >= PROF_KINDS || cap < 0 || (cap > 0 && (!start_ms || !stop_ms)))
        return fail(MOE_EINVAL, "moe_ctx_profile_timeline: bad argument");
    if (c->host_only || !c->prof.base) return fail(MOE_ESTATE, "moe_ctx_profile_timeline: profiling was never switched on");
    HIPCHK(hipStreamSynchronize(c->compute));
    HIPCHK(hipStreamSynchronize(c->copy));
    if (c->writeback) HIPCHK(hipStreamSynchronize(c->writeback));
    const ProfKind &p = c->prof.kind[kind];
    *n = (int32_t)std::min<size_t>(p.used, (size_t)INT32_MAX);
    for (size_t i = 0; i < p.used && i < (size_t)cap; ++i) {
        float a = 0.f, b = 0.f;
        HIPCHK(hipEventElapsedTime(&a, c->prof.base, p.start[i]));
        HIPCHK(hipEventElapsedTime(&b, c->prof.base, p.stop[i]));
        start_ms[i] = a;
        stop_ms[i] = b;
    }
    return MOE_OK;
} catch (...) {
    return on_exception("moe_ctx_profile_timeline");
}

extern "C" int32_t moe_ctx_profile_read(moe_ctx_t *c, moe_profile_t *out)
try {
    if (!c || !out) return fail(MOE_EINVAL, "moe_ctx_profile_read: null argument");
    if (c->host_only) return fail(MOE_ESTATE, "moe_ctx_profile_read: host-only context");
    HIPCHK(hipStreamSynchronize(c->compute));
    HIPCHK(hipStreamSynchronize(c->copy));
    if (c->writeback) HIPCHK(hipStreamSynchronize(c->writeback));
    moe_profile_entry_t *dst[PROF_KINDS] = {&out->gate, &out->w13, &out->w2, &out->copy, &out->ffn, &out->writeback};
    for (int k = 0; k < PROF_KINDS; ++k) {
        int32_t rc = prof_drain(c, k);
        if (rc) return rc;
        dst[k]->launches = c->prof.kind[k].launches;
        dst[k]->bytes = c->prof.kind[k].bytes;
        dst[k]->total_ms = c->prof.kind[k].ms;
    }
    return MOE_OK;
} catch (...) {
    return on_exception("moe_ctx_profile_read");
}

// ---------------------------------------------------------------------------------------------
// bookkeeping of one step (host only)
// ---------------------------------------------------------------------------------------------

struct StepPlan {
    std::vector<AccessRec> access;
    std::vector<CopyOp> demand;     // misses, and the tails of confirmed speculative loads
    std::vector<int> demand_of;     // per access: index into `demand`, or -1
    std::vector<CopyOp> spec;       // for the next layer
    std::vector<CopyOp> writeback;  // swap mode: evicted expert `expert` from pool buffer `buf` to host buffer `host_buf`
    std::vector<int> writeback_of;  // per access: index into `writeback`, or -1
    bool victim_needed = false;     // an expert needed in this step was evicted during it
    bool victims_resident = true;   // ... and every such expert was on the device when the step began (its access is a HIT)
};

static int32_t plan_step(moe_layer *l, moe_layer *next, const int32_t *idx, int32_t batch, const double *guess_score,
                         moe_step_trace_t *tr, StepPlan &plan)
{
    const moe_layer_config_t &cf = l->cfg;
    std::vector<int32_t> needed;
    for (int i = 0; i < batch * cf.top_k; ++i) {
        if (idx[i] < 0 || idx[i] >= cf.n_experts) return fail(MOE_EINVAL, "routing index %d out of range", idx[i]);
        needed.push_back(idx[i]);
    }
    std::sort(needed.begin(), needed.end());
    needed.erase(std::unique(needed.begin(), needed.end()), needed.end());
    std::vector<CopyOp> misses;
    // loads go to a free staging buffer instead of the victim's own when that one cannot be overwritten yet
    const bool redirect = l->swap || (int)needed.size() > cf.cache_slots;
    resolve_accesses(l->cache, l->ctx->pool, l->st, needed, (cf.flags & MOE_LAYER_NO_CACHE) != 0, plan.access, misses, redirect);
    size_t next_miss = 0;
    for (const AccessRec &a : plan.access) {
        if (a.victim >= 0 && std::binary_search(needed.begin(), needed.end(), a.victim)) {
            plan.victim_needed = true;
            bool hit = false;
            for (const AccessRec &v : plan.access) hit |= (v.expert == a.victim && v.status == MOE_HIT);
            plan.victims_resident &= hit;
        }
        PoolBuf &pb = l->ctx->bufs[a.buf];
        int di = -1;
        if (a.status == MOE_MISS) {
            CopyOp op = misses[next_miss++];
            op.offset = 0; op.bytes = l->lay.total; op.host_buf = l->host_buf_of[a.expert];
            l->st.bytes_demand += op.bytes;
            di = (int)plan.demand.size();
            plan.demand.push_back(op);
        } else if (a.status == MOE_PREFETCH_HIT && pb.have < l->lay.total) {
            // the guess was right but only its head was requested: the rest is fetched now, like a demand load
            CopyOp op{a.expert, a.buf, pb.have, l->lay.total - pb.have, l->host_buf_of[a.expert]};
            l->st.bytes_spec += op.bytes;
            di = (int)plan.demand.size();
            plan.demand.push_back(op);
        }
        if (a.status != MOE_HIT) pb.have = l->lay.total;
        plan.demand_of.push_back(di);
        // swap mode (Sec. 3.3): the expert that came in vacates its host buffer, the evicted one goes back to the
        // host -- into the buffer that was spare, so that this write need not wait for the load's read; the
        // vacated buffer is the spare from now on.
        int wi = -1;
        if (l->swap && a.status != MOE_HIT) {
            if (a.victim < 0 || l->host_buf_of[a.expert] < 0) return fail(MOE_ESTATE, "swap bookkeeping out of step for expert %d", a.expert);
            CopyOp wb{a.victim, a.victim_buf, 0, l->lay.total, l->spare_host};
            l->host_buf_of[a.victim] = l->spare_host;
            l->spare_host = l->host_buf_of[a.expert];
            l->host_buf_of[a.expert] = -1;
            l->st.bytes_writeback += wb.bytes;
            wi = (int)plan.writeback.size();
            plan.writeback.push_back(wb);
        }
        plan.writeback_of.push_back(wi);
    }
    std::vector<int32_t> guess, issued;
    if (next && guess_score && next->cfg.prefetch_m > 0) {
        guess = top_m(guess_score, next->cfg.n_experts, next->cfg.prefetch_m);
        stage_guesses(next->cache, l->ctx->pool, next->st, guess, issued, plan.spec);
        for (CopyOp &op : plan.spec) {
            const uint64_t head = l->ctx->spec_head_bytes;
            op.offset = 0;
            op.bytes = head ? std::min<uint64_t>(head, next->lay.total) : next->lay.total;
            op.host_buf = next->host_buf_of[op.expert];
            l->ctx->bufs[op.buf].have = op.bytes;
            next->st.bytes_spec += op.bytes;
        }
    }
    if (tr) {
        tr->batch = batch; tr->top_k = cf.top_k; tr->n_experts = cf.n_experts;
        for (int i = 0; i < batch * cf.top_k; ++i) tr->expert_idx[i] = idx[i];
        tr->n_access = (int32_t)plan.access.size();
        for (size_t i = 0; i < plan.access.size(); ++i)
            tr->access[i] = {plan.access[i].expert, plan.access[i].status, plan.access[i].slot, plan.access[i].victim};
        tr->n_guess = (int32_t)guess.size();
        for (size_t i = 0; i < guess.size(); ++i) { tr->guess_expert[i] = guess[i]; tr->guess_issued[i] = issued[i]; }
        if (next && guess_score)
            for (int e = 0; e < next->cfg.n_experts; ++e) tr->guess_score[e] = guess_score[e];
    }
    return MOE_OK;
}

static int32_t issue_copy(moe_ctx *c, moe_layer *owner, const CopyOp &op)
{
    PoolBuf &b = c->bufs[op.buf];
    if (op.host_buf < 0) return fail(MOE_ESTATE, "expert %d has no host buffer to load from", op.expert);
    // swap mode: the target may still be draining an evicted expert, the source may still be receiving one
    if (b.draining) { HIPCHK(hipStreamWaitEvent(c->copy, b.drained, 0)); b.draining = false; }
    if (owner->host_writer[op.host_buf] >= 0) {
        HIPCHK(hipStreamWaitEvent(c->copy, c->bufs[owner->host_writer[op.host_buf]].drained, 0));
        owner->host_writer[op.host_buf] = -1;
    }
    int ps = -1;
    int32_t rc = MOE_OK;
    if (c->prof.on && c->prof.copy_seq++ % (uint64_t)c->prof.copy_stride == 0) rc = prof_begin(c, PROF_COPY, c->copy, op.bytes, &ps);
    if (rc) return rc;
    HIPCHK(hipMemcpyAsync(b.ptr + op.offset, owner->host_blobs + (uint64_t)op.host_buf * owner->lay.total + op.offset, op.bytes,
                          hipMemcpyHostToDevice, c->copy));
    rc = prof_end(c, PROF_COPY, c->copy, ps);
    if (rc) return rc;
    HIPCHK(hipEventRecord(b.ready, c->copy));
    b.pending = true;
    owner->host_reader[op.host_buf] = op.buf;
    return MOE_OK;
}

// Swap mode: the evicted expert leaves pool buffer op.buf for host buffer op.host_buf on the write-back stream.
// The caller has made sure that no kernel still reads the buffer (as for a copy that overwrites it).
static int32_t issue_writeback(moe_ctx *c, moe_layer *owner, const CopyOp &op)
{
    PoolBuf &b = c->bufs[op.buf];
    if (owner->host_reader[op.host_buf] >= 0) {      // the load that vacated the target must have read all of it
        HIPCHK(hipStreamWaitEvent(c->writeback, c->bufs[owner->host_reader[op.host_buf]].ready, 0));
        owner->host_reader[op.host_buf] = -1;
    }
    HIPCHK(hipStreamWaitEvent(c->writeback, b.ready, 0));   // the victim's own load (it may have come in earlier in this very step)
    int ps = -1;
    int32_t rc = MOE_OK;
    if (c->prof.on && c->prof.copy_seq++ % (uint64_t)c->prof.copy_stride == 0) rc = prof_begin(c, PROF_WRITEBACK, c->writeback, op.bytes, &ps);
    if (rc) return rc;
    HIPCHK(hipMemcpyAsync(owner->host_blobs + (uint64_t)op.host_buf * owner->lay.total, b.ptr, op.bytes, hipMemcpyDeviceToHost, c->writeback));
    rc = prof_end(c, PROF_WRITEBACK, c->writeback, ps);
    if (rc) return rc;
    HIPCHK(hipEventRecord(b.drained, c->writeback));
    b.draining = true;
    owner->host_writer[op.host_buf] = op.buf;
    return MOE_OK;
}

// The transfers one access asks for: its load (a miss, or the tail of a confirmed guess) and, in swap mode, the
// write-back of the expert it evicted.  The load goes first, so that it is not queued behind anything, unless
// it targets the very buffer the victim still sits in (no staging buffer was free): then the victim leaves first
// and the load waits for that.
static int32_t issue_access_transfers(moe_ctx *c, moe_layer *l, const StepPlan &plan, int i)
{
    const int di = plan.demand_of[i], wi = plan.writeback_of[i];
    const bool victim_first = di >= 0 && wi >= 0 && plan.demand[di].buf == plan.writeback[wi].buf;
    int32_t rc = MOE_OK;
    if (victim_first) rc = issue_writeback(c, l, plan.writeback[wi]);
    if (!rc && di >= 0) rc = issue_copy(c, l, plan.demand[di]);
    if (!rc && wi >= 0 && !victim_first) rc = issue_writeback(c, l, plan.writeback[wi]);
    return rc;
}

static int32_t check_step_args(const moe_layer *l, const moe_layer *next, int32_t batch)
{
    if (!l) return fail(MOE_EINVAL, "layer is null");
    if (batch < 1 || batch > l->ctx->cfg.max_batch) return fail(MOE_EINVAL, "batch %d outside 1..%d", batch, l->ctx->cfg.max_batch);
    if (next && next->ctx != l->ctx) return fail(MOE_EINVAL, "next layer belongs to another context");
    if (next && next->cfg.hidden != l->cfg.hidden) return fail(MOE_EINVAL, "next layer has another hidden size");
    return MOE_OK;
}

extern "C" int32_t moe_layer_resolve(moe_layer_t *l, moe_layer_t *next, const int32_t *expert_idx, int32_t batch,
                                     const double *guess_score, moe_step_trace_t *trace)
try {
    int32_t rc = check_step_args(l, next, batch);
    if (rc) return rc;
    if (!expert_idx) return fail(MOE_EINVAL, "moe_layer_resolve: expert_idx is null");
    if (!l->ctx->host_only && !all_loaded(l)) return fail(MOE_ESTATE, "moe_layer_resolve: not every expert of the layer is loaded");
    rc = fold_pending(l->ctx);
    if (rc) return rc;
    StepPlan plan;
    rc = plan_step(l, next, expert_idx, batch, guess_score, trace, plan);
    if (rc) return rc;
    l->stepped = true;
    if (next) next->stepped = true;
    if (!l->ctx->host_only) {
        for (int i = 0; i < (int)plan.access.size(); ++i) { rc = issue_access_transfers(l->ctx, l, plan, i); if (rc) return rc; }
        for (const CopyOp &op : plan.spec) { rc = issue_copy(l->ctx, next, op); if (rc) return rc; }
    }
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_resolve");
}

// ---------------------------------------------------------------------------------------------
// the GPU step
// ---------------------------------------------------------------------------------------------

// Wait until every block of the gate kernel has published the launch's sequence number next to its results.
static int32_t wait_gate(moe_ctx *c, int32_t batch, uint32_t seq)
{
    volatile uint32_t *flag = c->gate_out->done;
    if (c->sync_wait) {
        HIPCHK(hipStreamSynchronize(c->compute));
    } else {
        int b = 0;
        for (uint64_t spin = 0; b < batch; ++spin) {
            while (b < batch && flag[b] == seq) ++b;
            if (b == batch) break;
            if (spin > 4096 && (spin & 255) == 0) {
                hipError_t q = hipEventQuery(c->ev_gate);
                if (q == hipSuccess) break;            // kernel over: the flags are re-read below
                if (q != hipErrorNotReady) { g_hip_err = (int32_t)q; return fail(MOE_EHIP, "gate kernel failed: %s", hipGetErrorString(q)); }
            }
            __builtin_ia32_pause();
        }
    }
    std::atomic_thread_fence(std::memory_order_acquire);
    for (int b = 0; b < batch; ++b)
        if (flag[b] != seq) return fail(MOE_ESTATE, "gate kernel finished but token %d published no result", b);
    return MOE_OK;
}

// Launch a kernel; while profiling is on, attach a start/stop event pair to the dispatch itself
// (hipExtLaunchKernelGGL), so the pair brackets the kernel's execution and nothing else.
template <typename K, typename... Args>
static int32_t launch_timed(moe_ctx *c, int kind, uint64_t bytes, K kernel, dim3 grid, dim3 block, size_t shm,
                            Args... args)
{
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->prof.on) {
        ProfKind &p = c->prof.kind[kind];
        if (p.used == Profiler::RING) { int32_t rc = prof_drain(c, kind); if (rc) return rc; }
        if (p.used == p.start.size()) {
            hipEvent_t a, b;
            HIPCHK(hipEventCreate(&a));
            HIPCHK(hipEventCreate(&b));
            p.start.push_back(a);
            p.stop.push_back(b);
        }
        e0 = p.start[p.used];
        e1 = p.stop[p.used];
        p.used++;
        p.launches++;
        p.bytes += bytes;
    }
    hipExtLaunchKernelGGL(kernel, grid, block, shm, c->compute, e0, e1, 0, args...);
    HIPCHK(hipGetLastError());
    return MOE_OK;
}

static int32_t launch_gate(moe_ctx *c, GateArgs ga, int32_t batch)
{
    if (++c->gate_seq == 0) ++c->gate_seq;             // 0 is what a fresh context holds
    ga.seq = c->gate_seq;
    int32_t rc = ga.wg2 ? launch_timed(c, PROF_GATE, 0, k_gate<true>, dim3(batch), dim3(GATE_THREADS), 0, ga)
                        : launch_timed(c, PROF_GATE, 0, k_gate<false>, dim3(batch), dim3(GATE_THREADS), 0, ga);
    if (rc) return rc;
    if (!c->sync_wait) HIPCHK(hipEventRecord(c->ev_gate, c->compute));
    return wait_gate(c, batch, ga.seq);
}

// Rows each wave keeps in flight (ring depth) in the w1/w3 and the w2 kernel.
#ifndef MOE_W13_G
#define MOE_W13_G 2
#endif
#ifndef MOE_W2_G
#define MOE_W2_G 4
#endif
#ifndef MOE_FUSED_G2
#define MOE_FUSED_G2 8
#endif
#ifndef MOE_W2T_G
#define MOE_W2T_G 4
#endif

// Format policy of a layer's blobs: the bit width, or bits * 10 + 8 with two-level metadata (48, 38, 28).
static int fmt_of(const BlobLayout &b) { return b.scale_group ? b.bits * 10 + 8 : b.bits; }

// Activation registers per (chunk, token) of each format: the budget that limits tokens per entry.
constexpr int act_regs_of(int fmt) { return (fmt == 3 || fmt == 38) ? 34 : (fmt == 2 ? 20 : (fmt == 28 ? 40 : 18)); }
template <int BITS> constexpr int act_regs() { return act_regs_of(BITS); }
constexpr int codes_per_chunk(int fmt) { return (fmt == 3 || fmt == 38 || fmt == 28) ? 64 : 32; }
constexpr int ACT_REG_BUDGET = 160;

static int chunks_per_lane(int cols, int fmt)       // 64-lane passes over one row (1, 2 or 4; 0 = too wide)
{
    const int n = (cols / codes_per_chunk(fmt) + 63) / 64;
    return n <= 1 ? 1 : (n <= 2 ? 2 : (n <= 4 ? 4 : 0));
}

static int max_tokens_per_entry(int hidden, int fmt)
{
    const int kch = std::max(1, chunks_per_lane(hidden, fmt));
    const int n = ACT_REG_BUDGET / (kch * act_regs_of(fmt));
    return n >= 4 ? 4 : (n >= 2 ? 2 : 1);
}

// Waves per block of the w1/w3 kernel.  8 (two per SIMD, measured best for the single-token kernels) while the
// activations leave room under the 256 registers a lane may then use; 4 (512 registers) for the variants that
// keep more activations, which would otherwise spill.
#ifndef MOE_W13_WAVES
#define MOE_W13_WAVES 8
#endif
template <int BITS, int KCH, int NT> constexpr int w13_waves() { return KCH * NT * act_regs<BITS>() <= 80 ? MOE_W13_WAVES : 4; }

template <int BITS, int KCH, int NT>
static int32_t launch_w13_t(moe_ctx *c, uint64_t bytes, int n_entries, const FfnArgs &A)
{
    if constexpr (KCH * NT * act_regs<BITS>() <= ACT_REG_BUDGET) {
        constexpr int WAVES = w13_waves<BITS, KCH, NT>();
        const dim3 grid(std::max(1, std::min((A.F + WAVES - 1) / WAVES, c->w13_blocks / n_entries)), n_entries);
        return launch_timed(c, PROF_W13, bytes, k_w13<BITS, KCH, NT, MOE_W13_G, WAVES>, grid, dim3(WAVES * WAVE), 0, A);
    } else {
        return fail(MOE_EINVAL, "no w1/w3 kernel for %d chunks per lane and %d tokens per entry", KCH, NT);
    }
}

template <int BITS, int KCH>
static int32_t launch_w13_k(moe_ctx *c, int nt, uint64_t bytes, int n_entries, const FfnArgs &A)
{
    if (nt == 1) return launch_w13_t<BITS, KCH, 1>(c, bytes, n_entries, A);
    if (nt == 2) return launch_w13_t<BITS, KCH, 2>(c, bytes, n_entries, A);
    return launch_w13_t<BITS, KCH, 4>(c, bytes, n_entries, A);
}

// table (device-side routing): the layer's expert -> device buffer map; entry j then serves the j-th selected expert
template <int BITS>
static int32_t launch_ffn_fmt(moe_layer *l, const std::vector<FfnEntry> &entries, int nt, bool w13_only, const uint8_t *const *table)
{
    moe_ctx *c = l->ctx;
    const BlobLayout &b = l->lay;
    const int kch = chunks_per_lane(b.hidden, BITS);                          // per w1/w3 row
    const int cs = (b.ffn / Fmt<BITS>::CODES + 63) / 64;                      // waves per block for w2
    if (kch == 0 || cs > 8) return fail(MOE_EINVAL, "shape too large for the GEMV kernels");
    for (size_t first = 0; first < entries.size(); first += MAX_ENTRIES) {
        const int n = (int)std::min<size_t>(MAX_ENTRIES, entries.size() - first);
        FfnArgs A{};
        for (int i = 0; i < n; ++i) A.e[i] = entries[first + i];
        A.h = c->h_buf; A.a = c->a_buf; A.ypart = c->ypart; A.ytab = c->ytab;
        A.H = b.hidden; A.F = b.ffn; A.group = b.group; A.scale_group = b.scale_group;
        A.stride13 = b.m13.row_stride; A.meta13 = b.m13.meta_off;
        A.stride2 = b.m2.row_stride; A.meta2 = b.m2.meta_off;
        A.off_w2 = b.off_w2;
        A.rows_per_block = c->w2_rows;
        if (table) {
            A.route_idx = c->route_idx;
            for (int e = 0; e < 16; ++e) A.table[e] = table[e];
        }
        // algorithmic bytes: every distinct expert of the launch is read once
        uint64_t n_distinct = 0;
        for (int i = 0; i < n; ++i) {
            bool seen = false;
            for (int j = 0; j < i && !table; ++j) seen |= (A.e[j].blob == A.e[i].blob);
            n_distinct += !seen;
        }
        const uint64_t bytes13 = n_distinct * 2 * (uint64_t)b.ffn * b.m13.row_stride;
        const uint64_t bytes2 = n_distinct * (uint64_t)b.hidden * b.m2.row_stride;
        int32_t rc;
        if (kch == 1) rc = launch_w13_k<BITS, 1>(c, nt, bytes13, n, A);
        else if (kch == 2) rc = launch_w13_k<BITS, 2>(c, nt, bytes13, n, A);
        else rc = launch_w13_k<BITS, 4>(c, nt, bytes13, n, A);
        if (rc) return rc;
        if (w13_only) continue;
        const dim3 g2((b.hidden + A.rows_per_block - 1) / A.rows_per_block, n), blk(cs * WAVE);
        const size_t shm = (size_t)A.rows_per_block * nt * cs * sizeof(float);
        if (nt == 1) rc = launch_timed(c, PROF_W2, bytes2, k_w2<BITS, 1, MOE_W2_G>, g2, blk, shm, A);
        else if (nt == 2) rc = launch_timed(c, PROF_W2, bytes2, k_w2<BITS, 2, MOE_W2_G>, g2, blk, shm, A);
        else rc = launch_timed(c, PROF_W2, bytes2, k_w2<BITS, 4, MOE_W2_G>, g2, blk, shm, A);
        if (rc) return rc;
    }
    return MOE_OK;
}

// Ring depths of the expert-after-expert one-launch kernel.
#ifndef MOE_SEQ_G1
#define MOE_SEQ_G1 2
#endif
#ifndef MOE_SEQ_G2
#define MOE_SEQ_G2 4
#endif

// The expert-after-expert one-launch kernel for a single token; *done = false when the shape does not fit it.
template <int BITS>
static int32_t launch_seq_fmt(moe_layer *l, const FusedArgs &A0, bool probe_only, bool *done)
{
    moe_ctx *c = l->ctx;
    const BlobLayout &b = l->lay;
    const int kch = chunks_per_lane(b.hidden, BITS);
    const int cs = (b.ffn / Fmt<BITS>::CODES + 63) / 64;
    const int grid = c->n_cu;
    *done = false;
    if (grid < 1 || grid > SEQ_FLAG_STRIDE) return MOE_OK;
    const int rpw = (b.ffn + grid * SEQ_WAVES - 1) / (grid * SEQ_WAVES);
    const int rows = ((b.hidden + grid - 1) / grid + MOE_SEQ_G2 - 1) / MOE_SEQ_G2 * MOE_SEQ_G2;
    constexpr bool has_kernel = BITS == 4 || BITS == 48 || BITS == 2 || BITS == 3;
    if (!has_kernel || kch == 0 || kch > 2 || (codes_per_chunk(BITS) == 64 && kch > 1) || cs > SEQ_WAVES || rpw > SEQ_MAX_ROWS || rows > 64 ||
        A0.n_exp < 1 || A0.n_exp > 2)
        return MOE_OK;
    *done = true;
    if (probe_only) return MOE_OK;
    if constexpr (has_kernel) {
        FusedArgs A = A0;
        A.rows_per_block = rows;
        A.barrier = c->seq_flags;
        A.barrier_target = ++c->barrier_count;
        A.error_flag = &c->gate_out_dev->ffn_error;
        const uint64_t bytes = (uint64_t)A.n_exp * (2 * (uint64_t)b.ffn * b.m13.row_stride + (uint64_t)b.hidden * b.m2.row_stride);
        const dim3 g(grid), blk(SEQ_WAVES * WAVE);
        if (kch == 1) return launch_timed(c, PROF_FFN, bytes, k_ffn_seq<BITS, 1, MOE_SEQ_G1, MOE_SEQ_G2>, g, blk, 0, A);
        if constexpr (BITS != 3) return launch_timed(c, PROF_FFN, bytes, k_ffn_seq<BITS, 2, MOE_SEQ_G1, MOE_SEQ_G2>, g, blk, 0, A);
    }
    return fail(MOE_EINVAL, "no one-launch kernel for this shape");
}

static int32_t launch_seq(moe_layer *l, const FusedArgs &A, bool probe_only, bool *done)
{
    switch (fmt_of(l->lay)) {
    case 4: return launch_seq_fmt<4>(l, A, probe_only, done);
    case 3: return launch_seq_fmt<3>(l, A, probe_only, done);
    case 2: return launch_seq_fmt<2>(l, A, probe_only, done);
    case 48: return launch_seq_fmt<48>(l, A, probe_only, done);
    default: *done = false; return MOE_OK;
    }
}

// The one-launch path for a single token; returns MOE_OK with *done = false when the shape does not fit it.
template <int BITS>
static int32_t launch_token_fmt(moe_layer *l, const FusedArgs &A0, bool one_launch, bool probe_only, bool *done)
{
    moe_ctx *c = l->ctx;
    const BlobLayout &b = l->lay;
    const int kch = chunks_per_lane(b.hidden, BITS);
    const int cs = (b.ffn / Fmt<BITS>::CODES + 63) / 64;
    const int grid = c->n_cu;
    const int rows = (one_launch || c->w2_token_rows <= 0) ? (b.hidden + grid - 1) / grid : c->w2_token_rows;
    *done = false;
    const int items_per_wave = (A0.n_exp * b.ffn + grid * FUSED_WAVES - 1) / (grid * FUSED_WAVES);
    constexpr bool has_one_launch = BITS != 38 && BITS != 28;      // no persistent one-launch kernel for these
    if (kch == 0 || kch > 2 || (codes_per_chunk(BITS) == 64 && kch > 1) || cs > 8 || cs * A0.n_exp > FUSED_WAVES || rows > 64 ||
        grid < 1 || grid > 1024 || items_per_wave + 2 > FUSED_MAX_ITEMS || (one_launch && !has_one_launch))
        return MOE_OK;
    *done = true;
    if (probe_only) return MOE_OK;
    FusedArgs A = A0;
    A.rows_per_block = rows;
    if (!one_launch) {
        const uint64_t bytes2 = (uint64_t)A.n_exp * b.hidden * b.m2.row_stride;
        // w2 half only (k_w13 ran before): blocks of n_exp * CS waves, no barrier
        return launch_timed(c, PROF_W2, bytes2, k_w2_token<BITS, MOE_W2T_G>, dim3((b.hidden + rows - 1) / rows),
                            dim3(A.n_exp * cs * WAVE), 0, A);
    }
    if constexpr (has_one_launch) {
        A.barrier = c->barrier;
        A.barrier_target = ++c->barrier_count;
        A.error_flag = &c->gate_out_dev->ffn_error;
        const uint64_t bytes = (uint64_t)A.n_exp * (2 * (uint64_t)b.ffn * b.m13.row_stride + (uint64_t)b.hidden * b.m2.row_stride);
        const dim3 g(grid), blk(FUSED_WAVES * WAVE);
        if (kch == 1) return launch_timed(c, PROF_FFN, bytes, k_ffn_token<BITS, 1, 2, MOE_FUSED_G2>, g, blk, 0, A);
        if constexpr (BITS != 3) return launch_timed(c, PROF_FFN, bytes, k_ffn_token<BITS, 2, 2, MOE_FUSED_G2>, g, blk, 0, A);
    }
    return fail(MOE_EINVAL, "no fused kernel for this shape");
}

static int32_t launch_token(moe_layer *l, const FusedArgs &A, bool one_launch, bool probe_only, bool *done)
{
    switch (fmt_of(l->lay)) {
    case 4: return launch_token_fmt<4>(l, A, one_launch, probe_only, done);
    case 3: return launch_token_fmt<3>(l, A, one_launch, probe_only, done);
    case 2: return launch_token_fmt<2>(l, A, one_launch, probe_only, done);
    case 48: return launch_token_fmt<48>(l, A, one_launch, probe_only, done);
    case 38: return launch_token_fmt<38>(l, A, one_launch, probe_only, done);
    case 28: return launch_token_fmt<28>(l, A, one_launch, probe_only, done);
    default: *done = false; return MOE_OK;
    }
}

// Matrix-core path for one pass: every expert of the pass with all its tokens, two launches (w1/w3, w2)
// plus the group-sum tables of their activation operands.
struct PassExpert { const uint8_t *blob; std::vector<int> pairs; };

// Streaming matrix-core form: persistent blocks over (entry, 128-row block, K part) items.
// An expert with more than 32 tokens becomes two entries (token tiles) that read the same weights.
static int32_t launch_mfma_stream(moe_layer *l, const std::vector<PassExpert> &experts, const float *w, int batch)
{
    moe_ctx *c = l->ctx;
    const BlobLayout &b = l->lay;
    const int K = l->cfg.top_k;
    static bool lds_attr_set = false;      // staging buffers above the default dynamic LDS limit
    if (!lds_attr_set) {
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream_q4<true, false>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream_q4<false, false>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream_q4<true, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream_q4<false, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream_q4<true, false, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream_q4<false, false, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<true, 1, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<true, 2, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<false, 1, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<false, 2, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<true, 1, 8>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<false, 1, 8>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<true, 1, 8, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<false, 1, 8, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<true, 2, 4, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<true, 1, 8, true, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<false, 1, 8, true, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<true, 2, 4, true, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<false, 2, 4, true, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_stream16_q4<false, 2, 4, true>), hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS_BYTES));
        lds_attr_set = true;
    }
    const int n_cu = c->n_cu > 0 ? c->n_cu : 256;
    // The kernels address tokens and pairs with one byte, so a large batch (a prompt, Sec. 3) goes through in
    // windows of 256 / top_k tokens: each window is a launch pair of its own over the same resident experts, with the
    // activation, scratch and accumulator pointers moved to the window's first token.
    const int window = MF_MAX_PAIRS / K;
    for (int w0 = 0; w0 < batch; w0 += window) {
        const int w1 = std::min(batch, w0 + window);
        TileArgs A{};
        int n = 0, first = 0, n_distinct = 0;
        for (const PassExpert &pe : experts) {
            std::vector<int> mine;
            for (int q : pe.pairs)
                if (q / K >= w0 && q / K < w1) mine.push_back(q);
            if (mine.empty()) continue;
            ++n_distinct;
            for (size_t t0 = 0; t0 < mine.size(); t0 += 32) {
                if (n >= 32) return fail(MOE_EINVAL, "more than 32 (expert, token tile) entries in one launch");
                const size_t t1 = std::min(mine.size(), t0 + 32);
                A.e[n].blob = pe.blob;
                A.e[n].n_tok = (int32_t)(t1 - t0);
                A.e[n].first = first;
                for (size_t i = t0; i < t1; ++i) {
                    const int q = mine[i];
                    A.tok[first] = (uint8_t)(q / K - w0);
                    A.pair[first] = (uint8_t)(q - w0 * K);
                    A.w[first] = w[q];
                    ++first;
                }
                ++n;
            }
        }
        if (n == 0) continue;
        auto shape = [&](int rows, int Kdim, bool may_split) {
            const int n_seg = (Kdim / 64 + TL_SG - 1) / TL_SG;
            A.row_blocks = (rows + TL_ROWS - 1) / TL_ROWS;
            int parts = 1;
            if (may_split) {
                // the step fixed the number of parts per window from its routing alone; the rows for the parts'
                // partial sums were budgeted there, the check below only guards the buffer
                parts = std::min(n_seg, std::max<int>(1, c->w2_parts.at(w0 / window)));
                const uint64_t left = (c->ypart_extra_floats - c->ypart_extra_used) / ((uint64_t)first * b.hidden);
                if (parts > 1 && (uint64_t)parts > left) parts = 1;
            }
            A.seg_per_part = (n_seg + parts - 1) / parts;
            A.k_parts = (n_seg + A.seg_per_part - 1) / A.seg_per_part;       // no empty part
            A.n_items = n * A.row_blocks * A.k_parts;
            return dim3(std::min(A.n_items, TL_BLOCKS_PER_CU * n_cu));
        };
        // algorithmic bytes: every distinct expert of the launch once (a second token tile reads it again)
        const uint64_t bytes13 = (uint64_t)n_distinct * 2 * b.ffn * b.m13.row_stride, bytes2 = (uint64_t)n_distinct * b.hidden * b.m2.row_stride;
        uint16_t *a_win = c->a_buf + (size_t)w0 * K * b.ffn;
        A.a = a_win;
        A.ypart = c->ypart + (size_t)w0 * K * b.hidden; A.ytab = c->ytab + (size_t)w0 * K; A.row_bias = w0 * K;
        A.act = c->h_buf + (size_t)w0 * b.hidden;
        const bool meta8 = b.scale_group > 0;
        const bool r1 = (c->mfma_form == 3 || c->mfma_form == 0) && !meta8 && !l->wide_meta.load(std::memory_order_relaxed);
        // Which kernels multiply a window (one or two token tiles of 16) is decided from the window's routing, never from
        // the experts that happen to share a launch: they add in different orders, and a token's result must not depend
        // on what the cache held.
        const bool small = c->win_small.at(w0 / window) != 0;
        // (the 16-token kernels address a matrix with 32-bit offsets)
        const bool fits32 = 2ull * b.ffn * b.m13.row_stride < (1ull << 31) && (uint64_t)b.hidden * b.m2.row_stride < (1ull << 31);
        const bool t16 = (c->mfma_form == 4 || c->mfma_form == 5 || c->mfma_form == 0) && !meta8 && fits32;
        const bool gs = c->mfma_form == 5 || c->mfma_form == 0;         // group-scaled arithmetic: any finite (scale, zero) pair
        const bool w8 = c->mfma16_waves == 8;
        const bool gs8 = meta8 && gs && fits32;                         // two-level metadata: the group-scaled kernels decode it in fp32
        const int max_tok = small ? 16 : 32;
        auto run_shift = [&](const MatLayout &m) { return (m.run_len == 0 || m.run_len >= m.cols / (uint32_t)b.group) ? 31 : __builtin_ctz(m.run_len); };
        A.K = b.hidden; A.N = b.ffn; A.stride = b.m13.row_stride; A.meta_off = b.m13.meta_off; A.mat_off = b.off_w13;
        A.meta2_off = b.m13.meta2_off; A.run_shift = run_shift(b.m13);
        const dim3 g13 = shape(2 * b.ffn, b.hidden, false);
        int32_t rc = gs8 ? (max_tok <= 16 ? launch_timed(c, PROF_W13, bytes13, k_mfma_stream16_q4<true, 1, 8, true, true>, g13, dim3(512), TL_LDS_BYTES, A)
                                          : launch_timed(c, PROF_W13, bytes13, k_mfma_stream16_q4<true, 2, 4, true, true>, g13, dim3(TL_THREADS), TL_LDS_BYTES, A))
                   : t16 && gs ? (max_tok <= 16 ? launch_timed(c, PROF_W13, bytes13, k_mfma_stream16_q4<true, 1, 8, true>, g13, dim3(512), TL_LDS_BYTES, A)
                                                : launch_timed(c, PROF_W13, bytes13, k_mfma_stream16_q4<true, 2, 4, true>, g13, dim3(TL_THREADS), TL_LDS_BYTES, A))
                   : t16 ? (max_tok <= 16 ? (w8 ? launch_timed(c, PROF_W13, bytes13, k_mfma_stream16_q4<true, 1, 8>, g13, dim3(512), TL_LDS_BYTES, A)
                                                : launch_timed(c, PROF_W13, bytes13, k_mfma_stream16_q4<true, 1, 4>, g13, dim3(TL_THREADS), TL_LDS_BYTES, A))
                                          : launch_timed(c, PROF_W13, bytes13, k_mfma_stream16_q4<true, 2, 4>, g13, dim3(TL_THREADS), TL_LDS_BYTES, A))
                     : meta8 ? launch_timed(c, PROF_W13, bytes13, k_mfma_stream_q4<true, true>, g13, dim3(TL_THREADS), TL_LDS_BYTES, A)
                     : r1  ? launch_timed(c, PROF_W13, bytes13, k_mfma_stream_q4<true, false, true>, g13, dim3(TL_THREADS), TL_LDS_BYTES, A)
                           : launch_timed(c, PROF_W13, bytes13, k_mfma_stream_q4<true, false>, g13, dim3(TL_THREADS), TL_LDS_BYTES, A);
        if (rc) return rc;
        A.act = a_win;
        A.K = b.ffn; A.N = b.hidden; A.stride = b.m2.row_stride; A.meta_off = b.m2.meta_off; A.mat_off = b.off_w2;
        A.meta2_off = b.m2.meta2_off; A.run_shift = run_shift(b.m2);
        const dim3 g2 = shape(b.hidden, b.ffn, true);
        if (A.k_parts > 1) {        // rows behind the pairs' own, counted from the window's first pair
            A.part_base = (int32_t)((uint64_t)batch * K + c->ypart_extra_used / b.hidden) - w0 * K;
            c->ypart_extra_used += (uint64_t)first * A.k_parts * b.hidden;
        }
        rc = gs8 ? (max_tok <= 16 ? launch_timed(c, PROF_W2, bytes2, k_mfma_stream16_q4<false, 1, 8, true, true>, g2, dim3(512), TL_LDS_BYTES, A)
                                  : launch_timed(c, PROF_W2, bytes2, k_mfma_stream16_q4<false, 2, 4, true, true>, g2, dim3(TL_THREADS), TL_LDS_BYTES, A))
           : t16 && gs ? (max_tok <= 16 ? launch_timed(c, PROF_W2, bytes2, k_mfma_stream16_q4<false, 1, 8, true>, g2, dim3(512), TL_LDS_BYTES, A)
                                        : launch_timed(c, PROF_W2, bytes2, k_mfma_stream16_q4<false, 2, 4, true>, g2, dim3(TL_THREADS), TL_LDS_BYTES, A))
           : t16 ? (max_tok <= 16 ? (w8 ? launch_timed(c, PROF_W2, bytes2, k_mfma_stream16_q4<false, 1, 8>, g2, dim3(512), TL_LDS_BYTES, A)
                                        : launch_timed(c, PROF_W2, bytes2, k_mfma_stream16_q4<false, 1, 4>, g2, dim3(TL_THREADS), TL_LDS_BYTES, A))
                                  : launch_timed(c, PROF_W2, bytes2, k_mfma_stream16_q4<false, 2, 4>, g2, dim3(TL_THREADS), TL_LDS_BYTES, A))
             : meta8 ? launch_timed(c, PROF_W2, bytes2, k_mfma_stream_q4<false, true>, g2, dim3(TL_THREADS), TL_LDS_BYTES, A)
             : r1  ? launch_timed(c, PROF_W2, bytes2, k_mfma_stream_q4<false, false, true>, g2, dim3(TL_THREADS), TL_LDS_BYTES, A)
                   : launch_timed(c, PROF_W2, bytes2, k_mfma_stream_q4<false, false>, g2, dim3(TL_THREADS), TL_LDS_BYTES, A);
        if (rc) return rc;
    }
    return MOE_OK;
}

static int32_t launch_mfma(moe_layer *l, const std::vector<PassExpert> &experts, const float *w, int batch)
{
    moe_ctx *c = l->ctx;
    const BlobLayout &b = l->lay;
    const int K = l->cfg.top_k;
    // the row-staging form takes up to 64 tokens per expert, indexes pairs with one byte and reads fp16 pairs only
    if (c->mfma_form != 1 || batch > 64 || batch * K > MF_MAX_PAIRS || b.scale_group > 0) return launch_mfma_stream(l, experts, w, batch);
    MfmaArgs A{};
    int n = 0, first = 0, max_tok = 0;
    for (const PassExpert &pe : experts) {
        A.e[n].blob = pe.blob;
        A.e[n].n_tok = (int32_t)pe.pairs.size();
        A.e[n].first = first;
        for (int q : pe.pairs) {
            A.tok[first] = (uint8_t)(q / K);
            A.pair[first] = (uint8_t)q;
            A.w[first] = w[q];
            ++first;
        }
        max_tok = std::max(max_tok, (int)pe.pairs.size());
        ++n;
    }
    const uint64_t bytes13 = (uint64_t)n * 2 * b.ffn * b.m13.row_stride, bytes2 = (uint64_t)n * b.hidden * b.m2.row_stride;
    A.act = c->h_buf; A.a = c->a_buf; A.ypart = c->ypart; A.ytab = c->ytab;
    A.K = b.hidden; A.N = b.ffn; A.stride = b.m13.row_stride; A.meta_off = b.m13.meta_off; A.mat_off = b.off_w13;
    // LDS: 32 staged rows (codes + pairs) or the final reduction buffer
    auto rows_lds = [&](int Kdim, int mt) {
        const int sg = std::min(Kdim / 64, MF2_SEG);
        return std::max<size_t>((size_t)32 * (sg * 32 + 16) + (size_t)32 * ((sg + 3) & ~3) * 4, (size_t)MF2_WAVES * mt * 16 * 64 * 4);
    };
    static bool lds_attr_set = false;  // these kernels stage 72 KB: above the default dynamic LDS limit
    if (!lds_attr_set) {
        const int lim = 96 * 1024;
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_rows_q4<true, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, lim));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_rows_q4<true, 2>), hipFuncAttributeMaxDynamicSharedMemorySize, lim));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_rows_q4<false, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, lim));
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mfma_rows_q4<false, 2>), hipFuncAttributeMaxDynamicSharedMemorySize, lim));
        lds_attr_set = true;
    }
    const int mt = max_tok > 32 ? 2 : 1;
    const dim3 blkr(MF2_WAVES * WAVE), gr13((2 * b.ffn + 31) / 32, n), gr2((b.hidden + 31) / 32, n);
    int32_t rr = mt == 2 ? launch_timed(c, PROF_W13, bytes13, k_mfma_rows_q4<true, 2>, gr13, blkr, rows_lds(b.hidden, 2), A)
                         : launch_timed(c, PROF_W13, bytes13, k_mfma_rows_q4<true, 1>, gr13, blkr, rows_lds(b.hidden, 1), A);
    if (rr) return rr;
    A.act = c->a_buf;
    A.K = b.ffn; A.N = b.hidden; A.stride = b.m2.row_stride; A.meta_off = b.m2.meta_off; A.mat_off = b.off_w2;
    return mt == 2 ? launch_timed(c, PROF_W2, bytes2, k_mfma_rows_q4<false, 2>, gr2, blkr, rows_lds(b.ffn, 2), A)
                   : launch_timed(c, PROF_W2, bytes2, k_mfma_rows_q4<false, 1>, gr2, blkr, rows_lds(b.ffn, 1), A);
}

static int32_t launch_ffn(moe_layer *l, const std::vector<FfnEntry> &entries, int nt, bool w13_only = false,
                          const uint8_t *const *table = nullptr)
{
    switch (fmt_of(l->lay)) {
    case 4: return launch_ffn_fmt<4>(l, entries, nt, w13_only, table);
    case 3: return launch_ffn_fmt<3>(l, entries, nt, w13_only, table);
    case 2: return launch_ffn_fmt<2>(l, entries, nt, w13_only, table);
    case 48: return launch_ffn_fmt<48>(l, entries, nt, w13_only, table);
    case 38: return launch_ffn_fmt<38>(l, entries, nt, w13_only, table);
    case 28: return launch_ffn_fmt<28>(l, entries, nt, w13_only, table);
    default: return fail(MOE_EINVAL, "unsupported bit width %d", l->lay.bits);
    }
}

// ---------------------------------------------------------------------------------------------
// device-side routing
// ---------------------------------------------------------------------------------------------

// Catch up the bookkeeping of the steps that were enqueued without waiting for their gate: wait for them, then
// replay their selections, oldest first, through the same cache logic a waiting step runs.
static int32_t fold_pending(moe_ctx *c)
{
    if (c->pending.empty()) return MOE_OK;
    HIPCHK(hipStreamSynchronize(c->compute));
    {   // the pending slots are consecutive in the ring (oldest first), possibly wrapping once
        const size_t entry = MOE_MAX_TOPK * sizeof(int32_t);
        const uint32_t first = c->pending.front().slot, n = (uint32_t)c->pending.size();
        const uint32_t head = std::min(n, moe_ctx::ROUTE_LOG - first);
        HIPCHK(hipMemcpy(c->route_log + (size_t)first * MOE_MAX_TOPK, c->route_log_dev + (size_t)first * MOE_MAX_TOPK, head * entry, hipMemcpyDeviceToHost));
        if (n > head) HIPCHK(hipMemcpy(c->route_log, c->route_log_dev, (n - head) * entry, hipMemcpyDeviceToHost));
    }
    std::vector<AccessRec> access;
    std::vector<CopyOp> misses;
    std::vector<int32_t> needed;
    for (const moe_ctx::PendingStep &p : c->pending) {
        moe_layer *l = p.layer;
        const int32_t *idx = c->route_log + (size_t)p.slot * MOE_MAX_TOPK;
        needed.assign(idx, idx + l->cfg.top_k);
        std::sort(needed.begin(), needed.end());
        needed.erase(std::unique(needed.begin(), needed.end()), needed.end());
        if (needed.front() < 0 || needed.back() >= l->cfg.n_experts) { c->pending.clear(); return fail(MOE_ESTATE, "device-routed step logged expert %d", needed.front() < 0 ? needed.front() : needed.back()); }
        access.clear();
        misses.clear();
        resolve_accesses(l->cache, c->pool, l->st, needed, false, access, misses);
        if (!misses.empty()) { c->pending.clear(); return fail(MOE_ESTATE, "device-routed step met an expert that is not resident"); }
    }
    c->pending.clear();
    return MOE_OK;
}

static bool all_resident(const moe_layer *l)
{
    if (l->swap || (l->cfg.flags & MOE_LAYER_NO_CACHE) || l->cfg.cache_slots != l->cfg.n_experts || !l->cache.staged.empty()) return false;
    for (int s = 0; s < l->cache.k; ++s)
        if (l->cache.slot_expert[s] < 0 || l->ctx->bufs[l->cache.slot_buf[s]].pending) return false;
    return true;
}

static FusedArgs token_args(moe_layer *l, const uint16_t *x_in, uint16_t *x_out)
{
    moe_ctx *c = l->ctx;
    FusedArgs fa{};
    fa.h = c->h_buf; fa.x = x_in; fa.x_out = x_out; fa.a = c->a_buf; fa.y = c->yacc;
    fa.H = l->lay.hidden; fa.F = l->lay.ffn; fa.group = l->lay.group; fa.scale_group = l->lay.scale_group;
    fa.stride13 = l->lay.m13.row_stride; fa.meta13 = l->lay.m13.meta_off;
    fa.stride2 = l->lay.m2.row_stride; fa.meta2 = l->lay.m2.meta_off; fa.off_w2 = l->lay.off_w2;
    return fa;
}

// One token through a layer whose experts are all on the device: no cache decision depends on the routing, so the
// gate, w1/w3 and w2 kernels are enqueued back to back and the call returns without waiting for any of them.
static bool device_routed_step_fits(moe_layer *l, const moe_layer *next, int32_t batch, const moe_step_trace_t *trace, bool spec)
{
    moe_ctx *c = l->ctx;
    if (!c->device_routing || batch != 1 || trace || !c->token_path || c->fused || l->cfg.top_k > 2 || c->gate_out->ffn_error) return false;
    if (!all_resident(l) || (spec && !all_resident(next))) return false;
    FusedArgs fa = token_args(l, nullptr, nullptr);
    fa.n_exp = l->cfg.top_k;
    bool fits = false;
    return launch_token(l, fa, false, true, &fits) == MOE_OK && fits;
}

static int32_t device_routed_step(moe_layer *l, const uint16_t *x_in, uint16_t *x_out, uint16_t *h_out)
{
    moe_ctx *c = l->ctx;
    const moe_layer_config_t &cf = l->cfg;
    if (c->pending.size() >= moe_ctx::ROUTE_LOG) { int32_t rc = fold_pending(c); if (rc) return rc; }
    // a log slot is free once its step has been folded: with fewer than ROUTE_LOG steps pending the oldest slots are
    uint32_t slot = c->pending.empty() ? 0 : (c->pending.back().slot + 1) % moe_ctx::ROUTE_LOG;
    GateArgs ga{};
    ga.x = x_in; ga.wg = l->gate_w_dev; ga.gamma = l->gamma_dev; ga.h_out = c->h_buf; ga.h_out2 = h_out;
    ga.out = c->gate_out_dev; ga.eps = (double)cf.rms_eps; ga.H = cf.hidden; ga.E = cf.n_experts; ga.K = cf.top_k;
    ga.route_idx = c->route_idx; ga.route_w = c->route_w; ga.route_log = c->route_log_dev + (size_t)slot * MOE_MAX_TOPK;
    int32_t rc = launch_timed(c, PROF_GATE, 0, k_gate<false>, dim3(1), dim3(GATE_THREADS), 0, ga);
    if (rc) return rc;
    c->pending.push_back({l, slot});
    l->steps_device_routed++;

    const uint8_t *table[16];
    for (int e = 0; e < 16; ++e) table[e] = c->bufs[l->cache.slot_buf[l->cache.find(e < cf.n_experts ? e : 0)]].ptr;
    std::vector<FfnEntry> entries(cf.top_k);
    for (int j = 0; j < cf.top_k; ++j) {
        entries[j] = FfnEntry{};
        entries[j].n_tok = 1; entries[j].tok[0] = 0; entries[j].pair[0] = j;
    }
    rc = launch_ffn(l, entries, 1, true, table);
    if (rc) return rc;
    FusedArgs fa = token_args(l, x_in, x_out);
    fa.n_exp = cf.top_k;
    for (int j = 0; j < cf.top_k; ++j) fa.a_row[j] = j;
    fa.route_idx = c->route_idx; fa.route_w = c->route_w;
    for (int e = 0; e < 16; ++e) fa.table[e] = table[e];
    bool done = false;
    rc = launch_token(l, fa, false, false, &done);
    if (!rc && !done) rc = fail(MOE_ESTATE, "device-routed step: the single-token kernels do not fit this shape");
    return rc;
}

// One decode step of one layer.  plain: the variant for callers that cannot allocate -- the host waits for the gate
// (no selection log in the arena) and the one-launch kernel with its barrier flags in the arena is not used.
static int32_t step_impl(moe_layer *l, moe_layer *next, const uint16_t *x_in, int32_t batch, uint16_t *x_out, uint16_t *h_out,
                         moe_step_trace_t *trace, bool plain)
{
    int32_t rc = check_step_args(l, next, batch);
    if (rc) return rc;
    moe_ctx *c = l->ctx;
    if (c->host_only) return fail(MOE_ESTATE, "moe_layer_step: host-only context");
    if (!x_in || !x_out) return fail(MOE_EINVAL, "moe_layer_step: null activation pointer");
    if (!all_loaded(l)) return fail(MOE_ESTATE, "moe_layer_step: not every expert of the layer is loaded");
    const moe_layer_config_t &cf = l->cfg;
    const bool spec = next && next->cfg.prefetch_m > 0 && c->cfg.n_staging > 0;
    if (spec && !all_loaded(next)) return fail(MOE_ESTATE, "moe_layer_step: next layer not fully loaded");
    l->stepped = true;
    if (spec) next->stepped = true;
    if (!plain && device_routed_step_fits(l, next, batch, trace, spec)) return device_routed_step(l, x_in, x_out, h_out);
    rc = fold_pending(c);
    if (rc) return rc;

    GateArgs ga{};
    ga.x = x_in; ga.wg = l->gate_w_dev; ga.wg2 = spec ? next->gate_w_dev : nullptr;
    ga.gamma = l->gamma_dev; ga.h_out = c->h_buf; ga.h_out2 = h_out; ga.out = c->gate_out_dev;
    ga.eps = (double)cf.rms_eps; ga.H = cf.hidden; ga.E = cf.n_experts; ga.E2 = spec ? next->cfg.n_experts : 0; ga.K = cf.top_k;
    rc = launch_gate(c, ga, batch);
    if (rc) return rc;

    const GateHostOut *go = c->gate_out;
    int32_t idx[MOE_MAX_BATCH * MOE_MAX_TOPK];
    float w[MOE_MAX_BATCH * MOE_MAX_TOPK];
    for (int i = 0; i < batch * cf.top_k; ++i) { idx[i] = go->idx[i]; w[i] = go->w[i]; }
    double score[MOE_MAX_EXPERTS] = {0};
    if (spec)
        for (int b = 0; b < batch; ++b)
            for (int e = 0; e < ga.E2; ++e) score[e] += go->spec_p[b * ga.E2 + e];

    StepPlan plan;
    rc = plan_step(l, next, idx, batch, spec ? score : nullptr, trace, plan);
    if (rc) return rc;
    c->ypart_extra_used = 0;
    if (trace) {
        for (int i = 0; i < batch * cf.top_k; ++i) trace->expert_w[i] = w[i];
        for (int i = 0; i < batch * cf.n_experts; ++i) trace->logits[i] = go->logits[i];
    }

    // Split the accesses into passes in which no pool buffer is used twice (only possible when more
    // experts are needed than the layer has slots).  A later pass's copies wait for the earlier pass's kernels.
    std::vector<std::vector<int>> passes(1);
    {
        std::vector<int32_t> used;
        for (int i = 0; i < (int)plan.access.size(); ++i) {
            const int32_t buf = plan.access[i].buf;
            if (std::find(used.begin(), used.end(), buf) != used.end()) { passes.emplace_back(); used.clear(); }
            used.push_back(buf);
            passes.back().push_back(i);
        }
    }
    // largest number of tokens routed to one expert decides the kernel variant
    int max_tok = 1;
    for (const AccessRec &a : plan.access) {
        int n = 0;
        for (int i = 0; i < batch * cf.top_k; ++i) n += (idx[i] == a.expert);
        max_tok = std::max(max_tok, n);
    }
    const int nt = std::min(max_tok == 1 ? 1 : (max_tok == 2 ? 2 : 4), max_tokens_per_entry(cf.hidden, fmt_of(l->lay)));

    if (c->gate_out->ffn_error) return fail(MOE_ESTATE, "an earlier fused FFN kernel gave up waiting at its grid barrier");
    const bool try_fused = c->token_path && batch == 1 && passes.size() == 1 && plan.access.size() <= 2 &&
                           (int)plan.access.size() == cf.top_k && !plan.victim_needed;
    bool fused_done = false;
    bool spec_issued = false;          // the speculative copies went out early (prompt-sized batches, below)
    // two-level metadata: a step of the streaming kernel stages one run's quad per row, so a run must cover the step
    auto runs_ok = [&](const MatLayout &m) { return m.run_len == 0 || m.run_len == m.cols / (uint32_t)cf.group || m.run_len % TL_SG == 0; };
    const bool use_mfma = batch >= c->mfma_min_batch && cf.bits == 4 && cf.group == 64 && runs_ok(l->lay.m13) && runs_ok(l->lay.m2);
    if (use_mfma) {
        // How many parts the w2 launches of a window split their contraction into decides the order in which a
        // pair's partial sums are added, so it must not depend on how the step's experts happen to be grouped into
        // launches (which follows from what is cached, in which buffers): it is fixed here from the routing alone,
        // as if all needed experts of the window ran in one launch -- one part per block that would idle then --
        // within the rows the partial sums have.  A step's result is then the same whatever the cache held.
        const int window = MF_MAX_PAIRS / cf.top_k, n_cu = c->n_cu > 0 ? c->n_cu : 256;
        const int row_blocks = (cf.hidden + TL_ROWS - 1) / TL_ROWS;
        const uint64_t extra_rows = c->ypart_extra_floats / cf.hidden, pairs = (uint64_t)batch * cf.top_k;
        const int max_parts = (int)std::min<uint64_t>(255, std::max<uint64_t>(1, extra_rows / pairs));
        c->w2_parts.clear();
        c->win_small.clear();
        for (int w0 = 0; w0 < batch; w0 += window) {
            const int w1 = std::min(batch, w0 + window);
            int count[MOE_MAX_EXPERTS] = {0}, entries = 0;
            for (int q = w0 * cf.top_k; q < w1 * cf.top_k; ++q) count[idx[q]]++;
            int most = 0;
            for (int e = 0; e < cf.n_experts; ++e) { entries += (count[e] + 31) / 32; most = std::max(most, count[e]); }
            c->win_small.push_back(most <= 16);
            // at least four: the experts that arrive during a step are multiplied one launch each, and with fewer
            // parts such a launch leaves most of the chip idle on the step's critical path
            const int want = std::max(4, (2 * n_cu + entries * row_blocks - 1) / std::max(1, entries * row_blocks));
            c->w2_parts.push_back(std::min(want, max_parts));
        }
    }
    auto pass_expert = [&](int i) {
        PassExpert pe;
        pe.blob = c->bufs[plan.access[i].buf].ptr;
        for (int q = 0; q < batch * cf.top_k; ++q)
            if (idx[q] == plan.access[i].expert) pe.pairs.push_back(q);
        return pe;
    };
    // The accesses `set` as one launch (pair): matrix cores, or GEMV entries of up to nt tokens each.
    auto launch_set = [&](const std::vector<int> &set) -> int32_t {
        if (set.empty()) return MOE_OK;
        if (use_mfma) {
            std::vector<PassExpert> g;
            for (int i : set) g.push_back(pass_expert(i));
            return launch_mfma(l, g, w, batch);
        }
        std::vector<FfnEntry> entries;
        for (int i : set) {
            FfnEntry en{};
            en.blob = c->bufs[plan.access[i].buf].ptr;
            for (int q = 0; q < batch * cf.top_k; ++q) {
                if (idx[q] != plan.access[i].expert) continue;
                en.tok[en.n_tok] = q / cf.top_k; en.pair[en.n_tok] = q; en.w[en.n_tok] = w[q];
                if (++en.n_tok == nt) { entries.push_back(en); en.n_tok = 0; }
            }
            if (en.n_tok) entries.push_back(en);
        }
        return launch_ffn(l, entries, nt);
    };
    // A step of several tokens in which every buffer that changes hands belonged to an expert resident when the step
    // began (a prompt, Sec. 3, needs nearly every expert of a layer, and so does a decode batch of a few dozen
    // tokens).  Those experts are multiplied first, in one launch, before any transfer is issued; a transfer into one
    // of their buffers -- a miss that found no free staging buffer, a speculative load for the next layer -- then
    // waits for that launch only, not for the multiplies of the experts still arriving, which follow one by one as
    // their copies land, each under the next one's transfer.  The link never waits for a multiply that itself waits
    // for the link.
    bool staged_step = false;
    if (batch > 1 && plan.victims_resident && (!use_mfma || batch > c->staged_min_batch)) {
        std::vector<int> first, arriving;
        std::vector<int32_t> read_first;       // buffers the first launch reads
        for (int i = 0; i < (int)plan.access.size(); ++i) {
            const AccessRec &a = plan.access[i];
            if (a.status != MOE_HIT) { arriving.push_back(i); continue; }
            PoolBuf &pb = c->bufs[a.buf];
            if (pb.pending) { HIPCHK(hipStreamWaitEvent(c->compute, pb.ready, 0)); pb.pending = false; }
            first.push_back(i);
            read_first.push_back(a.buf);
        }
        rc = launch_set(first);
        if (rc) return rc;
        bool guarded = false;
        auto needs_guard = [&](int32_t buf) { return !guarded && std::find(read_first.begin(), read_first.end(), buf) != read_first.end(); };
        for (int i : arriving) {
            const int di = plan.demand_of[i];
            if (di >= 0 && needs_guard(plan.demand[di].buf)) {
                HIPCHK(hipEventRecord(c->ev_compute, c->compute));
                HIPCHK(hipStreamWaitEvent(c->copy, c->ev_compute, 0));
                guarded = true;
            }
            rc = issue_access_transfers(c, l, plan, i);
            if (rc) return rc;
        }
        for (const CopyOp &op : plan.spec) {
            if (needs_guard(op.buf)) {
                HIPCHK(hipEventRecord(c->ev_compute, c->compute));
                HIPCHK(hipStreamWaitEvent(c->copy, c->ev_compute, 0));
                guarded = true;
            }
            rc = issue_copy(c, next, op);
            if (rc) return rc;
        }
        for (int i : arriving) {
            PoolBuf &pb = c->bufs[plan.access[i].buf];
            if (pb.pending) { HIPCHK(hipStreamWaitEvent(c->compute, pb.ready, 0)); pb.pending = false; }
            rc = launch_set(std::vector<int>{i});
            if (rc) return rc;
        }
        staged_step = true;
        spec_issued = true;
    }
    for (size_t p = 0; p < passes.size() && !staged_step; ++p) {
        if (p > 0) {
            HIPCHK(hipEventRecord(c->ev_compute, c->compute));
            HIPCHK(hipStreamWaitEvent(c->copy, c->ev_compute, 0));
        }
        for (int i : passes[p]) { rc = issue_access_transfers(c, l, plan, i); if (rc) return rc; }
        if (p + 1 == passes.size() && !plan.victim_needed && passes.size() == 1)
            for (const CopyOp &op : plan.spec) { rc = issue_copy(c, next, op); if (rc) return rc; }
        if (use_mfma) {
            // Experts already on the device go first, in one launch pair per window.  For a prompt-sized batch the
            // experts still in flight then follow one by one in the order their copies were issued, each waiting
            // for its own copy only: the multiply of one expert runs under the transfer of the next.
            const bool one_by_one = batch > 64;
            std::vector<PassExpert> group;
            std::vector<int> in_flight;
            for (int i : passes[p]) {
                PoolBuf &pb = c->bufs[plan.access[i].buf];
                if (one_by_one && pb.pending) { in_flight.push_back(i); continue; }
                if (pb.pending) { HIPCHK(hipStreamWaitEvent(c->compute, pb.ready, 0)); pb.pending = false; }
                group.push_back(pass_expert(i));
            }
            if (!group.empty()) {
                rc = launch_mfma(l, group, w, batch);
                if (rc) return rc;
            }
            for (int i : in_flight) {
                PoolBuf &pb = c->bufs[plan.access[i].buf];
                HIPCHK(hipStreamWaitEvent(c->compute, pb.ready, 0));
                pb.pending = false;
                rc = launch_mfma(l, std::vector<PassExpert>{pass_expert(i)}, w, batch);
                if (rc) return rc;
            }
            continue;
        }
        std::vector<FfnEntry> entries;
        for (int i : passes[p]) {
            const AccessRec &a = plan.access[i];
            PoolBuf &pb = c->bufs[a.buf];
            if (pb.pending) { HIPCHK(hipStreamWaitEvent(c->compute, pb.ready, 0)); pb.pending = false; }
            FfnEntry en{};
            en.blob = pb.ptr;
            for (int q = 0; q < batch * cf.top_k; ++q) {
                if (idx[q] != a.expert) continue;
                en.tok[en.n_tok] = q / cf.top_k; en.pair[en.n_tok] = q; en.w[en.n_tok] = w[q];
                if (++en.n_tok == nt) { entries.push_back(en); en.n_tok = 0; }
            }
            if (en.n_tok) entries.push_back(en);
        }
        if (try_fused) {
            FusedArgs fa = token_args(l, x_in, x_out);
            fa.n_exp = (int32_t)entries.size();
            for (int i = 0; i < fa.n_exp; ++i) { fa.blob[i] = entries[i].blob; fa.w[i] = entries[i].w[0]; fa.a_row[i] = entries[i].pair[0]; }
            if (c->fused == 2 && !plain) rc = launch_seq(l, fa, false, &fused_done);
            if (rc) return rc;
            if (fused_done) {
                // the expert-after-expert kernel did the whole FFN
            } else if (c->fused == 1 && !plain) {
                rc = launch_token(l, fa, true, false, &fused_done);
            } else {
                rc = launch_token(l, fa, false, true, &fused_done);       // does the shape fit the token kernels?
                if (!rc && fused_done) rc = launch_ffn(l, entries, nt, true);
                if (!rc && fused_done) rc = launch_token(l, fa, false, false, &fused_done);
            }
            if (rc) return rc;
        }
        if (!fused_done) {
            rc = launch_ffn(l, entries, nt);
            if (rc) return rc;
        }
    }
    if ((plan.victim_needed || passes.size() > 1) && !spec_issued) {
        // a buffer freed during this step may still be read by its kernels: speculative copies wait for them
        HIPCHK(hipEventRecord(c->ev_compute, c->compute));
        HIPCHK(hipStreamWaitEvent(c->copy, c->ev_compute, 0));
        for (const CopyOp &op : plan.spec) { rc = issue_copy(c, next, op); if (rc) return rc; }
    }
    if (!fused_done) {      // S7: the pairs' rows added per token in a fixed order, then the residual
        const uint64_t cap_rows = ((uint64_t)batch * cf.top_k * cf.hidden + c->ypart_extra_floats) / cf.hidden;
        hipLaunchKernelGGL(k_combine, dim3((cf.hidden / 4 + 255) / 256, batch), dim3(256), 0, c->compute, x_in, c->ypart, c->ytab, c->yacc,
                           x_out, cf.hidden, cf.top_k, (uint32_t)cap_rows);
        HIPCHK(hipGetLastError());
    }
    return MOE_OK;
}

extern "C" int32_t moe_layer_step(moe_layer_t *l, moe_layer_t *next, const uint16_t *x_in, int32_t batch,
                                  uint16_t *x_out, uint16_t *h_out, moe_step_trace_t *trace)
try {
    return step_impl(l, next, x_in, batch, x_out, h_out, trace, false);
} catch (...) {
    return on_exception("moe_layer_step");
}

extern "C" int32_t moe_layer_step_noalloc(moe_layer_t *l, moe_layer_t *next, const uint16_t *x_in, int32_t batch,
                                          uint16_t *x_out, uint16_t *h_out, moe_step_trace_t *trace)
try {
    int32_t rc = check_step_args(l, next, batch);
    if (rc) return rc;
    moe_ctx *c = l->ctx;
    if (c->host_only || !c->noalloc_scratch) return fail(MOE_ESTATE, "moe_layer_step_noalloc: the context has no GPU");
    if (batch > NOALLOC_MAX_BATCH || l->cfg.hidden > NOALLOC_MAX_HIDDEN || l->cfg.ffn > NOALLOC_MAX_FFN || l->cfg.top_k > NOALLOC_MAX_TOPK)
        return fail(MOE_EINVAL, "moe_layer_step_noalloc: batch %d, hidden %d, ffn %d, top_k %d exceed the fixed scratch (at most %d, %d, %d, %d)",
                    batch, l->cfg.hidden, l->cfg.ffn, l->cfg.top_k, NOALLOC_MAX_BATCH, NOALLOC_MAX_HIDDEN, NOALLOC_MAX_FFN, NOALLOC_MAX_TOPK);
    if (c->prof.on) return fail(MOE_ESTATE, "moe_layer_step_noalloc: switch the launch timing off first (it may create events)");
    // the kernels of this step take their scratch from the file-scope array: same kernels, other pointers
    struct Swap {
        moe_ctx *c; uint16_t *h, *a; float *y, *yp; uint32_t *yt; uint64_t extra; int32_t min_batch;
        ~Swap() { c->h_buf = h; c->a_buf = a; c->yacc = y; c->ypart = yp; c->ytab = yt; c->ypart_extra_floats = extra; c->mfma_min_batch = min_batch; }
    } restore{c, c->h_buf, c->a_buf, c->yacc, c->ypart, c->ytab, c->ypart_extra_floats, c->mfma_min_batch};
    uint8_t *s = c->noalloc_scratch;
    c->h_buf = reinterpret_cast<uint16_t *>(s); s += NOALLOC_H_BYTES;
    c->a_buf = reinterpret_cast<uint16_t *>(s); s += NOALLOC_A_BYTES;
    c->yacc = reinterpret_cast<float *>(s); s += NOALLOC_Y_BYTES;
    c->ypart = reinterpret_cast<float *>(s); s += NOALLOC_YPART_BYTES;
    c->ytab = reinterpret_cast<uint32_t *>(s);
    c->ypart_extra_floats = 0;
    c->mfma_min_batch = INT32_MAX;      // its four tokens at most run on the GEMV kernels, whose scratch is what the array is sized for
    return step_impl(l, next, x_in, batch, x_out, h_out, trace, true);
} catch (...) {
    return on_exception("moe_layer_step_noalloc");
}

extern "C" int32_t moe_layer_prefetch(moe_layer_t *l, const uint16_t *h_dev, int32_t batch, moe_step_trace_t *trace)
try {
    int32_t rc = check_step_args(l, nullptr, batch);
    if (rc) return rc;
    moe_ctx *c = l->ctx;
    if (c->host_only) return fail(MOE_ESTATE, "moe_layer_prefetch: host-only context");
    if (!h_dev) return fail(MOE_EINVAL, "moe_layer_prefetch: h_dev is null");
    if (!all_loaded(l)) return fail(MOE_ESTATE, "moe_layer_prefetch: not every expert of the layer is loaded");
    if (trace) trace->n_guess = 0;
    if (l->cfg.prefetch_m <= 0 || c->cfg.n_staging <= 0) return MOE_OK;
    rc = fold_pending(c);
    if (rc) return rc;
    l->stepped = true;
    GateArgs ga{};
    ga.x = h_dev; ga.wg2 = l->gate_w_dev; ga.out = c->gate_out_dev; ga.eps = 0.0; ga.H = l->cfg.hidden;
    ga.E2 = l->cfg.n_experts; ga.K = l->cfg.top_k;
    rc = launch_gate(c, ga, batch);
    if (rc) return rc;
    double score[MOE_MAX_EXPERTS] = {0};
    for (int b = 0; b < batch; ++b)
        for (int e = 0; e < ga.E2; ++e) score[e] += c->gate_out->spec_p[b * ga.E2 + e];
    std::vector<int32_t> guess = top_m(score, l->cfg.n_experts, l->cfg.prefetch_m), issued;
    std::vector<CopyOp> copies;
    stage_guesses(l->cache, c->pool, l->st, guess, issued, copies);
    for (CopyOp &op : copies) {
        op.offset = 0;
        op.bytes = c->spec_head_bytes ? std::min<uint64_t>(c->spec_head_bytes, l->lay.total) : l->lay.total;
        op.host_buf = l->host_buf_of[op.expert];
        c->bufs[op.buf].have = op.bytes;
        l->st.bytes_spec += op.bytes;
    }
    for (const CopyOp &op : copies) { rc = issue_copy(c, l, op); if (rc) return rc; }
    if (trace) {
        trace->n_guess = (int32_t)guess.size();
        for (size_t i = 0; i < guess.size(); ++i) { trace->guess_expert[i] = guess[i]; trace->guess_issued[i] = issued[i]; }
        for (int e = 0; e < l->cfg.n_experts; ++e) trace->guess_score[e] = score[e];
    }
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_prefetch");
}

extern "C" int32_t moe_stack_step(moe_layer_t *const *layers, int32_t n_layers, const uint16_t *x_in, int32_t batch,
                                  uint16_t *x_out, moe_step_trace_t *traces)
try {
    if (!layers || n_layers < 1) return fail(MOE_EINVAL, "moe_stack_step: no layers");
    for (int i = 0; i < n_layers; ++i)
        if (!layers[i] || layers[i]->ctx != layers[0]->ctx || layers[i]->cfg.hidden != layers[0]->cfg.hidden)
            return fail(MOE_EINVAL, "moe_stack_step: layer %d is null, of another context or another width", i);
    moe_ctx *c = layers[0]->ctx;
    const uint16_t *cur = x_in;
    for (int i = 0; i < n_layers; ++i) {
        uint16_t *dst = (i + 1 == n_layers) ? x_out : c->xbuf[i & 1];
        int32_t rc = moe_layer_step(layers[i], i + 1 < n_layers ? layers[i + 1] : nullptr, cur, batch, dst, nullptr,
                                    traces ? traces + i : nullptr);
        if (rc) return rc;
        cur = dst;
    }
    return MOE_OK;
} catch (...) {
    return on_exception("moe_stack_step");
}

// ---------------------------------------------------------------------------------------------
// state
// ---------------------------------------------------------------------------------------------

extern "C" int32_t moe_layer_stats(const moe_layer_t *l, moe_stats_t *o)
try {
    if (!l || !o) return fail(MOE_EINVAL, "moe_layer_stats: null argument");
    int32_t rc = fold_pending(l->ctx);
    if (rc) return rc;
    const Counters &s = l->st;
    *o = {s.steps, s.needed, s.hits, s.prefetch_hits, s.misses, s.evictions, s.spec_issued, s.spec_wasted, s.bytes_demand, s.bytes_spec,
          s.bytes_writeback, l->steps_device_routed};
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_stats");
}

extern "C" int32_t moe_layer_cache_state(const moe_layer_t *l, int32_t *slot_expert, uint64_t *slot_stamp, int32_t *staged,
                                         int32_t *n_staged)
try {
    if (!l) return fail(MOE_EINVAL, "moe_layer_cache_state: layer is null");
    int32_t rc = fold_pending(l->ctx);
    if (rc) return rc;
    for (int s = 0; s < l->cache.k; ++s) {
        if (slot_expert) slot_expert[s] = l->cache.slot_expert[s];
        if (slot_stamp) slot_stamp[s] = l->cache.slot_stamp[s];
    }
    if (staged)
        for (size_t i = 0; i < l->cache.staged.size() && i < MOE_MAX_EXPERTS; ++i) staged[i] = l->cache.staged[i].expert;
    if (n_staged) *n_staged = (int32_t)l->cache.staged.size();
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_cache_state");
}

extern "C" int32_t moe_layer_placement(const moe_layer_t *l, int32_t *host_buf_of, int32_t *spare_host)
try {
    if (!l) return fail(MOE_EINVAL, "moe_layer_placement: layer is null");
    if (host_buf_of)
        for (int e = 0; e < l->cfg.n_experts; ++e) host_buf_of[e] = l->host_buf_of[e];
    if (spare_host) *spare_host = l->spare_host;
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_placement");
}

extern "C" int32_t moe_layer_reset(moe_layer_t *l)
try {
    if (!l) return fail(MOE_EINVAL, "moe_layer_reset: layer is null");
    if (l->swap) return fail(MOE_ESTATE, "moe_layer_reset: a layer in swap mode cannot return to its initial placement; create it again");
    moe_ctx *c = l->ctx;
    int32_t rcf = fold_pending(c);
    if (rcf) return rcf;
    if (!c->host_only) {
        HIPCHK(hipStreamSynchronize(c->compute));
        HIPCHK(hipStreamSynchronize(c->copy));
    }
    // return staged buffers to the pool and take back the layer's current slot buffers as its own
    for (const StagedGuess &g : l->cache.staged) c->pool.free_staging.push_back(g.buf);
    l->own_bufs = l->cache.slot_buf;
    for (int32_t b : l->own_bufs) c->bufs[b].pending = false;
    cache_init(l);
    l->stepped = false;                 // both streams are idle and nothing is resident: experts may be loaded again
    if (l->cfg.init_policy == 1)
        for (int e = 0; e < l->cfg.cache_slots; ++e)
            if (l->loaded[e] == 7u) { int32_t rc = warm_fill(l, e); if (rc) return rc; }
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_reset");
}

extern "C" int32_t moe_ctx_read_y(moe_ctx_t *c, int32_t batch, int32_t hidden, float *y_host)
try {
    if (!c || !y_host) return fail(MOE_EINVAL, "moe_ctx_read_y: null argument");
    if (c->host_only) return fail(MOE_ESTATE, "moe_ctx_read_y: host-only context");
    if (batch < 1 || batch > c->cfg.max_batch || hidden < 1 || hidden > c->cfg.max_hidden)
        return fail(MOE_EINVAL, "moe_ctx_read_y: batch or hidden out of range");
    HIPCHK(hipStreamSynchronize(c->compute));
    HIPCHK(hipMemcpy(y_host, c->yacc, (size_t)batch * hidden * sizeof(float), hipMemcpyDeviceToHost));
    return MOE_OK;
} catch (...) {
    return on_exception("moe_ctx_read_y");
}

extern "C" int32_t moe_ctx_set_option(moe_ctx_t *c, const char *name, int32_t value)
try {
    if (!c || !name) return fail(MOE_EINVAL, "moe_ctx_set_option: null argument");
    const std::string n(name);
    if (n == "w13_blocks" && value >= 1) c->w13_blocks = value;
    else if (n == "w2_rows" && value >= 1 && value <= 256) c->w2_rows = value;
    else if (n == "w2_token_rows" && value >= 0 && value <= 64) c->w2_token_rows = value;
    else if (n == "sync_wait") c->sync_wait = value != 0;
    else if (n == "fused" && value >= 0 && value <= 2) c->fused = value;
    else if (n == "token_path") c->token_path = value != 0;
    else if (n == "spec_head_mb" && value >= 0) c->spec_head_bytes = (uint64_t)value << 20;
    else if (n == "mfma_min_batch" && value >= 1) c->mfma_min_batch = value;
    else if (n == "mfma_form" && value >= 0 && value <= 5) c->mfma_form = value;
    else if (n == "mfma16_waves" && (value == 4 || value == 8)) c->mfma16_waves = value;
    else if (n == "device_routing") c->device_routing = value != 0;
    else if (n == "staged_min_batch" && value >= 0) c->staged_min_batch = value;
    else if (n == "profile_copy_stride" && value >= 1) c->prof.copy_stride = value;
    else return fail(MOE_EINVAL, "moe_ctx_set_option: unknown option or bad value: %s = %d", name, value);
    return MOE_OK;
} catch (...) {
    return on_exception("moe_ctx_set_option");
}

// The timed part of moe_probe_bandwidth; the caller owns (and always releases) the events and the sink.
static int32_t probe_run(const void *src_dev, void *dst_dev, uint64_t bytes, int32_t blocks, int32_t iters, hipStream_t s,
                         hipEvent_t e0, hipEvent_t e1, uint32_t *sink, double *avg_ms)
{
    const size_t n16 = bytes / 16;
    for (int it = -1; it < iters; ++it) {      // one untimed warm-up launch
        if (it == 0) HIPCHK(hipEventRecord(e0, s));
        if (dst_dev) hipLaunchKernelGGL(k_probe_copy, dim3(blocks), dim3(256), 0, s, static_cast<const uint4 *>(src_dev), static_cast<uint4 *>(dst_dev), n16);
        else hipLaunchKernelGGL(k_probe_read, dim3(blocks), dim3(256), 0, s, static_cast<const uint4 *>(src_dev), n16, sink);
    }
    HIPCHK(hipGetLastError());
    HIPCHK(hipEventRecord(e1, s));
    HIPCHK(hipEventSynchronize(e1));
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, e0, e1));
    *avg_ms = (double)ms / iters;
    return MOE_OK;
}

extern "C" int32_t moe_probe_bandwidth(const void *src_dev, void *dst_dev, uint64_t bytes, int32_t blocks, int32_t iters,
                                       void *stream, double *avg_ms)
try {
    if (!src_dev || !avg_ms || bytes < 16 || blocks < 1 || iters < 1) return fail(MOE_EINVAL, "moe_probe_bandwidth: bad argument");
    hipEvent_t e0 = nullptr, e1 = nullptr;
    uint32_t *sink = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e == hipSuccess && !dst_dev) e = hipMalloc(reinterpret_cast<void **>(&sink), (size_t)blocks * 4);
    int32_t rc;
    if (e != hipSuccess) {
        g_hip_err = (int32_t)e;
        rc = fail(MOE_EHIP, "moe_probe_bandwidth: HIP set-up failed: %s", hipGetErrorString(e));
    } else {
        rc = probe_run(src_dev, dst_dev, bytes, blocks, iters, static_cast<hipStream_t>(stream), e0, e1, sink, avg_ms);
    }
    if (sink) (void)hipFree(sink);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    return rc;
} catch (...) {
    return on_exception("moe_probe_bandwidth");
}

extern "C" int32_t moe_layer_set_prefetch(moe_layer_t *l, int32_t m)
try {
    if (!l || m < 0 || m > MOE_MAX_GUESS) return fail(MOE_EINVAL, "moe_layer_set_prefetch: bad argument");
    int32_t rc = fold_pending(l->ctx);
    if (rc) return rc;
    l->cfg.prefetch_m = m;
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_set_prefetch");
}

extern "C" int32_t moe_layer_set_flags(moe_layer_t *l, int32_t flags)
try {
    if (!l || (flags & ~MOE_LAYER_NO_CACHE)) return fail(MOE_EINVAL, "moe_layer_set_flags: bad argument");
    if (l->swap && flags) return fail(MOE_EINVAL, "moe_layer_set_flags: a layer in swap mode cannot forget residency");
    int32_t rc = fold_pending(l->ctx);
    if (rc) return rc;
    l->cfg.flags = flags | (l->swap ? MOE_LAYER_SWAP : 0);
    return MOE_OK;
} catch (...) {
    return on_exception("moe_layer_set_flags");
}
