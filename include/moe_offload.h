/*
 * moe_offload.h -- C ABI of the MI355X (gfx950) MoE-offloading decode engine.
 *
 * The library implements the per-token decode step of a sparse Mixture-of-Experts
 * block with expert offloading, after "Fast Inference of Mixture-of-Experts
 * Language Models with Offloading" (arXiv 2312.17238):
 *
 *   - linear token-level gate and top-k expert selection            (Sec. 2.1)
 *   - an LRU cache of k experts per layer in device memory          (Sec. 3.1)
 *   - speculative loading: the next layer's gate applied to the
 *     hidden state the current layer's gate saw                     (Sec. 3.2)
 *   - one contiguous buffer per expert in pinned host memory, moved
 *     by a single asynchronous host-to-device copy, and b shared
 *     on-device staging buffers for speculative loads               (Sec. 3.3)
 *   - expert weights stored group-wise quantized (2/3/4 bit codes,
 *     a scale and a zero point per group), dequantized on the fly   (Sec. 4.2)
 *
 * Conventions
 *   - Every function returns MOE_OK (0) or a negative moe_status; nothing throws or
 *     aborts across this boundary.  moe_last_error() gives a thread-local message.
 *   - "dev" pointers are device (HBM) memory, "host" pointers are host memory.
 *     The library never frees caller memory; arenas passed to *_create must stay
 *     alive until the matching *_destroy.
 *   - Streams are hipStream_t handles passed as void*; the caller owns them.
 *     Kernels run on the compute stream, expert copies on the copy stream; the
 *     library orders the two with HIP events.  Both must have default priority.
 *   - One host thread drives a context; calls are not re-entrant.
 *   - fp16 values cross the boundary as IEEE binary16 bit patterns in uint16_t.
 */
#ifndef MOE_OFFLOAD_H
#define MOE_OFFLOAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_MAX_EXPERTS 16   /* experts per layer                    */
#define MOE_MAX_TOPK     4   /* active experts per token             */
#define MOE_MAX_BATCH   1024 /* tokens per step: a decode batch, or a prompt (or a piece of one) encoded layer by layer */
#define MOE_MAX_GUESS    4   /* speculatively loaded experts per step */

typedef enum {
    MOE_OK      =  0,
    MOE_EINVAL  = -1,  /* bad argument (null pointer, unsupported shape or format, batch > max_batch) */
    MOE_ESTATE  = -2,  /* call not valid in this state (e.g. step before every expert was loaded)    */
    MOE_ENOMEM  = -3,  /* a caller-provided arena is too small, or a small internal allocation failed */
    MOE_EHIP    = -4   /* a HIP runtime call failed; moe_last_hip_error() has its code               */
} moe_status;

/* How a needed expert was found by the cache (Sec. 3.1, 3.3). */
typedef enum {
    MOE_HIT          = 0,  /* resident in one of the layer's k slots: no transfer                    */
    MOE_PREFETCH_HIT = 1,  /* speculatively loaded earlier: installed by a buffer swap, no transfer   */
    MOE_MISS         = 2   /* one demand copy of the expert's blob over the host link                */
} moe_access_status;

typedef struct moe_ctx   moe_ctx_t;    /* owns the b staging buffers, scratch, events (shared by all layers, Sec. 3.3) */
typedef struct moe_layer moe_layer_t;  /* owns the layer's k device slots, its host blobs and its LRU state (Sec. 3.1) */

enum {
    MOE_CTX_HOST_ONLY = 1   /* no GPU: only the bookkeeping entry points work (used by CPU tests) */
};

typedef struct {
    int32_t n_staging;        /* b: shared on-device buffers for speculative loads (paper: 4)    */
    int32_t max_batch;        /* 1..MOE_MAX_BATCH                                                */
    int32_t max_hidden;       /* largest hidden size of any layer                                */
    int32_t max_ffn;          /* largest expert FFN width of any layer                           */
    int32_t max_top_k;        /* 1..MOE_MAX_TOPK                                                 */
    int32_t flags;            /* MOE_CTX_*                                                       */
    uint64_t max_expert_bytes;/* size of the largest expert blob (moe_expert_blob_bytes)         */
} moe_ctx_config_t;

enum {
    MOE_LAYER_NO_CACHE = 1,   /* ablation "without LRU cache": residency is forgotten before every step,
                                 so every needed expert is a demand copy (or a prefetch hit)       */
    MOE_LAYER_SWAP     = 2    /* hosts that cannot hold every expert (Sec. 3.3): an expert lives in exactly one
                                 buffer, on the host or on the device.  Experts 0..k-1 start on the device
                                 (init_policy must be 1), the other E-k in host buffers, and the pinned arena
                                 has E-k+1 buffers (one spare).  Loading an expert also writes the evicted one
                                 back to the host, into the spare buffer, on a stream of the library's own; the
                                 buffer the loaded expert vacated is the next spare.  Decisions, traces and
                                 results are those of the plain mode.  Set at creation only; excludes
                                 MOE_LAYER_NO_CACHE and moe_layer_reset                                */
};

typedef struct {
    int32_t hidden;           /* H: model width (multiple of 64)                                 */
    int32_t ffn;              /* F: expert FFN width (multiple of 64)                            */
    int32_t n_experts;        /* E <= MOE_MAX_EXPERTS                                            */
    int32_t top_k;            /* K <= MOE_MAX_TOPK (Mixtral: 2)                                  */
    int32_t bits;             /* 4, 3 or 2                                                       */
    int32_t group;            /* codes per (scale, zero) pair along the input dimension:
                                 4-bit: 32, 64 or 128; 3-bit: 64; 2-bit: 16                      */
    int32_t cache_slots;      /* k: device-resident experts of this layer; top_k <= k <= E       */
    int32_t prefetch_m;       /* m: experts guessed for this layer by its predecessor, 0..MOE_MAX_GUESS */
    float   rms_eps;          /* > 0: RMSNorm with this eps in front of the gate; 0: gate sees x */
    int32_t init_policy;      /* 0: cache starts empty; 1: experts 0..k-1 resident after loading */
    int32_t flags;            /* MOE_LAYER_*                                                     */
    int32_t scale_group;      /* 0: one fp16 (scale, zero) pair per group.  R > 0 (a power of two; with 2-bit
                                 codes at least 4 unless a row has no more than R groups): two-level metadata
                                 (Sec. 4.2 "scale group size") -- per group an 8-bit scale code and an 8-bit
                                 zero code, per run of R consecutive groups of a row (the whole row if it has
                                 fewer; the last run of a row may be shorter) four fp16:
                                 scale = (scale code - m[1]) * m[0], zero = (zero code - m[3]) * m[2]; the
                                 weight is (code - zero) * scale as before.  4.25 / 3.25 / 3.0 bits per weight
                                 for 4-bit g64, 3-bit g64, 2-bit g16, plus 8 bytes per run                   */
} moe_layer_config_t;

typedef struct {
    int32_t expert;           /* needed expert                                                   */
    int32_t status;           /* moe_access_status                                               */
    int32_t slot;             /* cache slot it occupies after this access                        */
    int32_t victim;           /* expert evicted from that slot, -1 if the slot was empty or on a hit */
} moe_access_t;

/* What one decode step decided.  Filled synchronously by moe_layer_step / moe_layer_resolve. */
typedef struct {
    int32_t batch, top_k, n_experts;
    int32_t expert_idx[MOE_MAX_BATCH * MOE_MAX_TOPK];   /* [b*top_k + j], best first              */
    float   expert_w  [MOE_MAX_BATCH * MOE_MAX_TOPK];   /* combine weights, sum to 1 per token    */
    double  logits    [MOE_MAX_BATCH * MOE_MAX_EXPERTS];/* [b*n_experts + e] gate logits (fp64)   */
    int32_t n_access;                                   /* distinct needed experts                */
    moe_access_t access[MOE_MAX_EXPERTS];               /* in the order they touched the cache    */
    int32_t n_guess;                                    /* speculative guesses for the next layer */
    int32_t guess_expert[MOE_MAX_GUESS];                /* most likely first                      */
    int32_t guess_issued[MOE_MAX_GUESS];                /* 1 if a copy into a staging buffer was issued */
    double  guess_score[MOE_MAX_EXPERTS];               /* summed next-layer gate probabilities   */
} moe_step_trace_t;

typedef struct {
    uint64_t steps;           /* decode steps of this layer                                      */
    uint64_t needed;          /* distinct needed experts, summed over steps                      */
    uint64_t hits, prefetch_hits, misses;
    uint64_t evictions;
    uint64_t spec_issued;     /* speculative copies issued for this layer                        */
    uint64_t spec_wasted;     /* ... of which this layer did not use                             */
    uint64_t bytes_h2d_demand;
    uint64_t bytes_h2d_spec;
    uint64_t bytes_d2h_writeback; /* MOE_LAYER_SWAP: evicted experts written back to host buffers    */
    uint64_t steps_device_routed; /* ... of `steps`, those enqueued without waiting for the gate (every
                                     expert resident, one token; option "device_routing")            */
} moe_stats_t;                /* "expert recall" (Sec. 4.1) = (hits + prefetch_hits) / needed    */

/* ---- sizes ---------------------------------------------------------------------------------- */

/* Bytes of one expert's contiguous blob (w1, w3, w2 codes and their fp16 scale/zero pairs) in the
 * library's private layout; 0 if the shape or format is unsupported.  Sec. 3.3: one buffer per expert. */
uint64_t moe_expert_blob_bytes(int32_t hidden, int32_t ffn, int32_t bits, int32_t group);
/* The same for two-level metadata (moe_layer_config_t.scale_group; 0 gives moe_expert_blob_bytes). */
uint64_t moe_expert_blob_bytes_2level(int32_t hidden, int32_t ffn, int32_t bits, int32_t group, int32_t scale_group);
/* Device arena bytes moe_ctx_create needs: b staging buffers plus activation scratch.  0 on bad config. */
uint64_t moe_ctx_dev_bytes(const moe_ctx_config_t *cfg);
/* Device bytes moe_layer_create needs: k buffers of the context's buffer size, the gate matrix, the gain. */
uint64_t moe_layer_dev_bytes(const moe_ctx_t *ctx, const moe_layer_config_t *cfg);
/* Pinned host bytes moe_layer_create needs: E blobs. */
uint64_t moe_layer_host_bytes(const moe_layer_config_t *cfg);

/* ---- life cycle ----------------------------------------------------------------------------- */

/* Create a context.  dev_arena: device memory of at least moe_ctx_dev_bytes(cfg), 256-byte aligned
 * (ignored with MOE_CTX_HOST_ONLY).  compute_stream / copy_stream: hipStream_t handles, distinct.
 * All cache slots and staging buffers of this context have one size (Sec. 3.3: equal-size buffers),
 * so a speculatively loaded expert is installed into a cache by swapping buffers, not by copying. */
int32_t moe_ctx_create(const moe_ctx_config_t *cfg, void *dev_arena, uint64_t dev_arena_bytes,
                       void *compute_stream, void *copy_stream, moe_ctx_t **out);
int32_t moe_ctx_destroy(moe_ctx_t *ctx);

/* Create one MoE layer.  gate_w_host: [E][H] fp32, copied.  rms_gamma_host: [H] fp16 bits or NULL
 * (NULL with rms_eps > 0 means gain 1).  dev_mem: moe_layer_dev_bytes, 256-byte aligned.
 * pinned_host_mem: moe_layer_host_bytes of page-locked host memory (Sec. 3.3), 64-byte aligned; in a
 * host-only context ordinary memory will do.  The expert's blob size must not exceed the context's
 * max_expert_bytes, hidden/ffn/top_k its maxima. */
int32_t moe_layer_create(moe_ctx_t *ctx, const moe_layer_config_t *cfg, const float *gate_w_host,
                         const uint16_t *rms_gamma_host, void *dev_mem, void *pinned_host_mem,
                         moe_layer_t **out);
int32_t moe_layer_destroy(moe_layer_t *layer);

/* Hand one matrix of one expert to the layer.  matrix: 0 = w1 [F][H], 1 = w3 [F][H], 2 = w2 [H][F],
 * row-major [out][in].  codes: one byte per weight, values < 2^bits.  scale/zero: fp16 bits,
 * [out][in/group], groups along `in`; the stored weight is (code - zero) * scale (Sec. 4.2).
 * All host memory, read during the call only.  The library repacks into the expert's blob in the
 * pinned arena; with init_policy 1, experts 0..k-1 are also copied to their slots once complete (with
 * MOE_LAYER_SWAP they are packed in ordinary memory of the library's own and keep no host copy).
 * Experts are loaded before the layer's first step: once the layer has taken part in moe_layer_step,
 * moe_stack_step, moe_layer_resolve or moe_layer_prefetch (as the layer itself or as `next`), both load calls
 * return MOE_ESTATE -- copies of the blob may be in flight and resident copies would go stale -- until
 * moe_layer_reset, after which matrices may be loaded again (a matrix may be loaded more than once before that). */
int32_t moe_layer_load_expert(moe_layer_t *layer, int32_t expert, int32_t matrix, const uint8_t *codes,
                              const uint16_t *scale_f16, const uint16_t *zero_f16);
/* The same for a layer with two-level metadata (scale_group > 0).  scale_code, zero_code: one byte per group,
 * [out][in/group]; run_meta: fp16 bits, [out][runs][4] with runs = ceil((in/group) / scale_group), the four
 * numbers of moe_layer_config_t.scale_group in that order.  All host memory, read during the call only. */
int32_t moe_layer_load_expert_2level(moe_layer_t *layer, int32_t expert, int32_t matrix, const uint8_t *codes,
                                     const uint8_t *scale_code, const uint8_t *zero_code, const uint16_t *run_meta_f16);
/* Read one weight back out of the packed host blob (checks the private layout without a GPU).  With two-level
 * metadata *scale_f16 and *zero_f16 receive the group's byte codes, and moe_layer_peek_run_meta the four fp16 of
 * the run the column belongs to. */
int32_t moe_layer_peek_weight(const moe_layer_t *layer, int32_t expert, int32_t matrix, int32_t row,
                              int32_t col, uint8_t *code, uint16_t *scale_f16, uint16_t *zero_f16);

int32_t moe_layer_peek_run_meta(const moe_layer_t *layer, int32_t expert, int32_t matrix, int32_t row,
                                int32_t col, uint16_t *run_meta_f16 /*[4]*/);

/* ---- the decode step ------------------------------------------------------------------------ */

/* One decode step of one layer for `batch` tokens (Sec. 3: token-by-token, layer-by-layer).
 *   x_in_dev  [batch][H] fp16, device: the block's input (residual stream).
 *   x_out_dev [batch][H] fp16, device: x_in + sum_j w_j expert_j(h); may alias x_in_dev.
 *   h_out_dev nullable, [batch][H] fp16: receives the gate input h (x, or RMSNorm(x)).
 *   next      nullable: the following layer.  If given and next->prefetch_m > 0 the step also applies
 *             next's gate to h and stages its guesses (Sec. 3.2), right after this layer's own loads
 *             were issued (Sec. 3.3).
 *   trace     nullable, host: what was decided.
 * The gate runs on the compute stream and the call waits for its result (the cache table lives on the
 * host); copies and the expert kernels are then enqueued and the call returns without waiting for
 * them: x_out is valid once the compute stream reaches this point. */
int32_t moe_layer_step(moe_layer_t *layer, moe_layer_t *next, const uint16_t *x_in_dev, int32_t batch,
                       uint16_t *x_out_dev, uint16_t *h_out_dev, moe_step_trace_t *trace);

/* moe_layer_step for callers that cannot allocate device memory: code that runs while a HIP graph is being captured
 * elsewhere in the process, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same decisions,
 * traces and results as moe_layer_step with option "mfma_min_batch" above the batch (its four tokens at most always run
 * on the GEMV kernels), computed by the same kernels; the difference is where those kernels keep
 * their intermediate results (the gate input h, the SwiGLU activations a, the pairs' fp32 partial outputs, the block
 * output y): not in the context's arena but in a fixed array inside the library's own device image (1.2 MB, held by
 * every GPU the library runs on until the process ends).  The call makes no device or pinned-host allocation, frees none and
 * creates no stream or event; its host-side bookkeeping uses the ordinary C++ heap.  Limits, checked with MOE_EINVAL:
 * batch <= 4, hidden <= 8192, ffn <= 16384, top_k <= 4.  MOE_ESTATE while launch timing (moe_ctx_profile_enable) is on,
 * and in a host-only context.  The host always waits for the gate here (no device-routed steps) and option "fused" is
 * ignored.  The array keeps the previous call's contents; what must start at zero is cleared by the step's own gate
 * kernel.  All calls on one GPU, from any context, share the one array: two that overlap in time (different
 * contexts on different streams) race; calls of one context are ordered by its compute stream.
 * moe_ctx_read_y does not see the y of such a step. */
int32_t moe_layer_step_noalloc(moe_layer_t *layer, moe_layer_t *next, const uint16_t *x_in_dev, int32_t batch,
                               uint16_t *x_out_dev, uint16_t *h_out_dev, moe_step_trace_t *trace);

/* Stand-alone speculative loading (Sec. 3.2): apply `layer`'s own gate to h_dev [batch][H] fp16 (the
 * previous layer's gate input) and stage up to prefetch_m guesses for `layer`.  Makes exactly the
 * decisions moe_layer_step(prev, next=layer) makes.  trace (nullable) gets n_guess, guess_*. */
int32_t moe_layer_prefetch(moe_layer_t *layer, const uint16_t *h_dev, int32_t batch, moe_step_trace_t *trace);

/* Run `n_layers` layers back to back on one batch: x_in_dev -> x_out_dev through layers[0..n-1], each
 * prefetching for its successor.  traces: nullable array of n_layers traces. */
int32_t moe_stack_step(moe_layer_t *const *layers, int32_t n_layers, const uint16_t *x_in_dev, int32_t batch,
                       uint16_t *x_out_dev, moe_step_trace_t *traces);

/* The cache/prefetch bookkeeping of one step on its own, for given routing (host arrays):
 * expert_idx [batch][top_k]; guess_score nullable [next->n_experts] (summed next-layer probabilities).
 * In a GPU context it also issues the copies it decides on; in a host-only context it moves no data.
 * moe_layer_step calls exactly this after its gate kernel. */
int32_t moe_layer_resolve(moe_layer_t *layer, moe_layer_t *next, const int32_t *expert_idx, int32_t batch,
                          const double *guess_score, moe_step_trace_t *trace);

/* ---- state ---------------------------------------------------------------------------------- */

/* Both calls below first bring the bookkeeping of device-routed steps up to date (option "device_routing"), which
 * waits for the compute stream when such steps are pending. */
int32_t moe_layer_stats(const moe_layer_t *layer, moe_stats_t *out);
/* Cache contents: slot_expert[k] (expert id or -1), slot_stamp[k] (recency, larger = more recent),
 * staged[MOE_MAX_EXPERTS] (n_staged ids speculatively loaded for this layer).  Any pointer may be NULL. */
int32_t moe_layer_cache_state(const moe_layer_t *layer, int32_t *slot_expert, uint64_t *slot_stamp,
                              int32_t *staged, int32_t *n_staged);
/* MOE_LAYER_SWAP: where every expert's blob is.  host_buf_of[E]: index of the host buffer that holds expert e,
 * or -1 while it is on the device; *spare_host: the host buffer holding nothing.  Without the flag expert e is in
 * buffer e and *spare_host is -1.  Either pointer may be NULL. */
int32_t moe_layer_placement(const moe_layer_t *layer, int32_t *host_buf_of, int32_t *spare_host);
/* Forget residency, staged guesses and statistics (cold cache, or warm per init_policy). Waits for both streams. */
int32_t moe_layer_reset(moe_layer_t *layer);
/* Change m, the number of experts its predecessor guesses for this layer (ablation "without pre-loading"). */
int32_t moe_layer_set_prefetch(moe_layer_t *layer, int32_t prefetch_m);
/* Set or clear MOE_LAYER_* flags. */
int32_t moe_layer_set_flags(moe_layer_t *layer, int32_t flags);

/* Diagnostic: copy the fp32 block output y [batch][hidden] of the most recent step (the weighted expert
 * sum before the residual add) to host memory.  Waits for the compute stream. */
int32_t moe_ctx_read_y(moe_ctx_t *ctx, int32_t batch, int32_t hidden, float *y_host);

/* Optional timing of the engine's own launches, with HIP events recorded on the stream each launch is
 * enqueued on (gate, w1/w3 kernel, w2 kernel, one-launch single-token FFN kernel `ffn`: compute stream;
 * expert copies: copy stream; write-backs of evicted experts in swap mode: the library's write-back stream).
 * `bytes` are algorithmic: each distinct expert a launch touches counts its packed w1+w3 (or w2) once;
 * a copy counts the blob.  enable(1) clears the accumulators; read waits for both streams.
 * Option "profile_copy_stride" = n > 1 times only every n-th transfer (copy and write-back entries then cover those
 * transfers only; the byte totals of all transfers are in moe_stats_t): two event records around every copy take
 * about 1 % off a saturated link. */
typedef struct { uint64_t launches; uint64_t bytes; double total_ms; } moe_profile_entry_t;
typedef struct { moe_profile_entry_t gate, w13, w2, copy, ffn, writeback; } moe_profile_t;
int32_t moe_ctx_profile_enable(moe_ctx_t *ctx, int32_t on);
int32_t moe_ctx_profile_read(moe_ctx_t *ctx, moe_profile_t *out);
/* Diagnostic: when each launch of one kind (0 gate, 1 w1/w3, 2 w2, 3 copy, 4 ffn, 5 write-back) recorded since
 * enable(1) -- and not yet consumed by moe_ctx_profile_read -- began and ended, in ms after the enable call.
 * *n receives how many there are; at most cap are written.  Waits for the streams. */
int32_t moe_ctx_profile_timeline(moe_ctx_t *ctx, int32_t kind, double *start_ms, double *stop_ms, int32_t cap, int32_t *n);

/* Launch-shape tuning knobs (defaults are the measured best for Mixtral shapes on MI355X):
 *   "w13_blocks" total thread blocks of the w1/w3 kernel (default 256: one per compute unit);
 *   "w2_rows"    output rows per block of the w2 kernel (default 32);
 *   "w2_token_rows" output rows per block of the single-token w2 kernel, at most 64 (default 0: hidden size /
 *                compute units, 16 for Mixtral's width);
 *   "sync_wait"  1: wait for the gate result with hipStreamSynchronize instead of polling host-mapped memory;
 *   "token_path" 1 (default): a single-token step runs w2 with the combine and the residual add inside the
 *                kernel (one block sees both experts' rows; no atomics, no separate residual kernel);
 *                0: the general kernels also for one token;
 *   "mfma_min_batch" batches at least this large (default 3, from where on they are the faster ones on MI355X; 16
 *                is the benchmark definition's threshold) run 4-bit group-64 experts on the matrix cores (grouped
 *                dequantize+GEMM); smaller batches, and other formats, use the GEMV kernels;
 *   "mfma_form"  which matrix-core kernels.  0 (default): form 5.  4: persistent streaming kernels with
 *                tiles of 16 tokens -- one tile per expert while no expert has more than 16 tokens of a window of up to
 *                256 / top_k tokens of the step, else two, decided per window from its routing alone, so that a token's
 *                result does not depend on which experts share a launch -- each dequantised weight rounded once to fp16
 *                before the multiply, as Sec. 4.2's fp16 experts do; fp16 metadata only (form 2 runs otherwise).  5: the
 *                kernels of form 4 with the weights not dequantised at all: the codes enter the matrix cores as they are
 *                and a group's product is corrected for the zero-point and scaled in fp32 (no rounding of a weight; any
 *                finite pair; fp16 and two-level metadata, the latter decoded in fp32).  2: form 4's arithmetic with
 *                tiles of 32 tokens.  3: as 2 with one fused multiply-add per pair of weights and the part its rounded
 *                constant leaves added back as a rank-1 term by one more matrix instruction per tile (fp16 metadata; with
 *                two-level metadata, and for a layer loaded with a pair whose (1024 + |zero|) * |scale| exceeds 16384 --
 *                the form computes that product in fp16 -- form 2 runs).  1: row-staging kernels that keep the codes
 *                exact and scale every group's product in fp32 (batches of at most 64 tokens, fp16 metadata; otherwise
 *                form 2 runs).  All meet the output tolerance;
 *   "mfma16_waves" waves per block of the kernels of forms 4 and 5 for up to 16 tokens per expert: 8 (default; 128
 *                registers, four waves per SIMD) or 4 (two groups of a step per wave; form 4 only); with two token tiles
 *                they always run 4;
 *   "spec_head_mb" 0 (default): a speculative load copies the whole expert at once, as the paper describes;
 *                N > 0: it copies only the first N MiB, and the rest is fetched (like a demand load) when the next
 *                layer confirms the guess.  Decisions, traces and results are identical; only how many bytes a wrong
 *                guess costs changes (N MiB instead of a whole expert).  Meant for links that are already saturated;
 *   "fused"      such a step runs w1/w3 and w2 as ONE persistent launch: 1 with a grid barrier between them, 2 expert
 *                after expert with one set of flags per expert (both measured slower than two launches on MI355X,
 *                hence default 0);
 *   "staged_min_batch" matrix-core batches larger than this (default 0: all of them; GEMV batches of more than one
 *                token always) run a step in three stages when every buffer that changes hands in it belonged to an
 *                expert resident at its start: those experts are multiplied first, then the transfers are issued (one
 *                into a buffer that launch reads waits for it alone), then the arriving experts are multiplied one by
 *                one as their copies land.  Otherwise, and below the threshold, a step whose buffers are used twice
 *                runs in passes, a pass's copies waiting for all kernels of the pass before;
 *   "device_routing" 1 (default): a single-token step of a layer whose experts are ALL on the device (cache_slots ==
 *                n_experts, every slot filled) and whose caller asks for no trace is enqueued without waiting for
 *                its gate kernel: no cache decision depends on the routing then, so the FFN kernels read the selection
 *                and the combine weights the gate kernel left in device memory, and moe_layer_step returns at once.
 *                Outputs are bit-identical to a waiting step's.  The recency stamps and counters such steps owe are
 *                caught up from a log of the selections in device memory (copied back after waiting for the compute
 *                stream) before any call reads or changes them: moe_layer_stats, moe_layer_cache_state, moe_layer_reset, a waiting step,
 *                moe_layer_resolve, moe_layer_prefetch, moe_layer_destroy, or when 8192 such steps are pending.
 *                0: every step waits for its gate. */
int32_t moe_ctx_set_option(moe_ctx_t *ctx, const char *name, int32_t value);

/* Calibration probe, independent of any context: `iters` launches of a plain streaming-read kernel over
 * src_dev (dst_dev NULL) or of a plain copy kernel src_dev -> dst_dev, `blocks` blocks of 256 threads,
 * 128-bit accesses; returns the average milliseconds per launch (HIP events on `stream`).  Used as the
 * measured ceiling beside the nominal HBM peak and as the known-size kernel that scales hardware counters. */
int32_t moe_probe_bandwidth(const void *src_dev, void *dst_dev, uint64_t bytes, int32_t blocks, int32_t iters,
                            void *stream, double *avg_ms);

const char *moe_last_error(void);
int32_t moe_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MOE_OFFLOAD_H */
