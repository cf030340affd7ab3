/*
 * expertflow.h -- C ABI of the MI355X (gfx950) MoE-layer hot path with adaptive
 * expert prefetching and cache-aware routing.
 *
 * One GPU, one context per model replica.  Plain C: opaque context, plain
 * pointers and sizes.  Every pointer is tagged [dev] (device memory on the
 * current HIP device), [host] (ordinary host memory) or [pinned] (page-locked
 * host memory).  `stream` arguments are a hipStream_t passed as void*
 * (NULL = the default stream).  The caller owns every buffer it passes; the
 * library owns the context, its HBM expert-slot pool, its copy stream, its
 * events and its scratch buffers.
 *
 * Asynchrony: ef_predict / ef_route / ef_moe_ffn only enqueue work on `stream`
 * (ef_moe_ffn may run part of a layer's kernels on a side stream of its own,
 * forked from and joined back into `stream` by events inside the call);
 * outputs are valid once the caller has synchronised that stream.
 * ef_cache_swap_in enqueues a host-to-device copy on the library's own copy
 * stream and returns at once.
 *
 * Errors: every call returns 0 (EF_OK) or a negative code; on error nothing
 * has been enqueued.  ef_last_error() gives the text of the last failure.
 *
 * Limits: n_experts <= 64, top_k <= 8 and <= n_experts, look-ahead H <= 7,
 * d_model a multiple of 64, d_ff and d_ff_shared multiples of 32.
 *
 * Expert weight layout ("packed blob").  An expert (SwiGLU: W1 [F,d] gate,
 * W3 [F,d] up, W2 [d,F] down, bf16) is stored as ef_expert_bytes(d,F) =
 * 3*d*F*2 bytes of 1 KiB "fragments".  A fragment holds a 32-row x 16-column
 * block of a row-major matrix M in matrix-core operand order: 64 lanes x 8
 * 16-bit numbers, lane l = 32*g + i (g in {0,1}, i in 0..31) holds
 *   natural order : M[r0 + i][c0 + 8*g + t],              t = 0..7
 *   paired order  : M[r0 + i][c0 + 8*(t/4) + 4*g + t%4],   t = 0..7
 * Section A, for rb in 0..F/32-1: d/16 natural-order fragments of W1 rows
 * [32rb, 32rb+32) (c0 = 0, 16, ...), then the same for W3.  Section B, at byte
 * 2*d*F*2, for cb in 0..d/32-1: F/16 paired-order fragments of W2 rows
 * [32cb, 32cb+32).  ef_pack_expert() builds a blob from row-major matrices.
 * Section A keeps the bf16 bit patterns.  Section B holds the same numbers as
 * fp16: the second FFN half runs the matrix cores in fp16 (fp32 accumulation)
 * so that the intermediate activation silu(g)*u between the halves keeps 11
 * significant bits instead of bf16's 8 (bf16 there puts single outputs of
 * Mixtral-sized layers at the edge of a 2e-2 absolute tolerance).  A bf16
 * number of magnitude in [2^-24, 2^16) is an fp16 number, so W2 is unchanged;
 * smaller magnitudes round to the nearest multiple of 2^-24, larger ones (and
 * inf / NaN) are refused by ef_pack_expert.  Activations beyond +-65504
 * saturate.  The layout makes every wavefront load of weights one contiguous
 * 1 KiB read that lands directly in matrix-core operand registers.
 */
#ifndef EXPERTFLOW_H
#define EXPERTFLOW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EF_MAX_EXPERTS 64
#define EF_MAX_TOPK 8
#define EF_MAX_HORIZON 7

enum {
    EF_OK = 0,
    EF_EINVAL = -1,       /* null pointer, bad shape, bad range, bad alignment */
    EF_ENOMEM = -2,       /* host or device allocation failed */
    EF_EHIP = -3,         /* a HIP runtime call failed */
    EF_EBUSY = -4,        /* no evictable cache slot */
    EF_ENOTRESIDENT = -5, /* strict mode: FFN needs an expert that is not in the cache */
    EF_ENOSYS = -6        /* not available (e.g. device call on a fake-copy context) */
};

/* ef_config.flags */
#define EF_FLAG_FAKE_COPY 1u   /* no device at all: the cache runtime runs against a fake copy
                                  engine and a fake clock (host-logic tests); kernels return EF_ENOSYS */
#define EF_FLAG_STRICT_RESIDENT 2u /* ef_moe_ffn fails with EF_ENOTRESIDENT instead of swapping in misses itself */
#define EF_FLAG_PROFILE 4u         /* bracket every kernel launch with HIP events on its own stream and
                                      accumulate per-kernel time, launches and algorithmic bytes in ef_stats */

#define EF_FLAG_PROFILE_FFN_UP 16u  /* as EF_FLAG_PROFILE, but only the first FFN half (the dominant kernel) */
#define EF_FLAG_FIXED_ESTIMATES 8u /* keep C_s and T_l at their initial values (reproducible horizon decisions) */

/* index of the per-kernel arrays in ef_stats */
enum {
    EF_K_PREDICT = 0,  /* gate + top-k + histogram of the look-ahead layers */
    EF_K_ROUTE = 1,    /* gate + softmax + biased top-k + per-tile counts of the current layer */
    EF_K_GROUP = 2,    /* per-expert prefix over the tiles + stable scatter: counts, offsets, perm, inv_perm */
    EF_K_FFN_UP_TILED = 3,   /* first FFN half, groups with many tokens (matrix-core bound tiles) */
    EF_K_PACK = 4,     /* token permutation into per-expert operand tiles */
    EF_K_FFN_UP = 5,   /* grouped act = silu(X W1^T) * (X W3^T) */
    EF_K_FFN_DOWN = 6, /* grouped Y = act W2^T */
    EF_K_COMBINE = 7,  /* weighted un-permute */
    EF_K_FFN_DOWN_TILED = 8, /* second FFN half, groups with many tokens */
    EF_K_DIST = 9,     /* intra-batch diversity Dist(t): norms, Gram tiles, reductions (one bracket) */
    EF_K_COUNT = 10
};

typedef struct ef_ctx ef_ctx;

typedef struct ef_config {
    int32_t n_layers;
    int32_t d_model;             /* d */
    int32_t n_experts;           /* E routed experts per layer */
    int32_t top_k;               /* k */
    int32_t d_ff;                /* F, hidden dim of a routed expert */
    int32_t d_ff_shared;         /* hidden dim of the always-resident dense SwiGLU (0 = none) */
    int32_t slots_total;         /* HBM expert cache: number of expert-sized slots in the pool */
    int32_t slots_per_layer_max; /* cap of resident experts per layer, 0 = no cap */
    int32_t max_tokens;          /* largest T any call will pass (sizes the scratch) */
    int32_t h_max;               /* clamp of the look-ahead horizon, 1..EF_MAX_HORIZON */
    int32_t renorm_topk;         /* 1: combine weights are renormalised over the selected k */
    float routed_scale;          /* factor on the combine weights */
    float cum_threshold;         /* tau of the expected-activation rule (paper Sec. 3.2.1) */
    int32_t stall_thresh;        /* feedback loop: stalls before S += 1 (paper Sec. 3.2.2) */
    int32_t overfetch_thresh;    /* feedback loop: overfetches before S -= 1 */
    uint32_t flags;
    float init_bandwidth_gbps;   /* starting value of the C_s estimate, GB/s */
    float init_layer_us;         /* starting value of the T_l estimate, microseconds */
    int32_t weight_bits;         /* routed experts: 0 or 16 = bf16 blobs, 4 = 4-bit blobs (see ef_pack_expert_q4) */
} ef_config;

typedef struct ef_stats {
    int64_t hits;               /* experts needed by a layer and found resident (ready or in flight) */
    int64_t misses;             /* experts needed by a layer and not resident: priority swap-ins */
    int64_t prefetch_issued;    /* prefetch swap-ins that started a copy */
    int64_t prefetch_redundant; /* prefetch requests for experts already resident ("overfetch") */
    int64_t evictions;
    int64_t bytes_copied;       /* host-to-device expert bytes */
    int64_t bytes_timed;        /* bytes of the copy chunks that copy_seconds covers (chunks that followed another
                                   chunk on the link without a gap: their time is transfer time) */
    int64_t layers_run;         /* ef_moe_ffn calls */
    int64_t tokens_run;         /* sum of T over ef_moe_ffn calls */
    double copy_seconds;        /* summed duration of the timed chunks (copy-stream events between consecutive
                                   chunks): bytes_timed / copy_seconds is the rate the link sustains */
    double stall_seconds;       /* time the compute stream spent waiting for swap-ins */
    double layer_seconds;       /* summed ef_route..ef_moe_ffn layer time (compute-stream events) */
    double bandwidth_Bps;       /* current C_s estimate */
    double layer_seconds_est;   /* current T_l estimate */
    double miss_rate;           /* R_miss = 1 - hits / (hits + misses)  (paper Sec. 2.2) */
    int32_t horizon;            /* current look-ahead S */
    int32_t stall_counter, overfetch_counter;
    int32_t reserved_;
    int64_t prefetch_used;      /* prefetched experts that a layer then used (counted at their first use) */
    int64_t prefetch_wasted;    /* prefetched experts evicted before any layer used them (the overfetch the
                                   feedback loop of paper Sec. 3.2.2 reacts to) */
    int64_t miss_copies;        /* priority copies (misses, and prefetches a layer caught still in the queue) */
    int64_t miss_copy_bytes;
    double miss_copy_seconds;   /* summed time from a priority copy's request to its completion: miss_copy_bytes /
                                   miss_copy_seconds is the rate a miss sees while prefetches are queued */
    /* Prediction quality against look-ahead distance (the trend of paper Sec. 4.3): of the experts layer l really
     * used, how many had the look-ahead made j layers earlier named (predicted demand > 0)?  Index j-1. */
    int64_t pred_overlap_hits[EF_MAX_HORIZON];
    int64_t pred_overlap_total[EF_MAX_HORIZON];
    /* EF_FLAG_PROFILE only: summed event time, launches, algorithmic bytes (minimal HBM traffic the
     * operation needs: operands read once, results written once) and, for the matrix-core kernels,
     * algorithmic flops (2 per multiply-add of the contraction, padding rows not counted) per kind */
    double kernel_seconds[EF_K_COUNT];
    double kernel_bytes[EF_K_COUNT];
    int64_t kernel_launches[EF_K_COUNT];
    double kernel_flops[EF_K_COUNT];
} ef_stats;

/* ---- utilities (host only, no device needed) -------------------------------------------- */

const char *ef_strerror(int code);

/* bytes of one packed expert blob: 3*d*F*2; 0 if d % 64 or F % 32 is non-zero */
size_t ef_expert_bytes(int d_model, int d_ff);

/*
 * 4-bit experts.  The paper evaluates one model in GPTQ-Int4 form (Sec. 4.1) without stating a
 * format; here a weight is w = (q - 8) * s with a code q in 0..15 and one bf16 scale s per matrix
 * row and group of 128 inputs.  An expert blob of ef_expert_bytes_q4(d,F) = 3*d*F/2 + 3*d*F/64
 * bytes holds, in this order: for rb in 0..F/32-1, for kq in 0..d/64-1: the W1 "quad" of rows
 * [32rb, 32rb+32) and inputs [64kq, 64kq+64), then the W3 quad; for cb in 0..d/32-1, for kq in
 * 0..F/64-1: the W2 quad of rows [32cb, 32cb+32); the W1 / W3 scales [F/32][d/128][2][32] bf16;
 * the W2 scales [d/32][F/128][32] bf16.  A quad is 64 lanes x 4 dwords: dword j of lane
 * l = 32*g + i holds the eight codes of the operand fragment of k-step 4kq + j (natural order for
 * W1 / W3, paired order for W2, as in the bf16 blob), code t at bits 4*(t/2) + 16*(t%2).
 * The FFN kernels form (q - 8) * s in fp16 (relative error <= 2^-12 per weight) and run the matrix
 * cores in fp16 with fp32 accumulation: tokens are converted from bf16 to fp16 (exact for
 * 2^-14 <= |x| < 65504; larger magnitudes overflow) and the intermediate activations are kept in
 * fp16.  Requires d_model, d_ff and d_ff_shared multiples of 128; with a shared FFN its blob is a
 * 4-bit blob too (ef_pack_expert_q4 with d_ff_shared).  Groups of up to 7 token
 * tiles run through weight-streaming kernels that dequantise on the operand fragment; larger groups
 * (prefill) are first expanded to a 16-bit blob of the same fp16 values (q - 8) * s in a staging
 * area the context owns (one blob per expert that can reach that size in one call) and then run
 * through the tiled matrix-core kernels in fp16.
 */
size_t ef_expert_bytes_q4(int d_model, int d_ff);   /* 0 if d_model % 128 or d_ff % 128 is non-zero */

/* Pack codes q1, q3 [F,d], q2 [d,F] (one byte per code, 0..15) and scales s1, s3 [F, d/128],
 * s2 [d, F/128] (bf16 bit patterns), all row-major [host], into blob [host] in the layout above. */
int ef_pack_expert_q4(const uint8_t *q1, const uint16_t *s1, const uint8_t *q3, const uint16_t *s3,
                      const uint8_t *q2, const uint16_t *s2, int d_model, int d_ff, void *blob);

/* Pack row-major W1 [F,d], W3 [F,d], W2 [d,F] (bf16 bit patterns) [host] into blob [host],
 * ef_expert_bytes(d,F) bytes, in the layout described at the top.  Model-load-time helper.
 * EF_EINVAL if W2 holds a value that is not finite in fp16 (|w| >= 65536, inf, NaN). */
int ef_pack_expert(const uint16_t *W1, const uint16_t *W3, const uint16_t *W2,
                   int d_model, int d_ff, void *blob);

/* ---- context ---------------------------------------------------------------------------- */

/* Allocates the slot pool (slots_total * ef_expert_bytes), scratch for max_tokens tokens, the copy
 * streams, one side stream for compute and the events.  With EF_FLAG_FAKE_COPY nothing touches the GPU. */
int ef_create(const ef_config *cfg, ef_ctx **out);
int ef_destroy(ef_ctx *ctx);
const char *ef_last_error(ef_ctx *ctx);

/* Register one layer.  gate_w [dev] [E,d] bf16 row-major; gate_b [dev] [E] f32 or NULL;
 * experts [pinned] E consecutive packed blobs (the authoritative copy; must outlive the context;
 * with EF_FLAG_FAKE_COPY any non-NULL value); shared_blob [dev] packed blob of the dense SwiGLU
 * with hidden d_ff_shared (in the context's weight format: bf16 or 4-bit), or NULL.  The library
 * keeps the pointers, it copies nothing. */
int ef_register_layer(ef_ctx *ctx, int layer, const void *gate_w, const float *gate_b,
                      const void *experts, const void *shared_blob);

/* ---- hot path ---------------------------------------------------------------------------- */

/*
 * Cross-layer prediction (pre-gating, paper Sec. 2.3.2 / 3.2.1, with the deviation Delta of
 * Sec. 3.2.2): the hidden states of `layer` go through the gates of layers layer+1..layer+H.
 * For j = 1..H: z = hidden * Wg_{layer+j}^T + b;  score = z + beta*resident_{layer+j} + Delta_j;
 * topk_ids[j-1][t][:] = the k best experts of token t in ascending id (ties: lower id);
 * hist[j-1][e] = number of (token, slot) assignments to e.  Residency is the cache state at call
 * time.  Layers past the last one are not predicted: H is clamped to n_layers-1-layer and the
 * effective H is returned in *H_eff (may be 0: nothing enqueued).
 *   hidden   [dev]  [T,d] bf16 row-major
 *   delta    [dev]  [R,H,E] f32 or NULL;  tok2req [dev] [T] i32 request of each token or NULL (=0)
 *   topk_ids [dev]  [H,T,k] i32;  hist [dev] [H,E] i32 (overwritten)
 */
int ef_predict(ef_ctx *ctx, int layer, const void *hidden, int T, int H,
               const float *delta, const int32_t *tok2req, float beta,
               int32_t *topk_ids, int32_t *hist, int *H_eff, void *stream);

/*
 * Cache-aware routing of one layer (paper Sec. 3.4; fallback "top-k of the router logits",
 * Sec. 3.2.2): z = hidden * Wg^T + b; p = softmax(z) over all E; selection score z + beta*resident;
 * top-k as in ef_predict; topk_w[t][j] = p[t][ids[t][j]] (unbiased), renormalised over the k if
 * renorm_topk, times routed_scale.  Then the stable grouping of the assignments a = t*k + j by
 * expert: counts[e], offsets (exclusive prefix, offsets[E] = T*k), perm[pos] = a, inv_perm[a] = pos.
 * All outputs [dev]: topk_ids [T,k] i32, topk_w [T,k] f32, counts [E] i32, offsets [E+1] i32,
 * perm [T*k] i32, inv_perm [T*k] i32.  T = 0 is allowed (counts/offsets are zeroed).
 */
int ef_route(ef_ctx *ctx, int layer, const void *hidden, int T, float beta,
             int32_t *topk_ids, float *topk_w, int32_t *counts, int32_t *offsets,
             int32_t *perm, int32_t *inv_perm, void *stream);

/*
 * ef_route for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same kernels and bit-identical results, but the kernels'
 * scratch (per-tile expert counts and their prefixes, partial logits of K-split gate launches) is a static
 * device array of EF_ROUTE_STATIC_SCRATCH_BYTES inside the library instead of buffers of the context; every
 * GPU the library runs on holds that array until the process ends.  The call allocates nothing, on the host
 * side of HIP or on the device, and calls no allocating routine.  T above EF_ROUTE_STATIC_MAX_TOKENS is
 * EF_EINVAL (T beyond the context's max_tokens is fine: this call does not use the context's scratch).
 * All calls on one GPU, of any context, share the one array: calls that overlap in time on that GPU (different
 * streams, different contexts) race; issue them on one stream or order them with events.  Nothing has to be
 * cleared between calls.  Arguments as ef_route.
 */
#define EF_ROUTE_STATIC_MAX_TOKENS 8192
#define EF_ROUTE_STATIC_SCRATCH_BYTES (4u << 20)
int ef_route_static(ef_ctx *ctx, int layer, const void *hidden, int T, float beta,
                    int32_t *topk_ids, float *topk_w, int32_t *counts, int32_t *offsets,
                    int32_t *perm, int32_t *inv_perm, void *stream);

/*
 * ef_route and ef_predict of the same layer on ONE pass over `hidden` (the look-ahead gates see the
 * same hidden states as the layer's own gate, paper Sec. 2.3.2, so the hidden states need to be read
 * from HBM only once).  Results are identical to calling ef_route(layer, ..., beta) and
 * ef_predict(layer, ..., H, delta, tok2req, beta) one after the other; arguments as there
 * (pred_ids [dev] [H,T,k], pred_hist [dev] [H,E]).
 */
int ef_route_predict(ef_ctx *ctx, int layer, const void *hidden, int T, float beta, int H,
                     const float *delta, const int32_t *tok2req,
                     int32_t *topk_ids, float *topk_w, int32_t *counts, int32_t *offsets,
                     int32_t *perm, int32_t *inv_perm,
                     int32_t *pred_ids, int32_t *pred_hist, int *H_eff, void *stream);

/*
 * Grouped SwiGLU expert FFN over the cache slots and weighted un-permute:
 * out[t] = sum_j topk_w[t][j] * FFN_{ids[t][j]}(hidden[t]) (+ dense shared FFN(hidden[t])).
 * Groups whose expert is ready run first; groups whose expert is still being copied run after
 * their copy event; experts not resident at all are swapped in here at miss priority (unless
 * EF_FLAG_STRICT_RESIDENT) while the resident groups compute.  counts_host [host] [E] is the
 * caller's host copy of `counts` (launch planning and cache decisions).  out [dev] [T,d] f32.
 * Advances the cache clock by one layer.
 */
int ef_moe_ffn(ef_ctx *ctx, int layer, const void *hidden, int T,
               const int32_t *topk_ids, const float *topk_w, const int32_t *counts_host,
               const int32_t *offsets, const int32_t *perm, const int32_t *inv_perm,
               float *out, void *stream);

/*
 * Make (layer, expert) resident in the HBM cache: pick a slot (free, else the two-level LRU's
 * victim: low tier first, paper Sec. 3.3.1) and queue the copy of the blob from the pinned store.
 * priority 0 = prefetch, due_in = layers until it is needed; priority 1 = miss of the layer being
 * run (due_in ignored).  An expert already resident is only promoted.  *slot_out (may be NULL)
 * receives the slot.  Returns EF_EBUSY if no slot can be evicted.
 *
 * Copies go over one link, so the library keeps one queue (paper Sec. 3.4: miss resolution gets the
 * highest priority in the memory queue): a worker thread of the context hands the copies to the copy
 * stream in chunks of at most copy_chunk_mib, at most copy_depth chunks ahead, and always takes the
 * oldest priority-1 copy before any prefetch; a prefetch a layer needs while it is still queued is
 * promoted.  The call itself returns at once.
 */
int ef_cache_swap_in(ef_ctx *ctx, int layer, int expert, int priority, int due_in, int *slot_out);

/* resident_host [host] [E]: 1 if the expert is in the cache (ready or copy in flight) */
int ef_cache_query(ef_ctx *ctx, int layer, uint8_t *resident_host);

/*
 * Horizon controller (paper Sec. 3.2.1): from the predicted histograms hist_host [host] [H,E] of
 * layers layer+1..layer+H, take experts in descending demand until their cumulative share reaches
 * cum_threshold (N_e); N_miss = those not resident; S = clamp(ceil(N_miss*E_s/(C_s*T_l)), 1, h_max)
 * with the current C_s and T_l estimates, further moved by the stall / overfetch feedback counters
 * (Sec. 3.2.2).  *H_next receives S; prefetch_list [host] [H*E] receives (j << 16 | expert) for the
 * non-resident experts of the first min(H,S) look-ahead layers, nearest layer first, in descending
 * demand; *n_prefetch their number.  Also re-tiers the cache for the new S.
 */
int ef_choose_horizon(ef_ctx *ctx, int layer, const int32_t *hist_host, int H, int T,
                      int *H_next, int32_t *prefetch_list, int *n_prefetch);

/*
 * One whole layer of the method in one call (Sec. 3.1 overview, 3.2, 3.3.2, 3.4):
 * ef_route_predict with look-ahead H (H < 0: the controller's current horizon) into library-owned
 * buffers; the grouping kernel hands counts and demand histograms to the host through host-mapped
 * memory and the call polls for them instead of synchronising the stream; ef_moe_ffn (enqueued first:
 * the GPU is idle until then); ef_choose_horizon; one ef_cache_swap_in(prefetch) per entry of its list
 * (EF_EBUSY skips that prefetch), whose copies overlap the FFN that is running by then.
 * Results are those of the separate calls made in that order.  *H_next (may be NULL) receives the horizon chosen for the
 * next layer, counts_host_out [host] [E] (may be NULL) the per-expert token counts.  out [dev]
 * [T,d] f32 is valid after the caller synchronises `stream`.  The call blocks the host until the
 * routing kernels of this layer have finished (not until the FFN has).  T must be positive.
 */
int ef_layer_step(ef_ctx *ctx, int layer, const void *hidden, int T, float beta, int H,
                  const float *delta, const int32_t *tok2req, float *out, int *H_next,
                  int32_t *counts_host_out, void *stream);

/*
 * Intra-batch diversity of the tokens of one iteration (paper Sec. 2.2, equation of Dist(t)): the sum
 * over token pairs of the Euclidean distance between their embeddings, the runtime signal the paper
 * names for the initial step size (Sec. 2.3.1, 3.1).  hidden [dev] [T, d_model] bf16 row-major, 16-byte
 * aligned, 1 <= T <= max_tokens.  tok_dist [dev] [T] f32 (may be NULL) receives per token j the sum of
 * ||v_i - v_j||_2 over the earlier tokens i < j; *dist [dev] f64 their total Dist(t).  fp32 inner
 * products on the matrix cores, fp64 final sums in a fixed order (bit-reproducible).  Enqueues on
 * `stream` only and uses the context's FFN scratch: not concurrent with ef_moe_ffn / ef_layer_step
 * of the same context on another stream.  EF_EINVAL when T*top_k*d_model floats of scratch cannot
 * hold the T*ceil(T/64) partial sums.
 */
int ef_token_dist(ef_ctx *ctx, const void *hidden, int T, float *tok_dist, double *dist, void *stream);

/* -------------------------------------------------------------------------------------------------
 * Deviation predictor (paper Sec. 3.2.2 "Cross-Layer Prediction and Delta Adjustment", 3.2.3-3.2.5).
 * Host code only (the paper runs this model on the CPU, asynchronously to the GPU kernels); all
 * pointers below are host pointers.  The model is a random-forest regressor over activation logs: one
 * example per (request, layer), features x = [e, S, l, prev_act] of length d_emb + 2 + L*M (Sec. 3.2.4),
 * label y in {0,1}^M, squared-error criterion (Sec. 3.2.5).  Its prediction for a future layer becomes
 * the `delta` rows of ef_predict / ef_route_predict / ef_layer_step.
 * ------------------------------------------------------------------------------------------------- */
typedef struct ef_forest ef_forest;

typedef struct {
    int n_features;       /* F = d_emb + 2 + L*M                                                  */
    int n_outputs;        /* M experts per layer, 1..EF_MAX_EXPERTS                               */
    int n_trees;          /* >= 1                                                                  */
    int max_depth;        /* >= 1: a tree has at most 2^max_depth leaves                           */
    int min_samples_leaf; /* >= 1                                                                  */
    int n_threads;        /* trees are grown / evaluated in parallel; 0 = all hardware threads     */
} ef_forest_config;

int ef_forest_create(const ef_forest_config *cfg, ef_forest **out);
int ef_forest_destroy(ef_forest *f);

/*
 * Sec. 3.2.4: feature vector of one (request, layer).  emb_table [V, d_emb] f32 row-major is the fixed
 * random embedding table, token_ids [n_tok] (each in 0..V-1) the request's tokens; e = their mean row
 * (summed in sequence order in fp64, rounded to f32).  prev_act [L*M] u8 holds, layer-major, the
 * experts the request activated in the layers before `layer` (the caller leaves the rest zero).
 * x [d_emb + 2 + L*M] f32 receives [e, S, layer, prev_act].
 */
int ef_delta_features(const float *emb_table, int V, int d_emb, const int32_t *token_ids, int n_tok,
                      int S, int layer, const uint8_t *prev_act, int L, int M, float *x);

/*
 * Sec. 3.2.5: grow the forest.  X [N, F] f32 row-major, Y [N, M] u8 (0/1).  bootstrap [n_trees, N]
 * i32 holds, per tree, the indices (0..N-1, with repetitions) of the samples it is grown on: the random
 * draws are the caller's; NULL grows every tree on all N samples.  Every feature is considered at
 * every node (the regressor default of the library the paper names).  A split maximises
 * sum_m sL[m]^2/nL + sum_m sR[m]^2/nR over the node's samples (equivalently minimises the summed
 * squared error), decided in exact integer arithmetic; ties go to the lower feature index, then the
 * lower threshold; a node stays a leaf unless the best split strictly improves on it, both sides keep
 * min_samples_leaf samples and its depth is below max_depth.  Threshold = midpoint of the two
 * neighbouring feature values (fp64); x <= threshold goes left.  Deterministic for given inputs,
 * whatever n_threads.  Replaces a previously fitted model.  1 <= N <= 2^20; every feature value finite
 * (EF_EINVAL otherwise).
 */
int ef_forest_fit(ef_forest *f, const float *X, const uint8_t *Y, int N, const int32_t *bootstrap);

/* Y_hat [n, M] f64 = mean over the trees (summed in tree order) of the leaf means.  EF_EINVAL before a fit. */
int ef_forest_predict(const ef_forest *f, const float *X, int n, double *Y_hat);

/*
 * Inspection (tests, serialisation).  ef_forest_tree_size: number of nodes of tree t (negative error code
 * on failure).  ef_forest_tree_export copies the nodes in creation order (node 0 is the root; children are
 * created left subtree first): feature [nodes] i32 (-1 = leaf), threshold [nodes] f64, left / right
 * [nodes] i32 (-1 at leaves), count [nodes] i32 (samples, repetitions counted), value [nodes, M] f64
 * (mean label).  Any output pointer may be NULL.
 */
int ef_forest_tree_size(const ef_forest *f, int t);
int ef_forest_tree_export(const ef_forest *f, int t, int32_t *feature, double *threshold, int32_t *left,
                          int32_t *right, int32_t *count, double *value);

/* Sec. 3.2.5: share of expert bits predicted correctly, a bit being predicted set when y_hat >= 0.5. */
int ef_forest_bit_accuracy(const double *Y_hat, const uint8_t *Y, int n, int M, double *accuracy);

/*
 * The deviation added to the pre-gate logits (Sec. 3.2.2): delta[r, e] = gain * (y_hat[r, e] - mean_e
 * y_hat[r, .]) as f32 (the mean summed in expert order in fp64).  A constant per row does not change a
 * top-k, so only the centred prediction matters; the paper does not give the mapping (a reading).
 */
int ef_delta_from_activation(const double *Y_hat, int n_rows, int M, float gain, float *delta);

/*
 * Sec. 3.2.2's prediction cache and the asynchronous producer that fills it.  A prediction is keyed
 * by (token id sequence, layer, step size S) and holds the forest's y_hat [M] for that request and
 * layer; beyond `capacity` entries the least recently used one leaves (a hit refreshes its entry).
 * ef_delta_cache_get returns 1 on a hit (y_hat copied out), 0 on a miss: the caller then uses a zero
 * delta row, i.e. plain top-k of the router logits, the fallback the section names.  All calls are
 * thread-safe.
 */
typedef struct ef_delta_cache ef_delta_cache;
int ef_delta_cache_create(int capacity, int M, ef_delta_cache **out);
int ef_delta_cache_destroy(ef_delta_cache *c);
int ef_delta_cache_put(ef_delta_cache *c, const int32_t *token_ids, int n_tok, int layer, int S, const double *y_hat);
int ef_delta_cache_get(ef_delta_cache *c, const int32_t *token_ids, int n_tok, int layer, int S, double *y_hat);
int ef_delta_cache_counts(ef_delta_cache *c, long long *hits, long long *misses, long long *entries);

/*
 * Producer: n_threads worker threads evaluate the forest for submitted (request, layer) pairs and put the
 * result into the cache, so the GPU loop never waits for the model.  The forest, the cache and the embedding
 * table must outlive the producer and the forest must not be refitted while it runs.  ef_delta_submit copies
 * its arguments, enqueues one job per layer in [layer_first, layer_first + n_layers) that is below L and not
 * yet cached, and returns at once.  prev_act [L*M] u8, layer-major: what the request has activated so far;
 * for target layer t only the rows of layers < t - S enter the features (what is known when layer t is
 * predicted S layers ahead, so that training examples built with the same rule see the same inputs), later
 * rows count as zero.  ef_delta_drain blocks until the queue is empty and the workers are idle.
 */
typedef struct ef_delta_producer ef_delta_producer;
int ef_delta_producer_create(const ef_forest *f, ef_delta_cache *cache, const float *emb_table, int V, int d_emb,
                             int L, int M, int n_threads, ef_delta_producer **out);
int ef_delta_producer_destroy(ef_delta_producer *p);
int ef_delta_submit(ef_delta_producer *p, const int32_t *token_ids, int n_tok, int S, int layer_first,
                    int n_layers, const uint8_t *prev_act);
int ef_delta_drain(ef_delta_producer *p);

/*
 * Assemble the delta argument of one predict call from the cache: for request r (token ids
 * token_ids[tok_off[r] .. tok_off[r+1])) and look-ahead j = 0..H-1 the row delta[r, j, .] [E = M] f32 is
 * ef_delta_from_activation of the cached prediction for layer `layer + 1 + j` and step size S, or zeros on
 * a miss / past the last layer.  delta [R, H, M] (host; pinned or host-mapped memory lets the caller hand it
 * to the device without a staging copy).  *n_hits (may be NULL) receives the number of rows found.
 */
int ef_delta_assemble(ef_delta_cache *c, const int32_t *token_ids, const int32_t *tok_off, int R, int layer,
                      int S, int H, int L, float gain, float *delta, int *n_hits);

/*
 * Inspection of the last ef_layer_step (tests, activation logging; cites no passage of the paper): synchronises
 * `stream`, then copies the routing state that call left in library-owned device buffers into host arrays.
 * Any pointer may be NULL.  topk_ids [T,k] i32, topk_w [T,k] f32, offsets [E+1] i32, perm / inv_perm [T*k] i32,
 * pred_ids [H_eff,T,k] i32 and pred_hist [H_eff,E] i32 (the demand histograms as the host received them),
 * with T and H_eff those of that call; *T_out / *H_eff_out (may be NULL) receive them.  EF_EINVAL before the
 * first ef_layer_step.
 */
int ef_layer_step_fetch(ef_ctx *ctx, int32_t *topk_ids, float *topk_w, int32_t *offsets, int32_t *perm,
                        int32_t *inv_perm, int32_t *pred_ids, int32_t *pred_hist, int *T_out, int *H_eff_out,
                        void *stream);

/*
 * Launch-shape tuning: which kernel form a group takes and how launches are split.  For sweeps and for tests
 * that force one kernel form; cites no passage of the paper.  No setting changes what is computed, only the
 * order in which partial sums over K slices are added.  ef_create installs the defaults (the measured best);
 * ef_set_tuning rejects values outside the ranges below with EF_EINVAL and changes nothing then.  "0 = auto"
 * fields let the library choose per launch.  Nothing in the library reads environment variables.
 */
typedef struct ef_tuning {
    int32_t tiled;                   /* 0/1: groups of many token tiles may take the matrix-core tiled kernels (1) */
    int32_t tiled_min_tiles;         /* 8..4096: routed groups take them from this many 32-token tiles on (10) */
    int32_t tiled_min_up_wgs;        /* >= 1: ... and only if the tiled first-half launch has this many workgroups (1) */
    int32_t tiled_min_down_wgs;      /* >= 1: ... and the second-half launch this many (1) */
    int32_t tiled_xcd_rotation;      /* 0/1: deal every group's weight-panel blocks from the least loaded XCD (1) */
    int32_t overlap_tiled;           /* 0/1: a phase's tiled launches run on a side stream beside its streamed ones (1) */
    int32_t sort_groups;             /* 0/1: groups with the most work first in a launch (1) */
    int32_t passes_of_four;          /* 0/1: streamed groups of >= 3 token tiles take passes of four tiles (1) */
    int32_t lds_shared;              /* 0/1: ... through the kernels whose waves share fragments in LDS (1) */
    int32_t lds_shared_occupancy;    /* workgroups per compute unit of those kernels: 1, 2, or 0 = two only beside a tiled
                                        launch that covers every compute unit (0) */
    int32_t up_want_waves;           /* >= 1: the streamed first half splits K inside a workgroup below this many waves (640) */
    int32_t up_k_slices;             /* 0 = auto, else 1, 2 or 4 */
    int32_t down_want_wgs;           /* 0 = auto (256; 512 for the LDS-shared kernels), else >= 1: target of the K-slice split */
    int32_t down_k_slices;           /* 0 = auto, else 1..8: K-slice planes of the second half (both launches) */
    int32_t down_slices_by_longest_k; /* 0/1: the tiled second half sizes its slices by the group with the longest K (1) */
    int32_t down_split_slice_counts; /* 0/1: the streamed and the tiled launch of a layer choose their slice counts separately (1) */
    int32_t gate_k_split;            /* 0 = auto, else 1..16: workgroups sharing the K range of one (tile, gate group) */
    int32_t gate_token_split;        /* 0/1: the gate's second step may split a tile's tokens over workgroups (1) */
    int32_t gate_fused_finish;       /* 0/1: decode-sized batches fuse the gate's second step with the grouping (1) */
    int32_t gate_stream;             /* 0/1: batches of many token tiles take the gate kernel that streams through LDS (1) */
    int32_t early_pack;              /* 0/1: ef_layer_step enqueues the token packing before the host has the counts (1) */
    int32_t copy_chunk_mib;          /* 1..1024: expert copies go to the link in chunks of at most this many MiB; a miss
                                        overtakes queued prefetches at the next chunk boundary (32) */
    int32_t copy_depth;              /* 1..8: chunks handed to the copy stream ahead of the one in transfer (2) */
    int32_t down_tail_split;         /* 0/1: a streamed second half of a little more than one round of workgroups over
                                        the compute units takes twice the K slices (1) */
    int32_t tiled_tail_slices;       /* a tiled second half of more than 256 workgroups cuts its last group into K slices
                                        that fill the launch's last, partly empty round: 0 = never, 1 = as many as a
                                        model of the launch finds best, 2 / 4 / 8 = that many (1) */
    int32_t dist_form;               /* ef_token_dist: 0 = by batch size (up to 256 tokens: differences summed directly,
                                        no Gram matrix), 1 = Gram blocks of 128 x 256 fed from registers, 2 = Gram blocks
                                        of 256 x 256 staged through LDS; 1 and 2 give the same bits (0) */
} ef_tuning;
int ef_get_tuning(ef_ctx *ctx, ef_tuning *out);
int ef_set_tuning(ef_ctx *ctx, const ef_tuning *t);

/* Statistics; synchronises outstanding timing events first (not for the hot loop). */
int ef_get_stats(ef_ctx *ctx, ef_stats *out);
int ef_reset_stats(ef_ctx *ctx);

/* Choose at run time which kernel kinds are bracketed with events: bit (1 << EF_K_*) per kind,
 * 0 = none (overrides the EF_FLAG_PROFILE* flags given at creation). */
int ef_set_profile(ef_ctx *ctx, unsigned kinds_mask);

/* Bracket only every `every`-th launch of each selected kind (default 1 = all).  An event record between two
 * kernels costs the stream a bubble of 2-3 us; a sample of the launches gives the same average duration
 * while the run being measured stays close to an unmeasured one.  Launch counts, times, bytes and flops in
 * ef_stats then cover the sampled launches only. */
int ef_set_profile_sampling(ef_ctx *ctx, int every);

/* Measured ceilings of the context's device, for the roofline figures of a benchmark (not a step of the method: the
 * paper's Sec. 4 reports throughput only; a roofline needs to know what the part delivers to any kernel).
 *   EF_PEAK_HBM_READ:   a plain streaming read of `bytes` bytes at `buf` (device memory, 16-byte aligned, a multiple of
 *                       8 MiB; use more than the 256 MiB the caches hold), `reps` times after one untimed pass; GB/s.
 *   EF_PEAK_MFMA_16BIT: a loop of 32x32x16 bf16 matrix-core instructions on registers, on every SIMD; TFLOP/s
 *                       (`buf`, `bytes` ignored).
 * Synchronous: enqueues on `stream`, times with events and waits.  Uses the routing scratch of the context: not to be
 * called while a routing call of the same context is in flight.  EF_EINVAL on bad arguments, EF_ENOSYS in fake-copy
 * contexts. */
#define EF_PEAK_HBM_READ 0
#define EF_PEAK_MFMA_16BIT 1
int ef_measure_peak(ef_ctx *ctx, int what, const void *buf, size_t bytes, int reps, double *result, void *stream);

/* Fake-copy contexts only: advance the fake clock; copies complete after bytes/bandwidth seconds. */
int ef_fake_advance_time(ef_ctx *ctx, double seconds);

#ifdef __cplusplus
}
#endif
#endif /* EXPERTFLOW_H */
