/*
 * libbaklava -- ragged per-head KV-cache decode path for AMD MI355X (gfx950).
 *
 * The method (BaKlaVa, arXiv 2502.13176) gives every (layer, KV head) cache its
 * own token budget from a one-time importance profile, so at decode time each
 * head's cache has a different length.  This library holds the part of that
 * method that runs once per generated token:
 *
 *   host, once      per-cache budgets from importance scores
 *   device, per step  append the new K/V row, single-query attention over every
 *                     ragged cache, optional accumulation of attention weights
 *   device, every few steps  eviction down to each cache's own budget
 *
 * Plain C ABI: pointers and sizes only.  Every pointer is marked HOST or DEVICE.
 * All functions return a status code (0 = BAKLAVA_OK); nothing aborts, throws or
 * prints.  Device entry points enqueue work on the caller's stream and return
 * without synchronising.  The caller owns every byte of device memory; the
 * library allocates only small host-side structures inside baklava_ctx.
 *
 * Notation: L layers, Hkv KV heads, G = Hq/Hkv query heads per KV head (query
 * head hq reads KV head hq / G), D head dimension, `batch` sequences.
 * Cache id  c = (layer * batch + b) * Hkv + h  (layer-major).
 * Budget id i = layer * Hkv + h  (budgets are a property of the model, the same
 * for every sequence).
 */
#ifndef BAKLAVA_H
#define BAKLAVA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  BAKLAVA_OK = 0,
  BAKLAVA_EINVAL = 1,      /* null pointer, bad shape / dtype / option, misaligned pointer          */
  BAKLAVA_EINFEASIBLE = 2, /* budgets cannot be met: m*lo > B, m*hi < B, budget < sink + recent     */
  BAKLAVA_ECAPACITY = 3,   /* an append would exceed a cache's capacity; workspace too small        */
  BAKLAVA_EHIP = 4,        /* a HIP runtime call failed; see baklava_last_hip_error()               */
  BAKLAVA_ESTATE = 5,      /* call order violated, e.g. attention over an empty cache               */
  BAKLAVA_ENOMEM = 6       /* a host-side allocation of the library failed                          */
};

enum { BAKLAVA_BF16 = 0, BAKLAVA_F32 = 1 };
enum { BAKLAVA_POLICY_SCORE = 0, BAKLAVA_POLICY_STREAMING = 1 };

/* Static text for a status code. */
const char* baklava_strerror(int status);
/* hipError_t value of the last failed HIP call made by this library on the calling thread. */
int baklava_last_hip_error(void);

/* ------------------------------------------------------------------------------------------
 * Host only.  No GPU is touched; usable on a machine without one.
 * ------------------------------------------------------------------------------------------ */

/*
 * Budgets proportional to importance, clipped to [lo, hi] and rounded so that they sum to
 * global_budget exactly.  This rule is not the paper's (its own allocation is Algorithm 2 below; its
 * principle, Methods, "Assigning Memory Budgets to KV-Caches", is only that more important caches
 * get more memory): it is the allocator the benchmark workloads ask for, made integer-only:
 *   w_i = max(1, floor(I_i / max(I) * 2^40)),  x_i(lam) = floor(lam * w_i / 2^40),
 *   lam = largest integer with sum_i clip(x_i) <= B,  b_i = clip(x_i(lam)),
 *   leftover tokens go one each to heads with lo <= x_i < hi in decreasing order of
 *   (lam*w_i mod 2^40, w_i, lower index first).
 * importance  HOST [m], finite and > 0.   budget_out  HOST [m].
 * Errors: EINVAL (null, m <= 0, lo < 0, hi < lo, non-finite or non-positive importance),
 *         EINFEASIBLE (m*lo > global_budget or m*hi < global_budget).
 */
int baklava_alloc_proportional(const double* importance, int32_t m, int64_t global_budget,
                               int32_t lo, int32_t hi, int32_t* budget_out);

/*
 * Algorithm 2 (KV-cache memory reallocation based on attention-head importance): caches with
 * importance < t shrink by floor(r * size); the freed tokens are shared by the
 * k = min(n, m - n) most important of the other caches (n = number shrunk), floor(F/k) each and
 * the remainder one apiece to the most important first.  No cache below t, or all below t:
 * output equals input.  Increased sizes are not clipped.
 * importance HOST [m], size_in HOST [m], budget_out HOST [m] (may alias size_in).
 * Errors: EINVAL (null, m <= 0, r outside [0,1], negative size, an importance or t that is not
 * finite: the algorithm orders importances and compares them with t).
 */
int baklava_alloc_threshold(const double* importance, int32_t m, const int32_t* size_in,
                            double t, double r, int32_t* budget_out);

/*
 * Arena layout replacing the per-head cache object of the paper's implementation (Methods: the
 * method is implemented as a custom KV-cache object initialised once with the found budgets): cache
 * c gets capacity budget[layer*Hkv+h] + slack rows at
 * token offset off[c] = sum of the capacities before it.
 * budget HOST [L*Hkv];  off_out HOST int64 [L*batch*Hkv];  cap_out HOST int32 [L*batch*Hkv];
 * total_tokens_out HOST scalar = rows each arena plane must hold.
 * Errors: EINVAL (null, non-positive shape, negative budget or slack, capacity overflow of int32).
 */
int baklava_layout(const int32_t* budget, int32_t L, int32_t Hkv, int32_t batch, int32_t slack,
                   int64_t* off_out, int32_t* cap_out, int64_t* total_tokens_out);

/*
 * Split-K schedule for decode attention over ragged caches: every cache is cut over its whole
 * capacity into runs of `chunk` rows (the kernels clamp a run to the live length, so the table
 * depends on capacities only).  The table is written in launch order, long caches first:
 * inside each layer when whole_model == 0 (a layer range is then a contiguous slice), over all
 * layers when whole_model == 1.  Partial slots are numbered cache by cache, so cache c owns the
 * `nsplit` consecutive slots that start at the slot of its first run.
 * With target_items > 0 a launch unit (each layer when whole_model == 0, the whole model
 * otherwise) that would have more than max(target_items, caches in the unit) work items gets
 * longer runs: the smallest multiple of 64 that brings it to that many items -- e.g. one
 * workgroup per compute unit, so that a launch is one even wave of workgroups -- after which the
 * runs inside each cache are made equal (rounded up to 64 rows) without adding an item.  A run
 * never exceeds 2^22 rows, whatever the target.
 * off_host HOST int64 [L*caches_per_layer], cap_host HOST int32 [same]; chunk a multiple of 64,
 * >= 256; items_out HOST [max_items] or NULL (count only); n_items_out HOST scalar.
 * Errors: EINVAL, ECAPACITY (more than max_items work items; n_items_out still receives the count).
 */
typedef struct {
  int32_t cache, start, count, slot;  /* rows [start, start+count) of `cache`; partial slot      */
  int32_t nsplit;                     /* work items of this cache                                */
  int32_t reserved;
  int64_t row0;                       /* arena row of `start`: off[cache] + start                */
} baklava_work_item;
int baklava_plan_schedule(const int64_t* off_host, const int32_t* cap_host, int32_t L,
                          int32_t caches_per_layer, int32_t chunk, int32_t target_items,
                          int32_t whole_model, int64_t max_items, baklava_work_item* items_out,
                          int64_t* n_items_out);

/* ------------------------------------------------------------------------------------------
 * Device.
 *
 * Calls that only enqueue kernels on the caller's stream (safe inside a stream capture):
 * baklava_reset, baklava_append, baklava_decode_attn, baklava_append_decode_attn (its token
 * position and its capacity check are then those of the capture; baklava_append_decode_attn_replay
 * is the variant made for replay), baklava_flush_scores, baklava_compact, and the one-time passes
 * further down.  Set-up calls that synchronise or copy synchronously and therefore must stay
 * outside a capture: baklava_create, baklava_set_option with the CHUNK_*, TARGET_* and
 * TILED_SELECT_ROWS options (they rebuild and upload a table after a device-wide synchronisation),
 * baklava_set_lengths, baklava_sync_lengths, baklava_profile_read.  The stream arguments are
 * hipStream_t handles passed as void* so that this header needs no HIP header.
 * ------------------------------------------------------------------------------------------ */

typedef struct baklava_ctx baklava_ctx;

typedef struct {
  int32_t L, Hq, Hkv, D, batch;
  int32_t dtype;          /* BAKLAVA_BF16 or BAKLAVA_F32: element type of k, v and of q / k_new / v_new */
  int32_t sink, recent;   /* rows at the front / back of a cache that eviction never removes        */
  int32_t policy;         /* BAKLAVA_POLICY_*                                                        */
  int32_t track_scores;   /* 1: attention calls add each token's attention weights to `score`; see
                             baklava_flush_scores for when the plane is up to date                  */
  void* k;                /* DEVICE [total_tokens, D] row-major, 16-byte aligned                     */
  void* v;                /* DEVICE [total_tokens, D]                                                */
  float* score;           /* DEVICE [total_tokens] accumulated attention per cached token            */
  int32_t* pos;           /* DEVICE [total_tokens] original sequence position of each cached token   */
  const int64_t* off;     /* DEVICE [n_caches] first row of cache c                                  */
  const int32_t* cap;     /* DEVICE [n_caches] rows cache c can hold                                 */
  int32_t* len;           /* DEVICE [n_caches] live rows of cache c (authoritative copy)             */
  const int32_t* budget;  /* DEVICE [L*Hkv]                                                          */
  void* workspace;        /* DEVICE scratch, 256-byte aligned, baklava_workspace_bytes() bytes       */
  size_t workspace_bytes;
} baklava_desc;

/*
 * Bytes of device workspace a context with this description needs (split partials, work-item
 * tables, kept-index lists, halo rows of the eviction move, the counters of the tile-by-tile
 * selection, and with track_scores the query rows and softmax normalisers of the attention calls
 * each cache has on record).  Pointer fields of `desc` are ignored.  cap_host HOST [n_caches],
 * budget_host HOST [L*Hkv].  Returns 0 on invalid arguments.
 */
size_t baklava_workspace_bytes(const baklava_desc* desc, const int32_t* cap_host,
                               const int32_t* budget_host);

/*
 * Creates a context.  The *_host arrays are copies of the device tables in `desc` (the library
 * keeps a host mirror of the lengths so that no call reads anything back from the device);
 * len_host may be NULL for all-empty caches, in which case the caller must have zeroed desc->len
 * or call baklava_reset.  Writes the work-item table into the workspace with a synchronous copy.
 * Supported shapes: D in {64, 128}; Hq a multiple of Hkv with Hq/Hkv <= 16 (<= 8 for F32);
 * sink, recent >= 0.
 * The arena must be packed the way baklava_layout lays it out: off_host[c] = sum of the capacities
 * of the caches before c (workspace planes that run parallel to the arena use the same offsets).
 * Errors: EINVAL (also: offsets that are not the packed prefix sums), EINFEASIBLE (some budget <
 * sink + recent under POLICY_SCORE, or < sink under POLICY_STREAMING), ECAPACITY (workspace_bytes
 * too small, or len > cap), ENOMEM, EHIP.
 */
int baklava_create(const baklava_desc* desc, const int64_t* off_host, const int32_t* cap_host,
                   const int32_t* len_host, const int32_t* budget_host, baklava_ctx** out);
int baklava_destroy(baklava_ctx* ctx);

/* Tuning knobs (tests sweep them; results must not depend on them beyond rounding order). */
enum {
  BAKLAVA_OPT_CHUNK_TOKENS = 1, /* shortest run of rows per split-K work item for launches over part of
                                   the layers (multiple of 64, >= 256); the item target below may
                                   lengthen it                                                        */
  BAKLAVA_OPT_KERNEL = 2,       /* 0 = automatic, 1 = vector-ALU kernel, 2 = MFMA kernel (bf16, D=128) */
  BAKLAVA_OPT_TIME_KERNEL = 3,  /* time every attention partial-kernel launch with a pair of HIP events
                                   (baklava_profile_read): 1 = recorded on the stream before and
                                   after the launch, 2 = carried by the kernel's own dispatch (MFMA
                                   kernel; the other kernel is timed as under 1), 0 = off.  ESTATE
                                   while timings taken in another mode are still unread.  A
                                   measurement aid: leave it off while a stream is being captured  */
  BAKLAVA_OPT_CHUNK_TOKENS_WHOLE = 4, /* the same for launches over all layers at once               */
  BAKLAVA_OPT_TARGET_ITEMS = 5, /* > 0: launches over part of the layers lengthen their runs, layer by
                                   layer, until a layer has at most this many work items; 0: off.
                                   Default: the device's number of compute units (one wave of
                                   workgroups) while a layer holds at most a quarter as many caches,
                                   otherwise five times that number, with a shortest run of 256 rows */
  BAKLAVA_OPT_TARGET_ITEMS_WHOLE = 6, /* the same for launches over all layers at once.  Default: five
                                   times the device's number of compute units                      */
  BAKLAVA_OPT_TRACK_SCORES = 7, /* 0: attention calls stop adding to the scores (calls already on
                                   record stay there until the next flush); 1: they resume.  Only a
                                   context created with track_scores can be switched to 1          */
  BAKLAVA_OPT_TILED_SELECT_ROWS = 8 /* eviction: caches whose capacity exceeds this many rows are ranked
                                   by several workgroups (tiles of 8192 rows) instead of one.
                                   >= 8192; default 36864, or 8192 for a context of fewer than 512
                                   caches.  Synchronises like the CHUNK options                   */
};
int baklava_set_option(baklava_ctx* ctx, int32_t option, int64_t value);

/* Empties every cache: device len <- 0 (fill kernel on `stream`), host mirror <- 0. */
int baklava_reset(baklava_ctx* ctx, void* stream);

/*
 * Declares the live lengths after the caller has filled arena rows itself (a prefill).
 * len_host HOST [n_caches]; copied to the device table on `stream` and to the host mirror.
 * Errors: EINVAL, ECAPACITY (len > cap).
 */
int baklava_set_lengths(baklava_ctx* ctx, const int32_t* len_host, void* stream);

/*
 * Appends the current token's key and value row to every cache of layers
 * [layer_begin, layer_begin + layer_count) -- the concatenations [K'; K_t], [V'; V_t] of Eq. 7.
 * The row's score starts at 0 and its pos is token_pos.
 * k_new, v_new DEVICE [layer_count, batch, Hkv, D] in the context's dtype, 16-byte aligned.
 * Errors: EINVAL, ECAPACITY (some cache of the range is full; nothing is enqueued).
 */
int baklava_append(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count, const void* k_new,
                   const void* v_new, int32_t token_pos, void* stream);

/*
 * Single-query attention over the reduced caches (Eq. 7, i.e. Eq. 1 with one query row per
 * head and the evicted rows absent) for layers [layer_begin, layer_begin + layer_count):
 *   out[hq] = softmax(q[hq] . K_c^T / sqrt(D)) V_c,  c = the cache of KV head hq / G.
 * q   DEVICE [layer_count, batch, Hq, D] in the context's dtype, 16-byte aligned.
 * out DEVICE [layer_count, batch, Hq, D] fp32, fully overwritten.
 * With track_scores, score[j] += sum over the G query heads of the softmax weight of row j; the
 * addition may be deferred to a later attention call over the same layer (baklava_flush_scores).
 * Accumulation is fp32 throughout.
 * Errors: EINVAL, ESTATE (a cache in range is empty).
 */
int baklava_decode_attn(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count,
                        const void* q, float* out, void* stream);

/*
 * baklava_append followed by baklava_decode_attn over the same layer range, as one kernel
 * launch: the whole of Eq. 7 for one decode step -- the new row joins each cache, then the query
 * attends over [K'; K_t], [V'; V_t].  Arguments and results as in the two separate calls.
 * Errors: EINVAL, ECAPACITY (some cache of the range is full; nothing is enqueued).
 */
int baklava_append_decode_attn(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count,
                               const void* k_new, const void* v_new, int32_t token_pos,
                               const void* q, float* out, void* stream);

/*
 * baklava_append_decode_attn for a step that is captured once into a HIP graph and replayed: nothing
 * the step needs is baked into the launch.  The new row's position is read on the device from
 * *token_pos_dev (DEVICE int32, 4-byte aligned; the caller advances it between replays, e.g. with a
 * kernel of its own inside the graph), and whether a cache still has room is decided on the device
 * from its length and capacity tables: a full cache receives no row, is attended as it stands, and
 * raises a status word that baklava_sync_lengths reports.  The host mirror of the lengths is
 * neither consulted nor advanced; call baklava_sync_lengths before the next call that relies on it
 * (baklava_append, baklava_append_decode_attn, baklava_decode_attn's empty-cache check,
 * baklava_lengths).  Only enqueues kernels: no memset, no copy, no synchronisation.
 * Errors: EINVAL.
 */
int baklava_append_decode_attn_replay(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count,
                                      const void* k_new, const void* v_new, const int32_t* token_pos_dev,
                                      const void* q, float* out, void* stream);

/*
 * Reads the device's length table back into the host mirror and returns ECAPACITY if, since the
 * last such call, a fused append found a cache full (the status word is then cleared).
 * Synchronises `stream`; not to be captured.
 */
int baklava_sync_lengths(baklava_ctx* ctx, void* stream);

/*
 * Score tracking keeps, per cached row, the attention it has received so far (summed over the
 * query heads of its group and over decode steps: the cumulative-attention statistic of the
 * heavy-hitter policies the paper's Related Work cites).  A row's weight in a call needs the
 * softmax normaliser of its whole cache, which is only known when the call is over, so the weights
 * of a call are added by a later attention call over the same layer, which streams the same K
 * rows anyway (a cache keeps up to 8 calls on record and adds them together), or by this
 * function: a pass over the K rows of the layer range alone.  After it the score plane of the
 * range holds every weight up to the latest call; without it the plane lacks at most the weights
 * of the calls on record, never anything else.  baklava_compact does this itself before it ranks
 * rows; baklava_reset and baklava_set_lengths drop what is on record.  The rows a recorded call
 * attended must keep their places until its weights are added: the library's own calls see to
 * that; a caller that rewrites arena rows itself calls baklava_set_lengths afterwards.
 * No-op without track_scores.  Enqueues kernels on `stream`, does not synchronise.
 * Errors: EINVAL, EHIP.
 */
int baklava_flush_scores(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count, void* stream);

/*
 * Eviction down to budget (f_evict, Eqs. 5-6: evicted rows vanish, survivors keep their order)
 * for every cache of the layer range whose length exceeds its budget.  Survivors: the first
 * `sink` rows, the last `recent` rows, and the budget - sink - recent middle rows with the
 * largest score (equal scores: the older row wins; scores compare as fp32, -0 == +0; NaN
 * scores are not supported).  POLICY_STREAMING keeps the sink rows and the budget - sink most
 * recent ones.  K, V, score and pos rows are moved in place; len <- min(len, budget).
 * kept_idx_out DEVICE int32 [total_tokens] or NULL: for each cache in range, entries
 * off[c] .. off[c] + new_len - 1 receive the old cache-local row index of each surviving row.
 * Rows at index >= new_len are unspecified afterwards.
 */
int baklava_compact(baklava_ctx* ctx, int32_t layer_begin, int32_t layer_count,
                    int32_t* kept_idx_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * One-time profiling (Algorithm 1), the step that produces the importance scores the budget
 * allocators above consume.
 * ------------------------------------------------------------------------------------------ */

/*
 * Algorithm 1, step 1, for every attention head of `batch` prompts of T tokens: causal attention of
 * the head over the prompt (Eq. 1 with the mask of autoregressive inference, logits scaled by
 * 1/sqrt(D)), the cosine between each token's value row v_t (the head's input) and the head's
 * output row for that token, and the mean of the cosines over the prompt.
 * q DEVICE bf16 [batch, Hq, T, D]; k, v DEVICE bf16 [batch, Hkv, T, D] (query head h reads KV head
 * h / (Hq/Hkv)); all 16-byte aligned.  D must be 128 and dtype BAKLAVA_BF16.
 * cos_out DEVICE fp32 [batch, Hq, T] (per-token cosines) or NULL; sim_out DEVICE fp32 [batch, Hq]
 * (mean per head); lse_out DEVICE fp32 [batch, Hq, T] or NULL: per token, log2 of the sum over its
 * visible keys of 2^(q_t.k_j log2(e)/sqrt(D)), the softmax normaliser baklava_prefill_scores needs.
 * A cosine whose norm product is below 1e-8 is divided by 1e-8 instead (a zero row gives 0).
 * workspace DEVICE, at least baklava_profile_workspace_bytes(batch, Hq, T) bytes, 16-byte aligned,
 * owned by the caller and free again once the stream has passed the call.
 * Enqueues two kernels on `stream`, does not synchronise.  Results are deterministic.
 * Errors: EINVAL (null, misaligned, bad shape), ECAPACITY (workspace too small), EHIP.
 */
size_t baklava_profile_workspace_bytes(int32_t batch, int32_t Hq, int32_t T);
int baklava_profile_similarity(const void* q, const void* k, const void* v, int32_t batch, int32_t Hq,
                               int32_t Hkv, int32_t T, int32_t D, int32_t dtype, float* cos_out,
                               float* sim_out, float* lse_out, void* workspace, size_t workspace_bytes,
                               void* stream);

/*
 * "Layer Importance Heuristic": the cosine between the input and the output hidden state of a layer,
 * token by token, and its mean over the prompt, for n_seq (layer, prompt) pairs at once.
 * x_in, x_out DEVICE bf16 [n_seq, T, hidden], 16-byte aligned, hidden a multiple of 8; dtype must be
 * BAKLAVA_BF16.  cos_out DEVICE fp32 [n_seq, T] or NULL; sim_out DEVICE fp32 [n_seq].  Zero rows as
 * in baklava_profile_similarity.  Layer importance follows with baklava_kv_importance (Hq = Hkv).
 * workspace DEVICE, at least baklava_layer_workspace_bytes(n_seq, T) bytes, 16-byte aligned.
 * Enqueues two kernels on `stream`; deterministic.
 * Errors: EINVAL, ECAPACITY (workspace too small), EHIP.
 */
size_t baklava_layer_workspace_bytes(int32_t n_seq, int32_t T);
int baklava_layer_similarity(const void* x_in, const void* x_out, int32_t n_seq, int32_t T, int32_t hidden,
                             int32_t dtype, float* cos_out, float* sim_out, void* workspace,
                             size_t workspace_bytes, void* stream);

/*
 * baklava_layer_similarity for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * per-workgroup partial sums go to a fixed device array inside the library
 * (BAKLAVA_LAYER_STATIC_MAX_TILES floats = 256 KiB, held by every GPU the library runs on until the
 * process ends) instead of a workspace; arguments, results and kernels are otherwise those of
 * baklava_layer_similarity, and the results are bit-identical to it.  The call allocates nothing
 * (no hipMalloc / hipFree, no allocating library routine).  The first call on a device looks up
 * the array's device address; make that one call outside a capture.
 * Limit: n_seq * ceil(T / 16) <= BAKLAVA_LAYER_STATIC_MAX_TILES, e.g. 32 layers x 32768 tokens.
 * All calls on one GPU share the array: calls that overlap in time on one GPU (different streams,
 * different host threads) race on it; calls on one stream are safe.  Nothing in it has to be
 * cleared between calls: a call only reads what it has written itself.
 * Errors: EINVAL (as baklava_layer_similarity; device index >= 64), ECAPACITY (beyond the limit
 * above: nothing is enqueued), EHIP.
 */
#define BAKLAVA_LAYER_STATIC_MAX_TILES 65536
int baklava_layer_similarity_static(const void* x_in, const void* x_out, int32_t n_seq, int32_t T,
                                    int32_t hidden, int32_t dtype, float* cos_out, float* sim_out,
                                    void* stream);

/*
 * Two-level allocation (host only): layer pools from the layer importances by the proportional
 * rule of baklava_alloc_proportional (bounds Hkv*lo .. Hkv*hi per layer, exact sum), then inside
 * each layer an equal split of the pool (remainder to the most important caches first, ties to the
 * lower index) followed by Algorithm 2 (baklava_alloc_threshold) with threshold t and fraction r.
 * The paper gives importances for layers and for the caches of a layer and Algorithm 2 for the
 * latter; how layer importances become pools is this library's reading.
 * layer_importance HOST [L]; head_importance HOST [L * Hkv]; budget_out HOST [L * Hkv]: each
 * layer's budgets sum to its pool, all of them to global_budget.
 * Errors: those of the two allocators.
 */
int baklava_alloc_two_level(const double* layer_importance, const double* head_importance, int32_t L,
                            int32_t Hkv, int64_t global_budget, int32_t lo, int32_t hi, double t, double r,
                            int32_t* budget_out);

/*
 * Attention scores of a whole prompt at once, for the eviction that precedes the decode loop
 * (f_evict of Eqs. 5-6 applied to a prefilled cache with the accumulated-attention policy):
 * score_j = sum over the Hq/Hkv query heads of the KV head and over the prompt tokens t >= j of the
 * causal softmax weight of key j for token t, i.e. what baklava_decode_attn's score tracking would
 * have accumulated had the T tokens been decoded one by one without eviction.
 * q DEVICE bf16 [batch, Hq, T, D]; lse DEVICE fp32 [batch, Hq, T] as written by
 * baklava_profile_similarity (or by any attention pass: log2-sum-exp of the scaled logits in log2
 * units); k DEVICE bf16: the T rows of sequence (b, KV head h) start at row row_off[b*Hkv + h] of the
 * plane (row_off DEVICE int64, e.g. a slice of an arena's offset table with k its K plane), or at
 * row (b*Hkv + h)*T when row_off is NULL; score_out DEVICE fp32, addressed by rows like k (e.g. the
 * arena's score plane): the T scores of every sequence are overwritten.  D must be 128, dtype
 * BAKLAVA_BF16.  Enqueues one kernel on `stream`; deterministic.
 * Errors: EINVAL (null, misaligned, bad shape), EHIP.
 */
int baklava_prefill_scores(const void* q, const void* k, const float* lse, const int64_t* row_off,
                           int32_t batch, int32_t Hq, int32_t Hkv, int32_t T, int32_t D, int32_t dtype,
                           float* score_out, void* stream);

/*
 * Algorithm 1, step 2, with the normalisation of "Head Importance Heuristic" (host only): the
 * similarities of the Hq/Hkv heads that share a KV cache are averaged, mapped from [-1, 1] to
 * [0, 1] by (s + 1) / 2, and importance is the complement.
 * similarity_host HOST double [L * Hq]; importance_out HOST double [L * Hkv].
 * Errors: EINVAL (null, Hq not a multiple of Hkv, a similarity outside [-1, 1] or not finite).
 */
int baklava_kv_importance(const double* similarity_host, int32_t L, int32_t Hq, int32_t Hkv,
                          double* importance_out);

/* Host mirror of the lengths; len_host_out HOST [n_caches].  No device access. */
int baklava_lengths(baklava_ctx* ctx, int32_t* len_host_out);

/* ------------------------------------------------------------------------------------------
 * Measurement aids.  Not part of the method: they exist so that the benchmark can time the dominant
 * kernel on the stream it runs on and calibrate the HBM byte counters against a transfer of known
 * size (together with BAKLAVA_OPT_TIME_KERNEL above).
 * ------------------------------------------------------------------------------------------ */

/*
 * Timing of the dominant kernel (the split-K attention partial kernel, which reads all
 * of the K/V bytes of Eq. 7): with BAKLAVA_OPT_TIME_KERNEL set, every attention call takes a pair
 * of HIP events for that kernel on the caller's stream: recorded right before and right after the
 * launch (mode 1: the pair also spans what the stream does between two commands), or handed to
 * the launch itself so that they carry the time stamps of the kernel's start and end (mode 2).
 * This call waits for the events, returns the summed elapsed time and the number of launches since
 * the last read, and clears the record.  total_ms_out, launches_out HOST scalars.
 */
int baklava_profile_read(baklava_ctx* ctx, double* total_ms_out, int64_t* launches_out);

/*
 * Streaming probe, independent of any context: streams `bytes` (a multiple of 16) through a
 * trivial kernel on `stream`.  mode 0 copies src to dst (both DEVICE, `bytes` long, 16-byte
 * aligned); modes 1 and 2 only read src, with ordinary and with non-temporal loads (dst DEVICE,
 * at least 1 KiB, is not meaningfully written); mode 3 is mode 2 on 64 workgroups only (what 64
 * compute units can pull on their own).
 * Used to calibrate the HBM byte counters against a transfer of known size and to measure the
 * bandwidth a plain streaming kernel reaches on the same device.
 * Errors: EINVAL (null, misaligned, bytes not a positive multiple of 16, bad mode), EHIP.
 */
int baklava_stream_probe(void* dst, const void* src, int64_t bytes, int32_t mode, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BAKLAVA_H */
