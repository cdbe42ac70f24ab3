/*
 * libmoin -- MI355X (gfx950) kernels for the MoIN inference hot path:
 * nearest-topic routing of whole sequences and the sequence-routed
 * multi-adapter LoRA linear layer.
 *
 * Conventions that hold for every call unless a comment says otherwise
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     never frees, reallocates or keeps it after the call returns.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No call synchronises or reads device data on the
 *     host, so ids produced by moin_route can feed moin_lora_linear directly.
 *   - Return value: MOIN_OK (0) or a negative moin_status.  Nothing throws or
 *     aborts across this boundary.  Faults only visible in device data (an
 *     expert id >= E, offsets that run backwards) set a sticky error word in
 *     the context and moin_check() reports MOIN_EDATA.  A sequence with a bad
 *     expert id is computed base-only; offsets that do not tile [0, T) in
 *     order make the whole batch base-only.  Every output row is written
 *     either way.
 *   - N = 0, S = 0 or T = 0 are successful no-ops.  Zero-length sequences are
 *     legal.
 *   - A context owns a private device workspace (grown on demand with
 *     hipMalloc, so a call that needs more may synchronise the device once).
 *     One context serves one stream at a time; it is not thread-safe.
 *   - bf16 rows must be 16-byte aligned: base pointers 16-byte aligned and
 *     D, d_in, r multiples of 8.
 */
#ifndef MOIN_H
#define MOIN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moin_ctx moin_ctx;
typedef struct moin_plan moin_plan;

typedef enum { MOIN_F32 = 0, MOIN_BF16 = 1 } moin_dtype;

typedef enum {
    MOIN_OK = 0,
    MOIN_EINVAL = -1, /* null pointer, negative size, unsupported shape/alignment */
    MOIN_ENOMEM = -2, /* workspace allocation failed */
    MOIN_EHIP = -3,   /* a HIP runtime call failed */
    MOIN_EDATA = -4,  /* sticky device-side data fault, reported by moin_check */
    MOIN_ETOOBIG = -5,  /* size beyond the fixed limit of an entry point that does not allocate */
    MOIN_ECAPTURE = -6  /* the call would have to grow device memory on a stream under capture */
} moin_status;

/* moin_route flags */
#define MOIN_ROUTE_RETAINED_ONLY 1u /* search only centroids whose slot is >= 0 */
#define MOIN_ROUTE_SAME_CENTROIDS 2u /* the caller vouches that centroids (and, with
                                        MOIN_ROUTE_RETAINED_ONLY, slot_of_centroid) hold the
                                        same bits as in the previous moin_route call on this
                                        context with the same pointers and shapes: the
                                        centroid norms kept from that call are used again.
                                        Ignored when there is no such call to go by. */

/* Which kernel a timing slot refers to (moin_timing_*). */
typedef enum {
    MOIN_K_PLAN = 0,
    MOIN_K_SHRINK = 1,        /* prefill: u = s * x A_e^T (on a quantised base it
                                 may write x in MXFP8 in the same pass)        */
    MOIN_K_LINEAR = 2,        /* prefill: y = x W^T + u B_e^T (base + expand); the
                                 base product of gathered batches of short sequences */
    MOIN_K_ROUTE = 3,         /* distance GEMM fused with argmin; moin_route_topk  */
    MOIN_K_ROUTE_AUX = 4,     /* centroid norms, histogram, slot map            */
    MOIN_K_DECODE_SHRINK = 5, /* decode: gather-matvec u = s * A_e x; also holds
                                 the base GEMM when both share one launch       */
    MOIN_K_DECODE_EXPAND = 6, /* decode: gather-matvec B_e u + base, writes y   */
    MOIN_K_DECODE_BASE = 7,   /* decode: thin base GEMM launched on its own     */
    MOIN_K_KMEANS_SORT = 8,   /* K-means update: stable grouping of points by centre */
    MOIN_K_KMEANS_SUM = 9,    /* K-means update: the pass over the embeddings    */
    MOIN_K_KMEANS_FINAL = 10, /* K-means update: means, objective; cluster pruning */
    MOIN_K_MX_QUANT = 11,     /* quantised base: bf16 -> MXFP8 codes + scales    */
    MOIN_K_MX_LINEAR = 12,    /* quantised base: y = xq Wq^T + u B_e^T           */
    MOIN_K_PROBE_MFMA = 13,   /* measurement aid: bf16 matrix-core loop            */
    MOIN_K_PROBE_READ = 14,   /* measurement aid: streaming read                   */
    MOIN_K_COUNT = 15
} moin_kernel_id;

/* ---- context ----------------------------------------------------------- */

/* Creates a context bound to HIP device `device`.  Allocates only its own
 * small bookkeeping (the sticky error word); workspace grows on first use. */
int moin_create(moin_ctx **out, int device);

/* Frees the context and its workspace.  The caller must have synchronised
 * every stream that still runs work issued through it.  NULL is a no-op. */
void moin_destroy(moin_ctx *ctx);

/* Static, NUL-terminated description of a moin_status value. */
const char *moin_strerror(int code);

/* Synchronises `stream`, returns MOIN_EDATA if any call since the last check
 * met a device-side data fault (and clears the word), else MOIN_OK. */
int moin_check(moin_ctx *ctx, void *stream);

/* ---- routing ------------------------------------------------------------
 * Section 3.3 "Model inference": the query embedding is matched to the nearest
 * topic embedding; Section 3.1: topic embeddings are the K-means centres, so the
 * same call is the assignment step of K-means.  Squared L2 distance, ties to
 * the lowest centroid index.  Section 4 "Implementation details" / 4.1
 * "Downstream tasks": only some clusters keep an adapter; a topic without one
 * falls back to the base model (slot -1), or -- with
 * MOIN_ROUTE_RETAINED_ONLY -- is left out of the search altogether.
 * Figure 3: per-topic counts.
 *
 *   emb              [N, D] row-major, dt (fp32 or bf16)
 *   centroids        [K, D] row-major, same dt
 *   slot_of_centroid [K] int32 or NULL: adapter slot of each centroid, -1 = none
 *   flags            0, MOIN_ROUTE_RETAINED_ONLY (needs slot_of_centroid) and / or
 *                    MOIN_ROUTE_SAME_CENTROIDS (a serving loop routes every batch against
 *                    the same topic table; request-sized batches -- bf16, D a multiple of
 *                    64, N <= 4096 -- then take a single kernel launch)
 *   expert_ids       [N] int32 out or NULL: slot_of_centroid[centroid] (or the
 *                    centroid index itself when slot_of_centroid is NULL)
 *   centroid_ids     [N] int32 out or NULL: argmin centroid index
 *   counts           [K] int32 out or NULL: number of queries per centroid;
 *                    overwritten, not accumulated
 * D must be a multiple of 8 (bf16) or 4 (fp32).  A NaN distance never wins; a
 * query whose distances are all NaN gets centroid 0.
 */
int moin_route(moin_ctx *ctx, const void *emb, const void *centroids, int64_t N,
               int32_t K, int32_t D, moin_dtype dt,
               const int32_t *slot_of_centroid, uint32_t flags,
               int32_t *expert_ids, int32_t *centroid_ids, int32_t *counts,
               void *stream);

/* Figure 3 on its own: counts[k] = #{i : ids[i] == k}, ids outside [0, K) are
 * ignored and raise the sticky data fault.  counts is overwritten. */
int moin_histogram(moin_ctx *ctx, const int32_t *ids, int64_t N, int32_t K,
                   int32_t *counts, void *stream);

/* ---- routed LoRA linear ---------------------------------------------------
 * Section 3.2: y = W x + W_b (W_a x) for every token, with the adapter
 * (W_a, W_b) = (A_stack[e], B_stack[e]) chosen per SEQUENCE (Section 1: each
 * query is routed to a single expert) and `scale` applied to the adapter
 * term.  Expert id -1 means the topic has no adapter: y = W x (Section 4.1).
 *
 *   x           [T, d_in]      bf16 row-major
 *   seq_offsets [S+1] int32    seq_offsets[0] = 0, non-decreasing, [S] = T
 *   expert_ids  [S]   int32    in [-1, E)
 *   W           [d_out, d_in]  bf16 (y = x W^T)
 *   A_stack     [E, r, d_in]   bf16   (may be NULL when E == 0 or r == 0)
 *   B_stack     [E, d_out, r]  bf16
 *   y           [T, d_out]     out, y_dt = MOIN_BF16 (round-to-nearest-even
 *                              from the fp32 accumulator) or MOIN_F32
 * Accumulation is fp32; u = s * W_a x is carried as a sum of two bf16 values
 * (high part + remainder) into the expand product.
 * d_in and r must be multiples of 8; d_out a multiple of 8 (bf16 y) or 4.
 * Small batches (T <= 1024) take the decode path: tokens are grouped by
 * expert so each distinct adapter is read from HBM once.  So do larger batches
 * of short sequences (T <= 128 S, i.e. 128 tokens per sequence on average or
 * fewer, down to one expert per token: "Future Works", per token adapters),
 * where a row tile per sequence would be mostly padding: their base product
 * runs over plain tiles of 256 tokens and the adapter term over the tokens
 * gathered by expert.
 */
int moin_lora_linear(moin_ctx *ctx, const void *x, const int32_t *seq_offsets,
                     const int32_t *expert_ids, int32_t S, int64_t T,
                     const void *W, const void *A_stack, const void *B_stack,
                     int32_t E, int32_t d_in, int32_t d_out, int32_t r,
                     float scale, void *y, moin_dtype y_dt, void *stream);

/* The grouping of sequences by expert depends only on (seq_offsets,
 * expert_ids, E); a plan computes it once for all projections of a layer
 * (Section 3.2: every linear layer carries an adapter).
 * moin_plan_build overwrites the plan; the plan must outlive, and must not be
 * rebuilt before the completion of, the calls that use it. */
int moin_plan_create(moin_ctx *ctx, moin_plan **out);
void moin_plan_destroy(moin_plan *plan);
int moin_plan_build(moin_ctx *ctx, moin_plan *plan, const int32_t *seq_offsets,
                    const int32_t *expert_ids, int32_t S, int64_t T, int32_t E,
                    void *stream);
int moin_lora_linear_planned(moin_ctx *ctx, const moin_plan *plan, const void *x,
                             const void *W, const void *A_stack,
                             const void *B_stack, int32_t d_in, int32_t d_out,
                             int32_t r, float scale, void *y, moin_dtype y_dt,
                             void *stream);

/* moin_lora_linear_planned for n (1..4) projections of a layer that read the same
 * input x [T, d_in] (q, k, v; gate, up): on the prefill path the adapters' first
 * products u_i = scale * x A_{i,e}^T of all n come out of ONE pass over x, then
 * each projection's main product runs as in moin_lora_linear_planned (in one launch
 * where all of them fit the streaming kernel); on the decode path the projections'
 * work shares the call's two launches (base products and first adapter products,
 * then second adapter products) where they agree in the number of parts of the base
 * product, else they run one after the other.  The results are, bit for bit, those of
 * n single calls.  W, A_stack, B_stack, y: host arrays
 * of n device pointers (stacks [E, r, d_in] / [E, d_out[i], r]; A_stack and B_stack
 * may be NULL when there are no adapters), d_out: host array of n widths; r and
 * scale are common.  Needs 2 n T r bf16 of workspace.  Errors as
 * moin_lora_linear_planned; n outside 1..4: MOIN_EINVAL. */
int moin_lora_linear_planned_shared(moin_ctx *ctx, const moin_plan *plan, const void *x, int32_t n,
                                    const void *const *W, const void *const *A_stack,
                                    const void *const *B_stack, int32_t d_in, const int32_t *d_out,
                                    int32_t r, float scale, void *const *y, moin_dtype y_dt,
                                    void *stream);

/* moin_route followed by moin_plan_build_ranked on the ids it produced, for a batch
 * whose N queries ARE its S = N sequences (Section 1: each query goes to one expert;
 * Section 3.2: the expert's adapter then serves every linear layer of that query).
 * A request-sized batch (bf16, D a multiple of 64, N <= 512, K <= 65536) takes ONE
 * launch: the workgroup that finishes the routing groups the batch by the ids it has
 * just written; any other batch takes the launches of the two calls.  Results are
 * those of the two calls.  Arguments as in moin_route and moin_plan_build_ranked;
 * expert_ids [N] is required (it is the plan's input and stays the caller's), the
 * ids are adapter slots of [0, E) or -1 when slot_of_centroid is given and centroid
 * indices otherwise (then E >= K is required); rank_of_expert may be NULL.
 * Errors: those of the two calls. */
int moin_route_plan(moin_ctx *ctx, moin_plan *plan, const void *emb, const void *centroids,
                    int64_t N, int32_t K, int32_t D, moin_dtype dt,
                    const int32_t *slot_of_centroid, uint32_t flags,
                    const int32_t *seq_offsets, int64_t T, int32_t E,
                    const int32_t *rank_of_expert, int32_t *expert_ids,
                    int32_t *centroid_ids, int32_t *counts, void *stream);

/* ---- HIP graphs and the library's own device memory ----------------------------
 * The context's workspace and a plan's buffer grow on demand (hipMalloc), which a
 * stream under capture must not do.  A call on a capturing stream that would have
 * to grow either returns MOIN_ECAPTURE and records nothing: make the first call
 * with the largest shapes outside the capture, or reserve beforehand.  A workspace
 * or plan buffer that a captured call has used is kept until moin_destroy /
 * moin_plan_destroy even when a later, larger call replaces it, so replays of the
 * graph keep reading valid memory (results of a replay are then only defined if
 * no other call on the context runs concurrently, as for eager calls).
 *   moin_reserve_workspace: the workspace holds at least `bytes` afterwards.
 *   moin_workspace_bytes:   its present size -- after an eager call with the
 *                           largest shapes, the figure to reserve elsewhere.
 *   moin_plan_reserve:      the plan's buffer holds the plan of any batch of at
 *                           most S sequences, T tokens and E experts.
 * Errors: MOIN_EINVAL (null, negative sizes), MOIN_ENOMEM, MOIN_ECAPTURE (`stream`
 * is being captured and growth is needed). */
int moin_reserve_workspace(moin_ctx *ctx, int64_t bytes, void *stream);
int64_t moin_workspace_bytes(const moin_ctx *ctx);
int moin_plan_reserve(moin_ctx *ctx, moin_plan *plan, int32_t S, int64_t T, int32_t E, void *stream);

/* moin_route for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as moin_route, but every intermediate result (centroid norms,
 * the packed per-query minima that workgroups merge, the arrival counter, centroid
 * ids when only counts are asked for) lives in a fixed 1 MiB array in the library's
 * device image instead of the context's workspace, so the call never calls
 * hipMalloc / hipFree and records no timing events.  Limits: N <= 65536 queries,
 * K <= 16384 centroids; beyond them MOIN_ETOOBIG and nothing is launched.  Every
 * call on a GPU shares that GPU's array: the kernels re-initialise what they
 * accumulate into on every call, and two calls that overlap on one GPU (different
 * streams, different contexts) race. */
#define MOIN_ROUTE_STATIC_MAX_N 65536
#define MOIN_ROUTE_STATIC_MAX_K 16384
int moin_route_static(moin_ctx *ctx, const void *emb, const void *centroids, int64_t N,
                      int32_t K, int32_t D, moin_dtype dt,
                      const int32_t *slot_of_centroid, uint32_t flags,
                      int32_t *expert_ids, int32_t *centroid_ids, int32_t *counts,
                      void *stream);

/* ---- per-kernel timing ----------------------------------------------------
 * When enabled, every kernel launch is bracketed by HIP events on the launch
 * stream.  moin_timing_read synchronises those events and returns, for one
 * kernel id, the summed duration in milliseconds and the number of launches
 * since the last moin_timing_reset.  Meant for benchmarks; off by default. */
int moin_timing_enable(moin_ctx *ctx, int on);
int moin_timing_reset(moin_ctx *ctx);
int moin_timing_read(moin_ctx *ctx, int kernel_id, double *ms_sum,
                     int64_t *launches);

/* ==== beyond the two core calls: rows the paper lists as next steps ============== */

/* ---- K-means (topic modelling) --------------------------------------------
 * Section 3.1: the topics are the cells of a plain K-means clustering of the
 * document embeddings, and its cluster centres are the topic embeddings that
 * moin_route searches.  The assignment step of an iteration IS moin_route;
 * moin_kmeans_update is the centre update: every centre becomes the mean of
 * the embeddings assigned to it.  The paper does not say what happens to a
 * centre nobody was assigned to: here it keeps its old value.
 *
 *   emb           [N, D] row-major, dt (fp32 or bf16)
 *   ids           [N] int32, centre of each embedding, in [0, K); others are
 *                 skipped and raise the sticky data fault
 *   centroids     [K, D] old centres, same dt
 *   new_centroids [K, D] out, out_dt (rounded to nearest even when bf16), or
 *                 NULL.  May be the same buffer as centroids when out_dt == dt.
 *   counts        [K] int32 out or NULL: points per centre (overwritten)
 *   inertia       [1] double out (DEVICE pointer) or NULL: the K-means objective
 *                 sum_i ||emb_i - centroids[ids_i]||^2 against the OLD centres
 * Column sums are accumulated in fp32 over at most 512 points at a time and in
 * fp64 across such pieces; the objective is summed in fp64.  Points are added
 * in index order, so results repeat bit for bit.  K <= 32768; D a multiple of
 * 8 (bf16) or 4 (fp32); N < 2^31 - 4096.
 */
int moin_kmeans_update(moin_ctx *ctx, const void *emb, const int32_t *ids, int64_t N,
                       const void *centroids, int32_t K, int32_t D, moin_dtype dt,
                       void *new_centroids, moin_dtype out_dt, int32_t *counts,
                       double *inertia, void *stream);

/* Section 4 "Implementation details": clusters that stay extremely small are
 * dropped and get no adapter (4697 of 5000 were kept).  The paper gives no
 * threshold, so it is an argument: slot_of_centroid[k] = rank of k among the
 * centres with counts[k] >= min_count (ascending k), -1 for the others -- the
 * table moin_route takes.  n_retained [1] int32 out (device) or NULL. */
int moin_retain_clusters(moin_ctx *ctx, const int32_t *counts, int32_t K, int32_t min_count,
                         int32_t *slot_of_centroid, int32_t *n_retained, void *stream);

/* `iters` rounds of (moin_route, moin_kmeans_update) with the centres updated
 * in place, then one more assignment, so that ids / counts belong to the centres
 * returned.  inertia: [iters + 1] doubles (device) or NULL; entry t is the
 * objective of assignment t against the centres it was made with, so the
 * sequence never increases (up to rounding of the centres to dt).  ids [N] is
 * required when N > 0.  No host synchronisation: the iteration count is fixed. */
int moin_kmeans_fit(moin_ctx *ctx, const void *emb, int64_t N, void *centroids, int32_t K,
                    int32_t D, moin_dtype dt, int32_t iters, int32_t *ids, int32_t *counts,
                    double *inertia, void *stream);

/* ---- adapter residency cache ------------------------------------------------
 * Section 2 (serving paragraph): the adapters of all topics are kept in CPU
 * memory and the most frequently routed ones are cached in GPU memory.  A
 * moin_cache maps E stored experts onto n_slots resident slots.  Per batch,
 * moin_cache_admit takes the batch's expert ids (a HOST array: paging is decided
 * on the host), makes every needed expert resident and returns one slot id per
 * sequence; moin_lora_linear then runs on the slot stacks (E = n_slots) with
 * those slot ids.  Policy: every sequence adds one to its expert's use count;
 * a needed expert is always loaded; free slots go lowest index first; the
 * victim is the resident expert not needed by the batch with the fewest uses,
 * then the least recently used, then the lowest slot; when every slot holds an
 * expert of the batch, the rest of the batch's experts get slot -1 (base model
 * only, Section 4.1).
 *
 * moin_cache_add_stack registers one projection: A_host [E, ...] / B_host
 * [E, ...] in HOST memory (pinned, if the copies are to be asynchronous) and
 * A_slots [n_slots, ...] / B_slots [n_slots, ...] in DEVICE memory, with the
 * bytes of one expert in each; all owned by the caller and alive as long as the
 * cache.  Stacks are registered before the first batch.  moin_cache_admit
 * enqueues the copies on `stream`, the stream the batch's kernels will run on
 * (so a slot is never overwritten under a kernel that still reads it); with no
 * stack registered it is pure bookkeeping and needs no GPU.  expert id -1 maps
 * to slot -1; ids outside [-1, E) fail with MOIN_EINVAL before anything
 * changes.  Not thread-safe.
 */
typedef struct moin_cache moin_cache;
typedef enum {
    MOIN_CACHE_BATCHES = 0,
    MOIN_CACHE_SEQ_HITS = 1,   /* sequences whose expert was resident          */
    MOIN_CACHE_SEQ_MISSES = 2, /* sequences whose expert was not               */
    MOIN_CACHE_LOADS = 3,      /* experts copied in (per expert, not per stack) */
    MOIN_CACHE_EVICTIONS = 4,
    MOIN_CACHE_OVERFLOWS = 5,  /* experts left without a slot                  */
    MOIN_CACHE_BYTES = 6,      /* host-to-device bytes enqueued                */
    MOIN_CACHE_STAT_COUNT = 7
} moin_cache_stat;
int moin_cache_create(moin_cache **out, int32_t E, int32_t n_slots);
void moin_cache_destroy(moin_cache *cache);
int moin_cache_add_stack(moin_cache *cache, const void *A_host, const void *B_host,
                         void *A_slots, void *B_slots, int64_t a_bytes_per_expert,
                         int64_t b_bytes_per_expert);
int moin_cache_admit(moin_cache *cache, const int32_t *expert_ids, int32_t S,
                     int32_t *slot_ids, void *stream);
/* Overlap mode, chosen before the first batch (later: MOIN_EINVAL): the copies of an
 * admission go on a stream the cache owns instead of `stream`, so a server can admit
 * batch k+1 right after it has enqueued the kernels of batch k and have the adapters
 * cross PCIe under those kernels.  For that to be safe the experts of the batch
 * admitted just before are protected from eviction like the batch's own (a newcomer
 * finds no slot -- slot -1 -- when every slot holds an expert of either), the copy
 * stream waits for the compute work enqueued on `stream` before the previous
 * admission, and `stream` is made to wait for the copies before the work enqueued on
 * it next.  The caller keeps to the order: kernels of batch k, then admit(k+1). */
int moin_cache_set_overlap(moin_cache *cache, int on);
/* Copies of the tables (HOST arrays, either may be NULL): slot_of_expert [E],
 * expert_in_slot [n_slots]; -1 = not resident / free. */
int moin_cache_table(const moin_cache *cache, int32_t *slot_of_expert,
                     int32_t *expert_in_slot);
/* stats [MOIN_CACHE_STAT_COUNT] (HOST array), totals since creation. */
int moin_cache_stats(const moin_cache *cache, int64_t *stats);

/* "Future Works", adaptive rank per topic (also Section 4.2: the rank could follow
 * the amount of training data): the same layer with a rank per expert.
 * rank_of_expert [E] int32 (DEVICE) or NULL; expert e uses the first
 * rank_of_expert[e] rows of A_stack[e] and columns of B_stack[e], 0 <= rank <= r,
 * a multiple of 8 (rank 0: base model only).  The stacks keep their [E, r, ...]
 * shape.  What lies beyond an expert's rank is not used: rows of A_e beyond it are
 * never read; columns of B_e from the rank up to the next multiple of 64 are
 * multiplied by zeros on the prefill path and must therefore be finite (zero
 * padding is the natural choice), further columns are never read.  The decode
 * path reads only rank_e rows / columns of every distinct adapter.  A rank that
 * is negative or not a multiple of 8 raises the sticky data fault (it is rounded
 * down; negative: full rank); a rank above r counts as r. */
int moin_lora_linear_ranked(moin_ctx *ctx, const void *x, const int32_t *seq_offsets,
                            const int32_t *expert_ids, int32_t S, int64_t T,
                            const void *W, const void *A_stack, const void *B_stack,
                            int32_t E, int32_t d_in, int32_t d_out, int32_t r,
                            const int32_t *rank_of_expert, float scale, void *y,
                            moin_dtype y_dt, void *stream);

/* moin_plan_build with per-expert ranks (see moin_lora_linear_ranked); the ranks are
 * resolved into the plan, rank_of_expert need not outlive the call's completion. */
int moin_plan_build_ranked(moin_ctx *ctx, moin_plan *plan, const int32_t *seq_offsets,
                           const int32_t *expert_ids, int32_t S, int64_t T, int32_t E,
                           const int32_t *rank_of_expert, void *stream);
/* "Future Works", quantising the base model (a QLoRA-like, aggressively quantised
 * base whose loss the experts recover; the paper names the idea only).  The
 * format here is OCP Microscaling MXFP8: along the last axis, blocks of 32
 * consecutive values share one power-of-two scale 2^(E-127) (E8M0 byte E) and
 * hold FP8 E4M3 elements (bias 7, largest finite value 448, no infinities).
 *
 * moin_mx_quantize: src [rows, cols] bf16 (DEVICE, finite values; NaN / Inf give
 * unspecified codes) -> codes [rows, cols] uint8 and rows * cols/32 scale bytes
 * (both DEVICE, caller-owned).  scale_layout: MOIN_MX_ROW_MAJOR, scales
 * [rows, cols/32]; MOIN_MX_BLOCKED (cols a multiple of 128), scales
 * [cols/128, rows, 4] -- the four bytes of 128 consecutive values of a row form
 * one word and the words of consecutive rows are adjacent, which is the order
 * the matrix-core kernel fetches them in.  E = max(0, floor(log2 max|v|) + 127 - 8) per
 * block (127 for a block of zeros); element = v / 2^(E-127) rounded to nearest
 * even, magnitudes above 448 clamped to 448.  cols must be a multiple of 32,
 * src and codes 16-byte aligned.  Used once for the weight. */
enum { MOIN_MX_ROW_MAJOR = 0, MOIN_MX_BLOCKED = 1 };
int moin_mx_quantize(moin_ctx *ctx, const void *src, int64_t rows, int64_t cols, void *codes,
                     void *scales, int32_t scale_layout, void *stream);

/* moin_lora_linear_ranked on a quantised base:
 *     y = dq(q(x)) dq(Wq)^T + scale * (x A_e^T) B_e^T
 * Wq [d_out, d_in] codes and Ws (MOIN_MX_BLOCKED layout: [d_in/128, d_out, 4])
 * come from moin_mx_quantize; x [T, d_in] is bf16 and is quantised by the call itself
 * (into the context's workspace) for the base product, which runs on the
 * block-scaled FP8 matrix cores; the adapter term uses the bf16 x and the bf16
 * stacks exactly as in moin_lora_linear.  rank_of_expert may be NULL.
 * Shapes: d_in a multiple of 128 and at least 256, r a multiple of 64, d_out a
 * multiple of 8; anything else returns MOIN_EINVAL.  Small batches (T <= 1024)
 * and batches of short sequences (T <= 128 S, see moin_lora_linear)
 * compute the base product for all tokens at once on the FP8 matrix cores and
 * add the adapter term with the decode path's gather-matvec kernels. */
int moin_lora_linear_mx(moin_ctx *ctx, const void *x, const int32_t *seq_offsets,
                        const int32_t *expert_ids, int32_t S, int64_t T,
                        const void *Wq, const void *Ws, const void *A_stack, const void *B_stack,
                        int32_t E, int32_t d_in, int32_t d_out, int32_t r,
                        const int32_t *rank_of_expert, float scale, void *y,
                        moin_dtype y_dt, void *stream);

/* moin_lora_linear_mx on a plan (moin_plan_build / moin_plan_build_ranked), for the
 * projections of a layer.  xq [T, d_in] / xs (MOIN_MX_BLOCKED layout,
 * [d_in/128, T, 4]) hold the quantised activations (device, 16-byte aligned), so
 * that projections that share their input (q, k, v; gate, up) quantise it once:
 *   MOIN_MX_X_INTERNAL  xq, xs NULL: the call quantises x into the context's workspace;
 *   MOIN_MX_X_EMIT      the call quantises x into xq / xs (the caller's buffers; with
 *                       adapters in a prefill batch that happens inside the shrink's
 *                       pass over x) and uses them;
 *   MOIN_MX_X_GIVEN     xq / xs are read: what an earlier MOIN_MX_X_EMIT call or
 *                       moin_mx_quantize(x, MOIN_MX_BLOCKED) wrote for the same x.
 * x (bf16) is needed in every case, for the adapter term.  A mode that does not
 * fit the pointers returns MOIN_EINVAL. */
enum { MOIN_MX_X_INTERNAL = 0, MOIN_MX_X_EMIT = 1, MOIN_MX_X_GIVEN = 2 };
int moin_lora_linear_mx_planned(moin_ctx *ctx, const moin_plan *plan, const void *x,
                                void *xq, void *xs, int32_t x_codes, const void *Wq, const void *Ws,
                                const void *A_stack, const void *B_stack, int32_t d_in,
                                int32_t d_out, int32_t r, float scale, void *y, moin_dtype y_dt,
                                void *stream);

/* ==== the paper's "Future Works" variants ========================================= */

/* "Future Works", better adapters: an activation function between the adapter's
 * two linear layers,
 *     y = x W^T + scale * act(x A_e^T) B_e^T,
 * applied to x A_e^T in fp32 before the scale.  The paper names no function; these
 * are the textbook ones: ReLU max(v, 0), SiLU v / (1 + exp(-v)), GELU
 * v/2 (1 + erf(v / sqrt 2)).  It is a property of the adapters the stacks hold (of
 * how they were trained), not of a call, so it is set on the context and holds
 * for every later moin_lora_linear* call on it (plain, ranked, planned, on a
 * quantised base; prefill and decode) until set again.  Default MOIN_ACT_NONE, the
 * paper's adapter.  Any other value: MOIN_EINVAL, setting unchanged. */
enum { MOIN_ACT_NONE = 0, MOIN_ACT_RELU = 1, MOIN_ACT_SILU = 2, MOIN_ACT_GELU = 3 };
int moin_set_adapter_activation(moin_ctx *ctx, int32_t activation);

/* The k (1..8) nearest topic embeddings of every query, nearest first, equal
 * distances by increasing centroid index ("Future Works", creating new experts on
 * the fly: a query on the boundary of several clusters, or one that needs several
 * adapters).  Arguments as moin_route; outputs are [N, k] row-major, each may be
 * NULL: centroid_ids, expert_ids (slot_of_centroid applied; -1 also where fewer
 * than k centroids took part), dist2 (fp32 squared distances, +inf where
 * unfilled).  Column 0 is moin_route's answer up to fp32 rounding of the
 * distances.  A request-time call (one wave per query, distances as plain sums of
 * squared differences), not the bulk router.  k outside 1..8: MOIN_EINVAL. */
int moin_route_topk(moin_ctx *ctx, const void *emb, const void *centroids, int64_t N,
                    int32_t K, int32_t D, moin_dtype dt, const int32_t *slot_of_centroid,
                    uint32_t flags, int32_t k, int32_t *expert_ids, int32_t *centroid_ids,
                    float *dist2, void *stream);

/* "Future Works", creating new experts on the fly (a server that merges existing
 * adapters for a query that needs several of them): writes ONE adapter of rank
 * n * r that stands for sum_m weights[m] * W_b[ids[m]] W_a[ids[m]], by concatenation:
 *     A_out[m r + j, :] = A[ids[m]][j, :]
 *     B_out[:, m r + j] = bf16(weights[m] * B[ids[m]][:, j])   (fp32 product, nearest even)
 * for m < n; an id of -1 (as moin_route_topk leaves where a list is short) gives a
 * block of zeros, and everything from n r up to r_out is zero.
 *   A_stack [E, r, d_in], B_stack [E, d_out, r]  bf16, device
 *   ids [n] int32, weights [n] fp32              device (no host read: they may come
 *                                                straight from moin_route_topk)
 *   A_out [r_out, d_in], B_out [d_out, r_out]    bf16, device: typically one slot of
 *                                                stacks of rank r_out, used through
 *                                                moin_lora_linear_ranked with rank n r
 * r, r_out, d_in multiples of 8, n r <= r_out, pointers 16-byte aligned; else
 * MOIN_EINVAL.  An id outside [-1, E) raises the sticky data fault (moin_check)
 * and gives a block of zeros. */
int moin_merge_adapters(moin_ctx *ctx, const void *A_stack, const void *B_stack, int32_t E,
                        int32_t r, int32_t d_in, int32_t d_out, const int32_t *ids,
                        const float *weights, int32_t n, int32_t r_out, void *A_out, void *B_out,
                        void *stream);

/* ==== measurement aids (not part of the method's path) =========================== */

/* Measurement aids: the ceilings of this very device, beside the datasheet peaks,
 * for the roofline fractions that bench.py reports (the hot path of the paper's
 * method does not call them).
 * moin_probe_out_len: elements that `out` of the two probes must hold.
 * moin_probe_mfma_bf16: every wave of a chip-filling grid runs `iters` times 32
 *   independent v_mfma_f32_16x16x32_bf16 on operands taken from `operands` (device,
 *   bf16 values, n_bytes a multiple of 16 and at least 16; the values matter: the
 *   matrix cores reach their power limit sooner on random data than on constants);
 *   out[i] (device, fp32) = sum of thread i's accumulators; *flops (host, may be
 *   NULL) = the flops of the launch.
 * moin_probe_mfma_mxfp8: the same for the block-scaled FP8 instruction of the
 *   quantised-base kernel: `iters` times 8 independent
 *   v_mfma_scale_f32_32x32x64_f8f6f4 per wave on FP8 E4M3 codes taken from `codes`,
 *   all block scales 1.
 * moin_probe_read: reads src (device, n_bytes a multiple of 16) once, eight 16-byte
 *   loads per thread in flight; out[i] (device) = sum mod 2^32 of the 32-bit words
 *   thread i read.
 * Time them with moin_timing_* (MOIN_K_PROBE_MFMA, MOIN_K_PROBE_READ).  Errors:
 * MOIN_EINVAL for null pointers or sizes as excluded above. */
int64_t moin_probe_out_len(moin_ctx *ctx);
int moin_probe_mfma_bf16(moin_ctx *ctx, const void *operands, int64_t n_bytes, int32_t iters,
                         float *out, double *flops, void *stream);
int moin_probe_mfma_mxfp8(moin_ctx *ctx, const void *codes, int64_t n_bytes, int32_t iters,
                          float *out, double *flops, void *stream);
int moin_probe_read(moin_ctx *ctx, const void *src, int64_t n_bytes, uint32_t *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOIN_H */
