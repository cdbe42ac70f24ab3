// Internal launch interface between the C-ABI front end (api.cpp) and the HIP
// kernels.  Every function only enqueues work on `stream`; shapes have been
// validated by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moin {

constexpr int TILE_M = 256;        // rows per plan tile (prefill)
// The decode path (tokens gathered by expert, each distinct adapter read once, base
// product over plain row tiles) serves batches of up to DECODE_MAX_T tokens and
// larger ones whose sequences are short -- at most GATHER_MAX_AVG_LEN tokens on
// average, down to one expert per token ("Future Works", per token adapters) --
// where a row tile per sequence would be mostly padding.
constexpr int DECODE_MAX_T = 1024;
constexpr int GATHER_MAX_AVG_LEN = 128;
constexpr int GROUP_CHUNK = 128;   // tokens per group record: a hot expert's tokens are spread over several

// sticky error bits (device word)
constexpr int ERR_BAD_EXPERT = 1;
constexpr int ERR_BAD_OFFSETS = 2;
constexpr int ERR_BAD_ID = 4;
constexpr int ERR_BAD_RANK = 8;    // a per-expert rank that is negative or not a multiple of 8
constexpr int RANK_FULL = 0x7fffffff;   // "no per-expert rank": kernels take min(r, rank)

// Device-resident result of grouping a batch by expert.
struct PlanView {
    // prefill tiles (no tile spans two sequences; tiles sorted by expert)
    int *tile_row0;    // [max_tiles] first token of the tile
    int *tile_rows;    // [max_tiles] 1..TILE_M valid rows
    int *tile_expert;  // [max_tiles] adapter slot or -1
    int *tile_rank;    // [max_tiles] rank of that adapter (RANK_FULL without a rank table, 0 for slot -1)
    int *n_tiles;      // [1]
    // decode grouping (built only for batches that take the decode path)
    int *tok_sorted;   // [T] token index, grouped by expert
    int4 *grp_meta;    // [max_groups] {adapter slot or -1, first, one-past-last position in tok_sorted, rank};
                       // an expert with more than GROUP_CHUNK tokens has several records
    int *grp_start;    // [max_groups + 1] scratch while building
    int2 *grp_tmp;     // [max_groups] scratch while building: {slot, rank} of each expert's group
    // plain row tiles over all T tokens, no adapter (built with the decode grouping when
    // T > DECODE_MAX_T): the base product of such a batch runs on them
    int *plain_row0, *plain_rows, *plain_expert, *plain_rank, *plain_n;   // [max_plain] x 4, [1]
    int max_plain;
    int *n_groups;     // [1]
    // scratch used while building
    unsigned long long *keys; // [pow2 >= S]
    int *tmp;                 // [4 * (S + 1)]
    int max_tiles;
    int max_groups;
    int S;
    int64_t T;
    int E;
    int decode;  // grouping arrays valid
};

// rank_of_expert: [E] or null (every adapter at the stacks' full rank)
hipError_t launch_plan(const PlanView &pv, const int *seq_offsets, const int *expert_ids,
                       const int *rank_of_expert, int *err_word, hipStream_t stream);

struct LinearArgs {
    const void *x, *W, *A_stack, *B_stack;
    void *u_hi, *u_lo;     // [T, r] bf16 scratch
    void *y;
    int y_f32;
    int d_in, d_out, r;
    float scale;
    int act = 0;           // activation on W_a x (moin_set_adapter_activation)
};

hipError_t launch_prefill_shrink(const PlanView &pv, const LinearArgs &a, hipStream_t stream);
// The shrinks of up to MAX_SHARED_X projections that read the same x (q, k, v; gate, up)
// in one launch: the column tiles of projection i take A_stack[i] and write u_hi[i] /
// u_lo[i] ([T, r] each), and x streams from HBM once for all of them.  a: x, d_in, r,
// scale, act as for the single shrink (its own A_stack / u pointers unused).
constexpr int MAX_SHARED_X = 4;
hipError_t launch_prefill_shrink_shared(const PlanView &pv, const LinearArgs &a, int n, const void *const *A_stack,
                                        void *const *u_hi, void *const *u_lo, hipStream_t stream);
hipError_t launch_prefill_linear(const PlanView &pv, const LinearArgs &a, hipStream_t stream);
// The main products of n projections that share x, d_in, r and the output type in ONE launch of the
// streaming kernel (a[i]: W, B_stack, u_hi, u_lo, y, d_out of projection i); every a[i] must satisfy
// stream_kernel_fits.  Results are those of n single launches, bit for bit.
hipError_t launch_prefill_linear_shared(const PlanView &pv, const LinearArgs *a, int n, hipStream_t stream);
// shapes the persistent streaming prefill kernel takes (anything else: the tiled kernel)
bool stream_kernel_fits(const LinearArgs &a);
// shrink + MXFP8 codes / blocked scales of x in one pass over x (d_in a multiple of 128)
hipError_t launch_prefill_shrink_quant(const PlanView &pv, const LinearArgs &a, void *xq, void *xs,
                                       hipStream_t stream);

struct DecodeArgs {
    LinearArgs lin;
    void *ug_hi, *ug_lo;   // [T, r] bf16, indexed by position in tok_sorted
    float *ybase;          // [k_splits, T, d_out] fp32 partial sums of x W^T over disjoint k ranges
    int k_splits;
    int ybase_by_pos = 0;  // rows of ybase follow the plan's by-expert token order (else token order)
};
// Number of k ranges the decode base GEMM is cut into for this shape (>= 1).
int decode_base_splits(int64_t T, int d_in, int d_out);
// ybase[s] = x[:, k range s] W[:, k range s]^T
hipError_t launch_decode_base(const PlanView &pv, const DecodeArgs &a, hipStream_t stream);
// ug = scale * A_e x per expert group
hipError_t launch_decode_shrink(const PlanView &pv, const DecodeArgs &a, hipStream_t stream);
// y = sum_s ybase[s] + B_e ug, rounded to the output type
hipError_t launch_decode_expand(const PlanView &pv, const DecodeArgs &a, hipStream_t stream);
// base GEMM and shrink in one launch (shapes for which decode_base_shrink_fits)
bool decode_base_shrink_fits(const PlanView &pv, const DecodeArgs &a);
hipError_t launch_decode_base_shrink(const PlanView &pv, const DecodeArgs &a, hipStream_t stream);
// The same two launches for the n (<= MAX_SHARED_X) projections of a call that read the same x
// (gate, up; q, k, v): their base tiles, shrink slabs and expand blocks side by side, so that the
// launches' ramp and tail are paid once.  decode_shared_fits says whether the projections agree in
// everything the launches share.
bool decode_shared_fits(const PlanView &pv, const DecodeArgs *d, int n);
hipError_t launch_decode_base_shrink_shared(const PlanView &pv, const DecodeArgs *d, int n, hipStream_t stream);
hipError_t launch_decode_expand_shared(const PlanView &pv, const DecodeArgs *d, int n, hipStream_t stream);
// y = x W^T in one pass (no adapters anywhere in the call)
hipError_t launch_decode_base_only(const PlanView &pv, const LinearArgs &a, hipStream_t stream);

struct RouteArgs {
    const void *emb, *cent;
    int64_t N;
    int K, D;
    int is_bf16;
    const int *slot;       // [K] or null
    int retained_only;
    float *cnorm;          // [K rounded up to 256] workspace
    float *cinit;          // [same] workspace: -cnorm / 2
    int *cid;              // [N] centroid ids (user buffer or workspace)
    int *expert_ids;       // [N] or null
    // small batches: per-query packed (score, index) minimum merged across
    // workgroups, and the arrival counter that elects the finishing workgroup
    unsigned long long *best;  // [ROUTE_SMALL_MAX_N, or N when group > 1] workspace
    int *arrivals;             // [1] workspace
    int *counts;               // [K] or null: zeroed by the norms kernel
    int group;                 // route_stream_group() of the call
    int self_clean = 0;        // small batches: best / arrivals are kept clean between calls by the kernel
                               // itself, counts are zeroed by its finishing workgroup (no reset launch)
    // small batches, optional: the routed batch is grouped by expert in the same launch (the queries
    // are the batch's S = N sequences; expert_ids must be given)
    const PlanView *plan = nullptr;
    const int *seq_offsets = nullptr, *rank_of_expert = nullptr;
    int *err_word = nullptr;
};
constexpr int ROUTE_PLAN_FUSED_MAX_S = 512;  // the grouping rides in the routing launch up to this many queries
constexpr int ROUTE_SMALL_MAX_N = 4096;  // up to here the K range is split across workgroups
// true for the batches the small-batch kernel takes (bf16, D a multiple of 64, N <= ROUTE_SMALL_MAX_N)
bool route_small_batch(int64_t N, int K, int D, int is_bf16);
// Workgroups that share one query tile in the large-batch bf16 kernel (1: none).
int route_stream_group(int64_t N, int K, int D, int is_bf16);
hipError_t launch_centroid_norms(const RouteArgs &a, hipStream_t stream);
hipError_t launch_route(const RouteArgs &a, hipStream_t stream);
// the k (1..8) nearest centroids per query: a.cid / a.expert_ids are [N, k], d2 [N, k] or null
hipError_t launch_route_topk(const RouteArgs &a, int k, float *d2, hipStream_t stream);
// true when launch_route itself fills a.counts (no histogram launch needed)
bool route_tallies_counts(const RouteArgs &a);
hipError_t launch_histogram(const int *ids, int64_t N, int K, int *counts, int zero_first,
                            int *err_word, hipStream_t stream);


// K-means centre update (kmeans.hip)
constexpr int KM_PIECE = 512;     // a cluster's points are summed in pieces of at most this many
constexpr int KM_MAX_K = 32768;   // per-chunk cursor table lives in LDS
struct KmeansArgs {
    const void *emb;       // [N, D]
    const int *ids;        // [N] centre of each point
    int64_t N;
    const void *cent;      // [K, D] old centres, same type as emb
    int K, D;
    int is_bf16;
    void *out;             // [K, D] new centres or null (objective / counts only)
    int out_bf16;
    int *counts;           // [K] (user buffer or workspace)
    double *inertia;       // [1] or null
    // workspace
    int *table;            // [n_chunks, K]
    int *seg_start;        // [K + 1]
    int *piece_start;      // [K + 1]
    int4 *pieces;          // [max_pieces]
    int *n_pieces;         // [1]
    int *perm;             // [N]
    float *partial;        // [max_pieces, D]
    double *inertia_part;  // [max_pieces * ncb]
    int chunk, n_chunks, max_pieces, ncb;
    int *err_word;
};
// Launch shape for a problem size: points per chunk, number of chunks, upper
// bound on the number of pieces, column blocks of 256 16-byte chunks per row.
void kmeans_shape(int64_t N, int K, int D, int is_bf16, int *chunk, int *n_chunks, int *max_pieces, int *ncb);
hipError_t launch_kmeans_sort(const KmeansArgs &a, hipStream_t stream);     // perm[] and the piece list
hipError_t launch_kmeans_segsum(const KmeansArgs &a, hipStream_t stream);   // piece sums + objective shares
hipError_t launch_kmeans_finalize(const KmeansArgs &a, hipStream_t stream); // means, objective
hipError_t launch_kmeans_retain(const int *counts, int K, int min_count, int *slot, int *n_retained,
                                hipStream_t stream);

// Quantised base (mx.hip): MXFP8 codes and scale bytes of the base operands.
struct MxLinearArgs {
    LinearArgs lin;        // x (bf16, for the shrink), A_stack, B_stack, u_hi / u_lo, y; lin.W unused
    const void *xq, *xs;   // [T, d_in] codes, [d_in / 128, T, 4] scales (workspace, written per call)
    const void *Wq, *Ws;   // [d_out, d_in] codes, [d_in / 128, d_out, 4] scales
    // > 0: plain mode -- the base product alone over all T tokens, no plan tiles, the
    // contraction range in this many parts (mx_plain_shape), part s written to
    // lin.y + s * T * d_out elements
    int plain_splits, plain_kb_per_split;
};
void mx_plain_shape(int64_t T, int d_in, int d_out, int *k_splits, int *kb_per_split);
// codes / scales of rows x cols bf16 values (cols a multiple of 32); scales row-major
// [rows, cols / 32] or, blocked (cols a multiple of 128), [cols / 128, rows, 4]
hipError_t launch_mx_quantize(const void *src, int64_t rows, int64_t cols, void *codes, void *scales,
                              int blocked, hipStream_t stream);
bool mx_stream_kernel_fits(int d_in, int r);
hipError_t launch_linear_mx_stream(const PlanView &pv, const MxLinearArgs &a, int n_cus, hipStream_t stream);
int compute_units();   // of the current device

hipError_t prepare_kernels();  // one-time attribute set-up (large dynamic LDS)

// merged adapter (merge.hip): see moin_merge_adapters
hipError_t launch_merge_adapters(const void *A_stack, const void *B_stack, int E, int r, int d_in, int d_out,
                                 const int *ids, const float *weights, int n, int r_out, void *A_out, void *B_out,
                                 int *err_word, hipStream_t stream);

// on-box ceilings (probe.hip): out holds probe_out_len() elements
int64_t probe_out_len();
hipError_t launch_probe_mfma(const void *operands, int64_t n_bytes, int iters, float *out, double *flops,
                             hipStream_t stream);
hipError_t launch_probe_mfma_mx(const void *codes, int64_t n_bytes, int iters, float *out, double *flops,
                                hipStream_t stream);
hipError_t launch_probe_read(const void *src, int64_t n_bytes, uint32_t *out, hipStream_t stream);

}  // namespace moin
