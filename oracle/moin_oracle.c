/*
 * moin_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct CPU definition of what the MoIN hot path
 * computes.  It exists so that the HIP library can be checked against
 * something that shares no code with it.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it; the product never does.
 *
 * Everything is the textbook definition written out with fp64 accumulation in
 * index order.  bf16 and fp32 inputs widen to fp64 exactly, so the only
 * rounding is that of the fp64 sums themselves.  No blocking, no fusion, no
 * reordering; OpenMP splits the outermost (token / query) loop only.
 *
 * What each function follows:
 *   route      -- Section 3.3 "Model inference": nearest-neighbour search of
 *                 the query embedding over the topic embeddings, which are the
 *                 K-means cluster centres (Section 3.1).  Squared L2; the
 *                 lowest index wins ties.
 *   slot map   -- Section 4 "Implementation details" (only 4697 of 5000
 *                 clusters keep an adapter) and Section 4.1 "Downstream
 *                 tasks" (a topic without an adapter falls back to the base
 *                 model; the 4697-variant searches retained topics only).
 *   histogram  -- documents per topic, Figure 3.
 *   kmeans_update -- Section 3.1 / Section 4 "Implementation details": the
 *                 topics are the cells of a plain K-means clustering of the
 *                 document embeddings and the topic embeddings are its cluster
 *                 centres.  This is the textbook centre update of one Lloyd
 *                 iteration: each centre becomes the mean of the embeddings
 *                 assigned to it; a centre nobody was assigned to keeps its
 *                 old value (the paper drops tiny clusters afterwards, it does
 *                 not say what its K-means does with empty ones).  Also the
 *                 clustering objective (sum of squared distances to the
 *                 assigned old centres).
 *   retain_clusters -- Section 4 "Implementation details": clusters below a
 *                 size threshold are dropped; the others are numbered in order.
 *   lora_linear-- Section 3.2: y = W x + W_b (W_a x), with one adapter per
 *                 sequence (Section 1: each query goes to a single expert),
 *                 a caller-given scale on the adapter term, and the base-only
 *                 fallback for expert id -1.
 *   mx_quantize / lora_linear_mx -- "Future Works", quantising the base
 *                 model: the paper only names the idea (a QLoRA-like, aggressively
 *                 quantised base with full-precision experts).  The format taken
 *                 here is the OCP Microscaling (MX) v1.0 "MXFP8" block format:
 *                 blocks of 32 consecutive elements along the contraction index
 *                 share one power-of-two scale (E8M0 byte) and hold FP8 E4M3
 *                 elements (OCP 8-bit floating point: bias 7, largest finite 448,
 *                 no infinities).  The base product runs on the quantised
 *                 weight and the quantised activations, the adapter term on the
 *                 unquantised bf16 activations.
 *
 * Parity pins live in tests/test_oracle_*.py (closed forms, numpy fp64
 * special cases, brute force, metamorphic relations).  Anything that would
 * need the paper's datasets or trained weights is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)

/* bf16 is the top 16 bits of an IEEE-754 binary32: widening is exact. */
static double bf16_to_f64(uint16_t h)
{
    union { uint32_t u; float f; } v;
    v.u = ((uint32_t)h) << 16;
    return (double)v.f;
}

/* ---- routing --------------------------------------------------------- */

/* Squared L2 distance of one query to one centroid, fp64, summed in index
 * order.  dt: 0 = fp32 storage, 1 = bf16 storage. */
static double dist2(const void *emb, const void *cent, int64_t i, int32_t k,
                    int32_t D, int dt)
{
    double acc = 0.0;
    if (dt == 0) {
        const float *q = (const float *)emb + (size_t)i * D;
        const float *c = (const float *)cent + (size_t)k * D;
        for (int32_t j = 0; j < D; ++j) {
            double diff = (double)q[j] - (double)c[j];
            acc += diff * diff;
        }
    } else {
        const uint16_t *q = (const uint16_t *)emb + (size_t)i * D;
        const uint16_t *c = (const uint16_t *)cent + (size_t)k * D;
        for (int32_t j = 0; j < D; ++j) {
            double diff = bf16_to_f64(q[j]) - bf16_to_f64(c[j]);
            acc += diff * diff;
        }
    }
    return acc;
}

/* Exported so tests can price a near-tie: D2(i, k) for chosen pairs. */
int moin_oracle_dist2(const void *emb, const void *cent, int32_t D, int dt,
                      const int64_t *qi, const int32_t *ki, int64_t n,
                      double *out)
{
    if (!emb || !cent || !qi || !ki || !out || D <= 0 || (dt != 0 && dt != 1))
        return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < n; ++p)
        out[p] = dist2(emb, cent, qi[p], ki[p], D, dt);
    return ORACLE_OK;
}

/*
 * centroid_ids[i] = argmin_k ||q_i - c_k||^2, scanning k upward and replacing
 * the incumbent only on a strictly smaller distance, so ties keep the lowest
 * index and a NaN distance never wins (a row of NaNs yields 0).
 * If `eligible` is non-NULL, centroids with eligible[k] == 0 are skipped
 * (search over retained topics only); if none is eligible the id is 0.
 * best_d2 / second_d2 (optional) receive the smallest and second smallest
 * distance seen, for the near-tie band of the parity tests.
 */
int moin_oracle_route(const void *emb, const void *cent, int64_t N, int32_t K,
                      int32_t D, int dt, const uint8_t *eligible,
                      int32_t *centroid_ids, double *best_d2,
                      double *second_d2)
{
    if (N < 0 || K <= 0 || D <= 0 || (dt != 0 && dt != 1)) return ORACLE_EINVAL;
    if (N == 0) return ORACLE_OK;
    if (!emb || !cent || !centroid_ids) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        double best = INFINITY, second = INFINITY;
        int32_t best_k = 0;
        for (int32_t k = 0; k < K; ++k) {
            if (eligible && !eligible[k]) continue;
            double d = dist2(emb, cent, i, k, D, dt);
            if (d < best) {
                second = best;
                best = d;
                best_k = k;
            } else if (d < second) {
                second = d;
            }
        }
        centroid_ids[i] = best_k;
        if (best_d2) best_d2[i] = best;
        if (second_d2) second_d2[i] = second;
    }
    return ORACLE_OK;
}

/*
 * The k nearest centroids of every query ("Future Works", creating new experts
 * on the fly: a query on the boundary of several clusters may need several
 * adapters): ids[i, 0..k) are the centroid indices in order of increasing
 * ||q_i - c||^2, equal distances in order of increasing index; d2[i, m] the
 * distances (fp64).  Column 0 is moin_oracle_route's answer.  With fewer than k
 * eligible centroids the remaining columns hold -1 / +inf.  A NaN distance
 * never enters the list.
 */
int moin_oracle_route_topk(const void *emb, const void *cent, int64_t N, int32_t K,
                           int32_t D, int dt, const uint8_t *eligible, int32_t k,
                           int32_t *ids, double *d2)
{
    if (N < 0 || K <= 0 || D <= 0 || k <= 0 || (dt != 0 && dt != 1)) return ORACLE_EINVAL;
    if (N == 0) return ORACLE_OK;
    if (!emb || !cent || !ids || !d2) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        int32_t *li = ids + (size_t)i * k;
        double *ld = d2 + (size_t)i * k;
        int32_t n = 0;                       /* entries in the list so far */
        for (int32_t m = 0; m < k; ++m) {
            li[m] = -1;
            ld[m] = INFINITY;
        }
        for (int32_t c = 0; c < K; ++c) {
            if (eligible && !eligible[c]) continue;
            double d = dist2(emb, cent, i, c, D, dt);
            if (!(d == d)) continue;
            /* c is larger than every index in the list: it goes behind its equals */
            int32_t pos = n;
            while (pos > 0 && d < ld[pos - 1]) --pos;
            if (pos >= k) continue;
            int32_t last = n < k ? n : k - 1;
            for (int32_t m = last; m > pos; --m) {
                li[m] = li[m - 1];
                ld[m] = ld[m - 1];
            }
            li[pos] = c;
            ld[pos] = d;
            if (n < k) ++n;
        }
    }
    return ORACLE_OK;
}

/* expert_ids[i] = slot_of_centroid[centroid_ids[i]]; -1 marks a topic whose
 * adapter was never trained, i.e. "use the base model alone". */
int moin_oracle_slot_map(const int32_t *centroid_ids, int64_t N,
                         const int32_t *slot_of_centroid, int32_t K,
                         int32_t *expert_ids)
{
    if (N < 0 || K <= 0) return ORACLE_EINVAL;
    if (N == 0) return ORACLE_OK;
    if (!centroid_ids || !slot_of_centroid || !expert_ids) return ORACLE_EINVAL;
    for (int64_t i = 0; i < N; ++i) {
        int32_t c = centroid_ids[i];
        if (c < 0 || c >= K) return ORACLE_EINVAL;
        expert_ids[i] = slot_of_centroid[c];
    }
    return ORACLE_OK;
}

/* counts[k] = number of i with ids[i] == k.  counts is overwritten. */
int moin_oracle_histogram(const int32_t *ids, int64_t N, int32_t K,
                          int64_t *counts)
{
    if (N < 0 || K <= 0 || !counts) return ORACLE_EINVAL;
    for (int32_t k = 0; k < K; ++k) counts[k] = 0;
    if (N == 0) return ORACLE_OK;
    if (!ids) return ORACLE_EINVAL;
    for (int64_t i = 0; i < N; ++i) {
        if (ids[i] < 0 || ids[i] >= K) return ORACLE_EINVAL;
        counts[ids[i]] += 1;
    }
    return ORACLE_OK;
}

/* ---- routed LoRA linear ---------------------------------------------- */

/*
 * "Future Works", better adapters: an activation function between the two LoRA
 * linear layers.  The paper names none; these are the textbook definitions.
 *   0  identity (the paper's adapter)      2  SiLU  v / (1 + exp(-v))
 *   1  ReLU  max(v, 0)                     3  GELU  v/2 (1 + erf(v / sqrt 2))
 */
enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_RELU = 1, ORACLE_ACT_SILU = 2, ORACLE_ACT_GELU = 3 };

static double adapter_activation(double v, int32_t activation)
{
    switch (activation) {
    case ORACLE_ACT_RELU: return v > 0.0 ? v : 0.0;
    case ORACLE_ACT_SILU: return v / (1.0 + exp(-v));
    case ORACLE_ACT_GELU: return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));
    default: return v;
    }
}

/*
 * y[p, :] for the tokens listed in rows[0..n_rows) (rows == NULL: all T
 * tokens, n_rows must then equal T).  For a token t that lies in sequence s
 * with e = expert_ids[s]:
 *     base_o = sum_i W[o,i] x[t,i]
 *     u_j    = sum_i A[e,j,i] x[t,i]           (e >= 0 only)
 *     y[t,o] = base_o + scale * sum_j B[e,o,j] u_j
 * and y[t,o] = base_o when e == -1.  u is never rounded.
 * rank_of_expert (may be NULL): "Future Works", adaptive rank per topic -- expert
 * e uses only its first rank_of_expert[e] rows of A[e] and columns of B[e]
 * (0 <= rank <= r); the stacks keep their [E, r, ...] shape and whatever lies
 * beyond an expert's rank is never read.
 * activation (see above; 0 = the paper's linear adapter): applied to u, so
 *     y[t,o] = base_o + scale * sum_j B[e,o,j] act(u_j).
 * x, W, A_stack, B_stack hold bf16 bit patterns; y is fp64, n_rows x d_out.
 * work: caller-provided temporaries, work_slots * (d_in + r) doubles; each
 * OpenMP thread (at most work_slots of them) keeps its widened token and its
 * u vector in its own slot.
 */
int moin_oracle_lora_linear(const uint16_t *x, const int32_t *seq_offsets,
                            const int32_t *expert_ids, int32_t S, int64_t T,
                            const uint16_t *W, const uint16_t *A_stack,
                            const uint16_t *B_stack, int32_t E, int32_t d_in,
                            int32_t d_out, int32_t r, double scale,
                            const int32_t *rank_of_expert, int32_t activation,
                            const int64_t *rows, int64_t n_rows, double *y,
                            double *work, int32_t work_slots)
{
    if (S < 0 || T < 0 || d_in <= 0 || d_out <= 0 || r < 0 || E < 0 ||
        n_rows < 0 || work_slots <= 0 || activation < ORACLE_ACT_NONE || activation > ORACLE_ACT_GELU)
        return ORACLE_EINVAL;
    if (n_rows == 0) return ORACLE_OK;
    if (!x || !seq_offsets || !W || !y || !work) return ORACLE_EINVAL;
    if (S > 0 && !expert_ids) return ORACLE_EINVAL;
    if (!rows && n_rows != T) return ORACLE_EINVAL;
    if (seq_offsets[0] != 0 || seq_offsets[S] != T) return ORACLE_EINVAL;
    for (int32_t s = 0; s < S; ++s) {
        if (seq_offsets[s + 1] < seq_offsets[s]) return ORACLE_EINVAL;
        if (expert_ids[s] < -1 || expert_ids[s] >= E) return ORACLE_EINVAL;
        if (expert_ids[s] >= 0 && (!A_stack || !B_stack)) return ORACLE_EINVAL;
        if (expert_ids[s] >= 0 && rank_of_expert &&
            (rank_of_expert[expert_ids[s]] < 0 || rank_of_expert[expert_ids[s]] > r))
            return ORACLE_EINVAL;
    }
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(work_slots)
    for (int64_t p = 0; p < n_rows; ++p) {
        int64_t t = rows ? rows[p] : p;
        if (t < 0 || t >= T) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        /* which sequence holds token t: first s with seq_offsets[s+1] > t */
        int32_t s = 0;
        while (s < S && seq_offsets[s + 1] <= t) ++s;
        int32_t e = expert_ids[s];
        int slot = 0;
#ifdef _OPENMP
        extern int omp_get_thread_num(void);
        slot = omp_get_thread_num();
#endif
        double *xt = work + (size_t)slot * ((size_t)d_in + (size_t)r);
        double *u = xt + d_in;
        for (int32_t i = 0; i < d_in; ++i)
            xt[i] = bf16_to_f64(x[(size_t)t * d_in + i]);
        const int32_t re = (e >= 0 && rank_of_expert) ? rank_of_expert[e] : r;
        if (e >= 0) {
            const uint16_t *A = A_stack + (size_t)e * r * d_in;
            for (int32_t j = 0; j < re; ++j) {
                double acc = 0.0;
                for (int32_t i = 0; i < d_in; ++i)
                    acc += bf16_to_f64(A[(size_t)j * d_in + i]) * xt[i];
                u[j] = adapter_activation(acc, activation);
            }
        }
        for (int32_t o = 0; o < d_out; ++o) {
            double base = 0.0;
            for (int32_t i = 0; i < d_in; ++i)
                base += bf16_to_f64(W[(size_t)o * d_in + i]) * xt[i];
            double out = base;
            if (e >= 0) {
                const uint16_t *B = B_stack + (size_t)e * d_out * r;
                double lora = 0.0;
                for (int32_t j = 0; j < re; ++j)
                    lora += bf16_to_f64(B[(size_t)o * r + j]) * u[j];
                out = base + scale * lora;
            }
            y[(size_t)p * d_out + o] = out;
        }
    }
    return bad ? ORACLE_EINVAL : ORACLE_OK;
}

/* ---- merged adapters --------------------------------------------------- */

/* fp32 -> bf16 bits, round to nearest even (finite inputs). */
static uint16_t f32_to_bf16_rne(float f)
{
    union { uint32_t u; float f; } v;
    v.f = f;
    uint32_t lsb = (v.u >> 16) & 1u;
    return (uint16_t)((v.u + 0x7FFFu + lsb) >> 16);
}

/*
 * "Future Works", creating new experts on the fly: an adapter that stands for a
 * weighted set of existing ones, sum_m w_m W_b[e_m] W_a[e_m], written as ONE
 * adapter of rank n * r by concatenation (exact up to the rounding of the scaled
 * W_b back to bf16):
 *     A_out[m * r + j, :] = A[e_m][j, :]
 *     B_out[:, m * r + j] = bf16(w_m * B[e_m][:, j])    product taken in fp32
 * for m < n, j < r; an id of -1 contributes zeros; rows of A_out / columns of
 * B_out from n * r up to r_out are zero.  A_stack [E, r, d_in], B_stack
 * [E, d_out, r], A_out [r_out, d_in], B_out [d_out, r_out]: bf16 bits.
 */
int moin_oracle_merge_adapters(const uint16_t *A_stack, const uint16_t *B_stack, int32_t E,
                               int32_t r, int32_t d_in, int32_t d_out, const int32_t *ids,
                               const float *weights, int32_t n, int32_t r_out,
                               uint16_t *A_out, uint16_t *B_out)
{
    if (E <= 0 || r <= 0 || d_in <= 0 || d_out <= 0 || n < 0 || r_out < 0) return ORACLE_EINVAL;
    if ((int64_t)n * r > r_out) return ORACLE_EINVAL;
    if (!A_stack || !B_stack || !A_out || !B_out || (n > 0 && (!ids || !weights))) return ORACLE_EINVAL;
    for (int32_t m = 0; m < n; ++m)
        if (ids[m] < -1 || ids[m] >= E) return ORACLE_EINVAL;
    for (size_t q = 0; q < (size_t)r_out * d_in; ++q) A_out[q] = 0;
    for (size_t q = 0; q < (size_t)d_out * r_out; ++q) B_out[q] = 0;
    for (int32_t m = 0; m < n; ++m) {
        const int32_t e = ids[m];
        if (e < 0) continue;
        for (int32_t j = 0; j < r; ++j)
            for (int32_t i = 0; i < d_in; ++i)
                A_out[((size_t)m * r + j) * d_in + i] = A_stack[((size_t)e * r + j) * d_in + i];
        for (int32_t o = 0; o < d_out; ++o)
            for (int32_t j = 0; j < r; ++j) {
                const float b = (float)bf16_to_f64(B_stack[((size_t)e * d_out + o) * r + j]);
                B_out[(size_t)o * r_out + (size_t)m * r + j] = f32_to_bf16_rne(weights[m] * b);
            }
    }
    return ORACLE_OK;
}

/* ---- MX (microscaled) FP8 base operands -------------------------------- */

/* Value of an FP8 E4M3 code (OCP 8-bit floating point specification): 1 sign
 * bit, 4 exponent bits with bias 7, 3 mantissa bits; exponent field 0 holds
 * the subnormals m/8 * 2^-6; there are no infinities and S.1111.111 is NaN. */
static double e4m3_to_f64(uint8_t c)
{
    const int sign = c >> 7, ef = (c >> 3) & 15, m = c & 7;
    double v;
    if (ef == 15 && m == 7) return NAN;
    if (ef == 0) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, ef - 7);
    return sign ? -v : v;
}

/* Nearest E4M3 code of a finite value: round to nearest, ties to the code with
 * an even mantissa, magnitudes beyond the largest finite value (448) saturate
 * to it.  Written as a search over all 127 finite magnitudes so that the
 * rounding rule is the definition itself and not a bit trick. */
static uint8_t f64_to_e4m3(double v)
{
    const uint8_t sign = signbit(v) ? 0x80 : 0;
    const double a = fabs(v);
    int best = 0;
    double best_err = a;                       /* code 0 is the value 0 */
    for (int c = 1; c <= 0x7E; ++c) {
        const double err = fabs(e4m3_to_f64((uint8_t)c) - a);
        if (err < best_err || (err == best_err && (c & 1) == 0)) {
            best = c;
            best_err = err;
        }
    }
    return (uint8_t)(sign | best);
}

/* Shared scale of one block (MX v1.0, conversion of a vector to an MX block):
 * the largest power of two not above the block's largest magnitude, divided by
 * the largest power of two of the element format (2^8 for E4M3), stored as the
 * biased exponent byte E (scale = 2^(E-127)), kept inside 0..254.  A block of
 * zeros takes scale 1 (E = 127); the specification leaves that case open. */
static uint8_t mx_block_scale(const double *v, int n)
{
    double amax = 0.0;
    for (int i = 0; i < n; ++i)
        if (fabs(v[i]) > amax) amax = fabs(v[i]);
    if (amax == 0.0) return 127;
    int ex;
    (void)frexp(amax, &ex);                    /* amax = f * 2^ex, 0.5 <= f < 1 */
    int E = (ex - 1) - 8 + 127;                /* floor(log2 amax) - emax + bias */
    if (E < 0) E = 0;
    if (E > 254) E = 254;
    return (uint8_t)E;
}

#define MX_BLOCK 32

/* Quantises rows x cols finite bf16 values (cols a multiple of 32) to MXFP8:
 * codes[rows, cols] E4M3 bytes and scales[rows, cols/32] E8M0 bytes, the
 * element being the rounded quotient value / scale. */
int moin_oracle_mx_quantize(const uint16_t *src, int64_t rows, int32_t cols,
                            uint8_t *codes, uint8_t *scales)
{
    if (rows < 0 || cols <= 0 || cols % MX_BLOCK) return ORACLE_EINVAL;
    if (rows == 0) return ORACLE_OK;
    if (!src || !codes || !scales) return ORACLE_EINVAL;
    const int32_t nb = cols / MX_BLOCK;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i)
        for (int32_t b = 0; b < nb; ++b) {
            double v[MX_BLOCK];
            for (int k = 0; k < MX_BLOCK; ++k) {
                v[k] = bf16_to_f64(src[(size_t)i * cols + (size_t)b * MX_BLOCK + k]);
                if (!isfinite(v[k])) {
#pragma omp atomic write
                    bad = 1;
                    v[k] = 0.0;
                }
            }
            const uint8_t E = mx_block_scale(v, MX_BLOCK);
            scales[(size_t)i * nb + b] = E;
            for (int k = 0; k < MX_BLOCK; ++k)
                codes[(size_t)i * cols + (size_t)b * MX_BLOCK + k] =
                    f64_to_e4m3(ldexp(v[k], 127 - (int)E));
        }
    return bad ? ORACLE_EINVAL : ORACLE_OK;
}

/* out[i, j] = value(codes[i, j]) * 2^(scales[i, j / 32] - 127), exact in fp64. */
int moin_oracle_mx_dequantize(const uint8_t *codes, const uint8_t *scales, int64_t rows,
                              int32_t cols, double *out)
{
    if (rows < 0 || cols <= 0 || cols % MX_BLOCK) return ORACLE_EINVAL;
    if (rows == 0) return ORACLE_OK;
    if (!codes || !scales || !out) return ORACLE_EINVAL;
    const int32_t nb = cols / MX_BLOCK;
    for (int64_t i = 0; i < rows; ++i)
        for (int32_t j = 0; j < cols; ++j)
            out[(size_t)i * cols + j] = ldexp(e4m3_to_f64(codes[(size_t)i * cols + j]),
                                              (int)scales[(size_t)i * nb + j / MX_BLOCK] - 127);
    return ORACLE_OK;
}

/*
 * The routed LoRA linear layer on a quantised base: like
 * moin_oracle_lora_linear, but the base term is
 *     base_o = sum_i Wd[o,i] xd[t,i]
 * with Wd the dequantised MXFP8 weight (Wq codes [d_out, d_in], Ws scales
 * [d_out, d_in/32]) and xd the token's activations after a round trip through
 * the same MXFP8 quantisation; the adapter term still uses the bf16 x:
 *     y[t,o] = base_o + scale * sum_j B[e,o,j] act(sum_i A[e,j,i] x[t,i]).
 * work: work_slots * (2 * d_in + r) doubles.
 */
int moin_oracle_lora_linear_mx(const uint16_t *x, const int32_t *seq_offsets,
                               const int32_t *expert_ids, int32_t S, int64_t T,
                               const uint8_t *Wq, const uint8_t *Ws, const uint16_t *A_stack,
                               const uint16_t *B_stack, int32_t E, int32_t d_in,
                               int32_t d_out, int32_t r, double scale,
                               const int32_t *rank_of_expert, int32_t activation,
                               const int64_t *rows, int64_t n_rows, double *y,
                               double *work, int32_t work_slots)
{
    if (S < 0 || T < 0 || d_in <= 0 || d_in % MX_BLOCK || d_out <= 0 || r < 0 || E < 0 ||
        n_rows < 0 || work_slots <= 0 || activation < ORACLE_ACT_NONE || activation > ORACLE_ACT_GELU)
        return ORACLE_EINVAL;
    if (n_rows == 0) return ORACLE_OK;
    if (!x || !seq_offsets || !Wq || !Ws || !y || !work) return ORACLE_EINVAL;
    if (S > 0 && !expert_ids) return ORACLE_EINVAL;
    if (!rows && n_rows != T) return ORACLE_EINVAL;
    if (seq_offsets[0] != 0 || seq_offsets[S] != T) return ORACLE_EINVAL;
    for (int32_t s = 0; s < S; ++s) {
        if (seq_offsets[s + 1] < seq_offsets[s]) return ORACLE_EINVAL;
        if (expert_ids[s] < -1 || expert_ids[s] >= E) return ORACLE_EINVAL;
        if (expert_ids[s] >= 0 && (!A_stack || !B_stack)) return ORACLE_EINVAL;
        if (expert_ids[s] >= 0 && rank_of_expert &&
            (rank_of_expert[expert_ids[s]] < 0 || rank_of_expert[expert_ids[s]] > r))
            return ORACLE_EINVAL;
    }
    const int32_t nb = d_in / MX_BLOCK;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(work_slots)
    for (int64_t p = 0; p < n_rows; ++p) {
        int64_t t = rows ? rows[p] : p;
        if (t < 0 || t >= T) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        int32_t s = 0;
        while (s < S && seq_offsets[s + 1] <= t) ++s;
        int32_t e = expert_ids[s];
        int slot = 0;
#ifdef _OPENMP
        extern int omp_get_thread_num(void);
        slot = omp_get_thread_num();
#endif
        double *xt = work + (size_t)slot * (2 * (size_t)d_in + (size_t)r);
        double *xd = xt + d_in;
        double *u = xd + d_in;
        for (int32_t i = 0; i < d_in; ++i)
            xt[i] = bf16_to_f64(x[(size_t)t * d_in + i]);
        /* the token through the quantiser and back */
        for (int32_t b = 0; b < nb; ++b) {
            const double *v = xt + (size_t)b * MX_BLOCK;
            const uint8_t Eb = mx_block_scale(v, MX_BLOCK);
            for (int k = 0; k < MX_BLOCK; ++k)
                xd[(size_t)b * MX_BLOCK + k] =
                    ldexp(e4m3_to_f64(f64_to_e4m3(ldexp(v[k], 127 - (int)Eb))), (int)Eb - 127);
        }
        const int32_t re = (e >= 0 && rank_of_expert) ? rank_of_expert[e] : r;
        if (e >= 0) {
            const uint16_t *A = A_stack + (size_t)e * r * d_in;
            for (int32_t j = 0; j < re; ++j) {
                double acc = 0.0;
                for (int32_t i = 0; i < d_in; ++i)
                    acc += bf16_to_f64(A[(size_t)j * d_in + i]) * xt[i];
                u[j] = adapter_activation(acc, activation);
            }
        }
        for (int32_t o = 0; o < d_out; ++o) {
            double base = 0.0;
            for (int32_t i = 0; i < d_in; ++i)
                base += ldexp(e4m3_to_f64(Wq[(size_t)o * d_in + i]),
                              (int)Ws[(size_t)o * nb + i / MX_BLOCK] - 127) * xd[i];
            double out = base;
            if (e >= 0) {
                const uint16_t *B = B_stack + (size_t)e * d_out * r;
                double lora = 0.0;
                for (int32_t j = 0; j < re; ++j)
                    lora += bf16_to_f64(B[(size_t)o * r + j]) * u[j];
                out = base + scale * lora;
            }
            y[(size_t)p * d_out + o] = out;
        }
    }
    return bad ? ORACLE_EINVAL : ORACLE_OK;
}

/* ---- K-means centre update -------------------------------------------- */

static double emb_at(const void *a, size_t idx, int dt)
{
    return dt == 0 ? (double)((const float *)a)[idx] : bf16_to_f64(((const uint16_t *)a)[idx]);
}

/* new_c[k] = mean of emb[i] over {i : ids[i] == k} (fp64 sums in index order),
 * old_c[k] when the set is empty; counts[k] = set size; *inertia = sum_i
 * ||emb[i] - old_c[ids[i]]||^2 summed in index order.  ids outside [0, K) are
 * an error.  Single-threaded on purpose: one fixed summation order. */
int moin_oracle_kmeans_update(const void *emb, const int32_t *ids, int64_t N,
                              const void *old_c, int32_t K, int32_t D, int dt,
                              double *new_c, int64_t *counts, double *inertia)
{
    if (N < 0 || K <= 0 || D <= 0 || !old_c || !new_c || !counts) return ORACLE_EINVAL;
    if (N > 0 && (!emb || !ids)) return ORACLE_EINVAL;
    for (int32_t k = 0; k < K; ++k) {
        counts[k] = 0;
        for (int32_t j = 0; j < D; ++j) new_c[(size_t)k * D + j] = 0.0;
    }
    double total = 0.0;
    for (int64_t i = 0; i < N; ++i) {
        const int32_t k = ids[i];
        if (k < 0 || k >= K) return ORACLE_EINVAL;
        counts[k] += 1;
        double d2 = 0.0;
        for (int32_t j = 0; j < D; ++j) {
            const double q = emb_at(emb, (size_t)i * D + j, dt);
            const double diff = q - emb_at(old_c, (size_t)k * D + j, dt);
            new_c[(size_t)k * D + j] += q;
            d2 += diff * diff;
        }
        total += d2;
    }
    for (int32_t k = 0; k < K; ++k)
        for (int32_t j = 0; j < D; ++j) {
            if (counts[k] > 0) new_c[(size_t)k * D + j] /= (double)counts[k];
            else new_c[(size_t)k * D + j] = emb_at(old_c, (size_t)k * D + j, dt);
        }
    if (inertia) *inertia = total;
    return ORACLE_OK;
}

/* Section 4 "Implementation details": clusters that stay extremely small are
 * dropped and the remaining ones get an adapter each.  The paper names no
 * threshold, so it is an input: a cluster is kept iff it has at least min_count
 * members; kept clusters are numbered 0, 1, ... in ascending cluster index (the
 * adapter slots), dropped ones get -1.  Returns the number kept. */
int moin_oracle_retain_clusters(const int64_t *counts, int32_t K, int64_t min_count,
                                int32_t *slot_of_centroid)
{
    if (K <= 0 || !counts || !slot_of_centroid) return ORACLE_EINVAL;
    int32_t kept = 0;
    for (int32_t k = 0; k < K; ++k) {
        if (counts[k] >= min_count) slot_of_centroid[k] = kept++;
        else slot_of_centroid[k] = -1;
    }
    return kept;
}

int moin_oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
