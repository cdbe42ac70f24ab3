// Nearest-topic routing (Section 3.3: nearest-neighbour search of the query
// embedding over the topic embeddings; Section 3.1: those are the K-means
// centres) and the per-topic histogram (Figure 3).
//
// bf16 path: argmin_k ||q - c_k||^2 = argmin_k (||c_k||^2 - 2 q.c_k); the dot
// products are one dense bf16 MFMA contraction [K x D] . [D x N].  Centroids
// are the MFMA row operand and queries the column operand, so one lane holds
// 16 centroid scores of a single query per accumulator and the running
// (score, index) minimum lives in registers; nothing but the winning index
// ever leaves the workgroup.  A workgroup owns 256 queries and sweeps all
// centroid tiles in ascending order, which makes "lowest index wins a tie"
// fall out of a strict '<'.
// fp32 path: small inputs only; direct sum of squared differences in fp32.
#include <type_traits>

#include "gemm_core.h"
#include "kernels.h"
#include "plan_body.h"

namespace moin {

using CfgRoute = GemmCore<256, 256, 64, 4, 2>;      // rows: centroids, cols: queries; any D % 8 == 0
using CfgRouteDma = DmaCore<256, 256, 64, 4, 2, 2>;  // D % 64 == 0
using CfgRouteSmall = DmaCore<64, 64, 64, 2, 2, 6>;  // small batches: one (centroid chunk, query tile) per workgroup

struct RouteKParams {
    const char *emb, *cent;
    const float *cnorm;   // [K padded to a multiple of 256]; +inf for excluded / padding
    const float *cinit;   // [same]: -||c||^2 / 2, -inf for excluded / padding
    const int *slot;
    int *cid;
    int *expert_ids;
    unsigned long long *best;
    int *arrivals;        // small-batch kernel
    int *counts;          // small batches only: tallied by the finishing workgroup (zeroed beforehand)
    int64_t N;
    int K, D;
    int group;            // streaming kernel: workgroups that share one query tile
    int self_clean;       // small-batch kernel: best / arrivals are clean on entry and are left clean
                          // (the finishing workgroup resets them and zeroes counts before its tally)
    // small-batch kernel, optional: the finishing workgroup goes on to group the routed batch by
    // expert (queries = the batch's sequences), so that routing and grouping are one launch
    int with_plan;
    PlanView plan;
    const int *seq_offsets, *rank_of_expert;
    int *err_word;
};

__device__ __forceinline__ bool lex_less(float v, int i, float bv, int bi)
{
    return (v < bv) || (v == bv && i < bi);
}

// Folds one finished centroid tile into the running per-lane minima.  A lane
// holds, per accumulator, 16 centroid scores of one query in ascending
// centroid order, so a strict '<' keeps the lowest index among equal scores.
template <class C>
__device__ __forceinline__ void fold_scores(const typename C::Acc &acc, const float *cnorm_tile,
                                            int idx_tile, float (&bestv)[C::FN], int (&besti)[C::FN])
{
    const int lane = threadIdx.x & 63;
    const int wm = (threadIdx.x >> 6) / C::WN;
    const float *cn = cnorm_tile + wm * C::WTM + 4 * (lane >> 5);
#pragma unroll
    for (int i = 0; i < C::FM; ++i) {
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            const f32x4_t c4 = *reinterpret_cast<const f32x4_t *>(cn + i * 32 + e4 * 8);
            const int idx0 = idx_tile + wm * C::WTM + i * 32 + e4 * 8 + 4 * (lane >> 5);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
#pragma unroll
                for (int j = 0; j < C::FN; ++j) {
                    const float s = fmaf(-2.f, acc.v[i][j][e4 * 4 + q], c4[q]);
                    const bool lt = s < bestv[j];
                    bestv[j] = lt ? s : bestv[j];
                    besti[j] = lt ? idx0 + q : besti[j];
                }
            }
        }
    }
}

template <class C>
__global__ __launch_bounds__(C::NT) void route_kernel(RouteKParams p)
{
    extern __shared__ __align__(16) char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int64_t q0 = (int64_t)blockIdx.x * C::BN;
    const int nq = (int)min((int64_t)C::BN, p.N - q0);
    const uint32_t ld = (uint32_t)p.D * 2u;
    const int nkb = (p.D + C::BK - 1) / C::BK;
    const int nct = (p.K + C::BM - 1) / C::BM;
    const char *qb = p.emb + q0 * (int64_t)ld;

    float bestv[C::FN];
    int besti[C::FN];
#pragma unroll
    for (int j = 0; j < C::FN; ++j) {
        bestv[j] = __builtin_inff();
        besti[j] = 0;
    }

    typename C::Acc acc;
    C::zero(acc);
    const int total = nct * nkb;

    if constexpr (C::IS_DMA) {
        static_assert(C::NS == 2, "stage bookkeeping below assumes two stages");
        const auto lq = C::template make_lanes<C::B_I>(nq);
        // the last centroid tile may be short: its lanes clamp to the last valid row
        const auto lc_full = C::template make_lanes<C::A_I>(C::BM);
        const auto lc_last = C::template make_lanes<C::A_I>(p.K - (nct - 1) * C::BM);
#define MOIN_ROUTE_ISSUE(blk, stage)                                                         \
    do {                                                                                     \
        const int ct_ = (blk) / nkb, kb_ = (blk) - ct_ * nkb;                                \
        typename C::template Lanes<C::A_I> lc_;                                              \
        _Pragma("unroll") for (int q_ = 0; q_ < C::A_I; ++q_) {                              \
            lc_.row[q_] = (ct_ == nct - 1) ? lc_last.row[q_] : lc_full.row[q_];              \
            lc_.c16[q_] = lc_full.c16[q_];                                                   \
        }                                                                                    \
        C::issue((stage), p.cent + (int64_t)ct_ * C::BM * ld, ld, lc_, qb, ld, lq,           \
                 (uint32_t)kb_ * (C::BK * 2));                                               \
    } while (0)
        MOIN_ROUTE_ISSUE(0, smem);
        int kb = 0, ct = 0;
        for (int it = 0; it < total; ++it) {
            wait_vm_then_barrier<0>();
            if (it + 1 < total) MOIN_ROUTE_ISSUE(it + 1, smem + ((it + 1) & 1) * C::STAGE_BYTES);
            C::compute_stage(smem + (it & 1) * C::STAGE_BYTES, acc);
            if (++kb == nkb) {
                fold_scores<C>(acc, p.cnorm + ct * C::BM, ct * C::BM, bestv, besti);
                C::zero(acc);
                kb = 0;
                ++ct;
            }
        }
        __syncthreads();
#undef MOIN_ROUTE_ISSUE
    } else {
        const auto vq = C::template make_view<C::B_CH>(qb, ld, nq);
        typename C::Stage g;
        auto issue = [&](int it) __attribute__((always_inline)) {
            const int ct = it / nkb, kb = it - ct * nkb;
            const int crow = ct * C::BM;
            const auto vc = C::template make_view<C::A_CH>(p.cent + (int64_t)crow * ld, ld,
                                                           min(C::BM, p.K - crow));
            C::load_stage(g, vc, vq, (uint32_t)kb * (C::BK * 2), ld);
        };
        issue(0);
        C::store_stage(smem, g);
        __syncthreads();
        int kb = 0, ct = 0;
        for (int it = 0; it < total; ++it) {
            char *cur = smem + (it & 1) * C::STAGE_BYTES;
            char *nxt = smem + ((it + 1) & 1) * C::STAGE_BYTES;
            const bool more = it + 1 < total;
            if (more) issue(it + 1);
            C::compute_stage(cur, acc);
            if (++kb == nkb) {
                fold_scores<C>(acc, p.cnorm + ct * C::BM, ct * C::BM, bestv, besti);
                C::zero(acc);
                kb = 0;
                ++ct;
            }
            if (more) C::store_stage(nxt, g);
            __syncthreads();
        }
    }

    // merge the two lane halves (rows 4*(lane>>5) interleave), then the WM waves
#pragma unroll
    for (int j = 0; j < C::FN; ++j) {
        const float ov = __shfl_xor(bestv[j], 32);
        const int oi = __shfl_xor(besti[j], 32);
        if (lex_less(ov, oi, bestv[j], besti[j])) {
            bestv[j] = ov;
            besti[j] = oi;
        }
    }
    float *sv = reinterpret_cast<float *>(smem);                  // [WM][BN]
    int *si = reinterpret_cast<int *>(smem + C::WM * C::BN * 4);  // [WM][BN]
    if (lane < 32) {
#pragma unroll
        for (int j = 0; j < C::FN; ++j) {
            const int col = wn * C::WTN + j * 32 + lane;
            sv[wm * C::BN + col] = bestv[j];
            si[wm * C::BN + col] = besti[j];
        }
    }
    __syncthreads();
    for (int col = threadIdx.x; col < nq; col += C::NT) {
        float bv = sv[col];
        int bi = si[col];
#pragma unroll
        for (int w = 1; w < C::WM; ++w) {
            const float v = sv[w * C::BN + col];
            const int i = si[w * C::BN + col];
            if (lex_less(v, i, bv, bi)) {
                bv = v;
                bi = i;
            }
        }
        if (p.cid) p.cid[q0 + col] = bi;
        if (p.expert_ids) p.expert_ids[q0 + col] = p.slot ? p.slot[bi] : bi;
    }
}

// Order-preserving map of a finite float (or +-inf) to an unsigned integer.
__device__ __forceinline__ uint32_t float_order_key(float f)
{
    const uint32_t u = f32_bits(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Large batches, D a multiple of 64: same tiling as route_kernel, with the
// block pipeline of the prefill linear kernel -- two direct-to-LDS stages, the
// fragments of a k-step read under the MFMAs of the one before, the block barrier
// placed between the block's two k-steps (the second one's fragments are in
// registers by then) and the first fragments of the next block read during the
// second.  Eight waves, two per SIMD, each a 64 x 128 patch of
// v_mfma_f32_16x16x32_bf16 accumulators: while one wave folds a finished tile the
// other keeps the matrix core busy.  The blocks of all centroid tiles form one
// stream; a finished tile is folded into the running best between two blocks.
// argmin ||q - c||^2 is taken as argmax (q.c - ||c||^2 / 2): the first MFMA of a
// tile takes -||c||^2 / 2 as its addend, so accumulators are never cleared and the
// fold is a compare and two selects per score.  The position inside the tile
// travels as a small code (tile, accumulator row block, element) that is the same
// for all lanes, i.e. a scalar operand.
__global__ __launch_bounds__(CfgRouteDma::NT) void route_stream_kernel(RouteKParams p)
{
    using C = CfgRouteDma;
    extern __shared__ __align__(16) char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = uniform(threadIdx.x >> 6);
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int g = lane >> 4;
    // `group` workgroups next to each other on one XCD share a query tile and
    // take every group-th centroid tile: the XCD's L2 then holds few query
    // tiles at a time, each fetched once for all of its workgroups, instead of
    // one tile per compute unit that falls out of the cache between two uses.
    const int G = p.group;
    const int slot = blockIdx.x >> 3;
    const int member = slot % G;
    const int64_t qtile = (int64_t)(slot / G) * 8 + (blockIdx.x & 7);
    const int64_t q0 = qtile * C::BN;
    if (q0 >= p.N) return;
    const int nq = (int)min((int64_t)C::BN, p.N - q0);
    const uint32_t ld = (uint32_t)p.D * 2u;
    const int nkb = p.D / C::BK;
    const int nct = (p.K + C::BM - 1) / C::BM;
    const int last_rows = p.K - (nct - 1) * C::BM;
    const char *qb = p.emb + q0 * (int64_t)ld;
    const int my_tiles = (nct - member + G - 1) / G;   // >= 1: G <= nct
    const int total = my_tiles * nkb;

    // DMA mapping (see DmaCore): instruction j of a wave fills tile rows
    // (wave*4 + j)*8 .. +8; only j's parity enters the chunk swizzle
    constexpr int LOADS = C::A_I;
    static_assert(C::A_I == 4 && C::B_I == 4 && C::KSTEPS == 4 && C::NS == 2, "pipeline shape");
    // Per-lane constants of the requests are worked out from the lane id at every use (through an
    // opaque copy): kept alive across the main loop they would be spilled around the accumulators,
    // and a spill's reload waits for every request in flight.
    auto fresh_lane = [&]() __attribute__((always_inline)) {
        int v = lane;
        asm volatile("; lane id, rematerialised" : "+v"(v));
        return v;
    };
    // requests of one block (centroid tile ct, contraction block kb): n = 0..3 centroid rows, 4..7 query rows.
    // The block's position along k is in the uniform base pointers; a request costs an add, a min and
    // a multiply-add besides itself.
    struct Fetch {
        const char *pc, *pq;
        uint32_t dma_row, c16a, c16b, c_last;
    };
    auto fetch_of = [&](int ct, int kb) __attribute__((always_inline)) {
        Fetch f;
        f.pc = p.cent + (int64_t)ct * C::BM * ld + kb * (C::BK * 2);
        f.pq = qb + kb * (C::BK * 2);
        f.c_last = (uint32_t)((ct == nct - 1) ? last_rows : C::BM) - 1u;
        const uint32_t ln = (uint32_t)fresh_lane();
        f.dma_row = (uint32_t)(wave * (LOADS * 8)) + (ln >> 3);
        f.c16a = ((ln & 7) ^ (ln >> 4)) * 16;   // even j; odd j: ^ 64
        f.c16b = f.c16a ^ 64u;
        return f;
    };
    auto issue_one = [&](const Fetch &f, char *stage, int n) __attribute__((always_inline)) {
        const int j = n & (LOADS - 1);
        const bool q = n >= LOADS;
        const uint32_t row = min(f.dma_row + 8u * j, q ? (uint32_t)(nq - 1) : f.c_last);
        const uint32_t off = __umul24(row, ld) + ((j & 1) ? f.c16b : f.c16a);
        __builtin_amdgcn_global_load_lds(MOIN_GPTR((q ? f.pq : f.pc) + off),
                                         MOIN_LPTR(stage + (q ? C::A_BYTES : 0) + (wave * LOADS + j) * 1024), 16, 0, 0);
    };
    auto issue = [&](int ct, int kb, char *stage) __attribute__((always_inline)) {
        const Fetch f = fetch_of(ct, kb);
#pragma unroll
        for (int n = 0; n < 2 * LOADS; ++n) issue_one(f, stage, n);
    };
    // -||c||^2 / 2 of a centroid tile (256 floats) into 1 KB of LDS behind the stages: one request of
    // wave 0; the accumulators of the tile's first k-step take their start values from there.  Two
    // such slots in turn: with one block per tile (D = 64) the next tile's values are requested while
    // other waves may still be reading this tile's.
    char *cbuf = smem + C::SMEM_BYTES;
    int tseq = 0;   // tiles done so far
    auto fetch_init = [&](int ct_, int slot) __attribute__((always_inline)) {
        if (wave == 0)
            __builtin_amdgcn_global_load_lds(MOIN_GPTR(reinterpret_cast<const char *>(p.cinit + ct_ * C::BM) + lane * 16),
                                             MOIN_LPTR(cbuf + slot * 1024), 16, 0, 0);
    };

    // MFMA operand of a lane (v_mfma_f32_16x16x32_bf16): row lane % 16 of a 16-row block, elements
    // 8 (lane / 16) .. + 8 of the k-step's 32, i.e. logical 16-byte chunk 4 ks + lane / 16 of the
    // row.  ONE set of fragments: a fragment is read again, for the next k-step, as soon as the last
    // MFMA that uses it has been issued (centroid fragment i after row i of the 4 x 8 grid of MFMAs,
    // query fragment j after the MFMA (3, j)), so the reads travel under the MFMAs that follow and
    // the second wave of the SIMD covers what is left.  (Two sets, as in the 32 x 32 x 16 form this
    // kernel had, do not fit beside 128 accumulator registers at two waves per SIMD; the narrower
    // instruction is worth it: on N(0,1) operands a loop of nothing but MFMAs sustains 13 % more
    // flops with it before the chip throttles.)
    constexpr int FM = C::WTM / 16, FN = C::WTN / 16;
    static_assert(FM == 4 && FN == 8 && C::BK == 64, "fragment grid of a wave");
    // (the swizzle of a row inside a 16-row block depends on lane % 16 only, and k-step 1 is k-step
    // 0's address ^ 64; like the requests' constants, the lane's offset is rematerialised per k-step)
    const int baseA = wm * C::WTM * C::ROWB, baseB = C::A_BYTES + wn * C::WTN * C::ROWB;
    bf16x8_t fa[FM], fb[FN];
    auto lane_off = [&](int ks) __attribute__((always_inline)) {
        const int ln = fresh_lane();
        return (((ln & 15) * C::ROWB) | ((((ln >> 4) ^ ((ln & 15) >> 1)) & 7) * 16)) ^ (ks * 64);
    };
    auto read_a = [&](const char *stage, int lo, int i) __attribute__((always_inline)) {
        fa[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(stage + baseA + i * 16 * C::ROWB + lo));
    };
    auto read_b = [&](const char *stage, int lo, int j) __attribute__((always_inline)) {
        fb[j] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(stage + baseB + j * 16 * C::ROWB + lo));
    };
    f32x4_t acc[FM][FN];
    // start values of a tile's accumulators: element e of accumulator (i, j) belongs to centroid row
    // wm*WTM + 16 i + 4 (lane / 16) + e of the tile
    // One k-step: the 4 x 8 MFMAs row by row.  FIRST: a tile's first k-step starts from
    // -||c||^2 / 2.  RELOAD: every fragment is read again from `stage` at k-step `ks` once it is free.
    auto kstep = [&](auto first_tag, auto reload_tag, const char *stage, int ks, auto issue_tag, const Fetch &f,
                     char *dst) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first_tag)::value, RELOAD = decltype(reload_tag)::value;
        constexpr bool ISSUE = decltype(issue_tag)::value;
        const int lo = lane_off(ks);
        const char *cmine = cbuf + (tseq & 1) * 1024 + (wm * C::WTM + 4 * (fresh_lane() >> 4)) * 4;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            f32x4_t ci = {0.f, 0.f, 0.f, 0.f};
            if (FIRST) ci = *reinterpret_cast<const f32x4_t *>(cmine + i * 64);
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], FIRST ? ci : acc[i][j], 0, 0, 0);
                if (RELOAD && i == FM - 1) {
                    read_b(stage, lo, j);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // the eight requests of the block two ahead, one after every third MFMA of the rows
                // that carry no query-fragment reads: together right behind the barrier they kept
                // both waves of a SIMD, which leave the barrier at the same time, off the matrix
                // core for as long as their issue takes
                if (ISSUE && i < FM - 1 && j % 3 == 1 && i * 3 + j / 3 < 2 * LOADS) {
                    issue_one(f, dst, i * 3 + j / 3);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (RELOAD) read_a(stage, lo, i);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    float bestv[FN];
    int bestc[FN];   // (tile << 5) | (accumulator row block i << 2) | element
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        bestv[j] = -__builtin_inff();
        bestc[j] = 0;
    }

    int kb = 0, ct = member;   // block being computed
    int pkb = 2, pct = member; // block to fetch next (two ahead)
    while (pkb >= nkb) {       // D = 64: one block per centroid tile
        pkb -= nkb;
        pct += G;
    }
    auto body = [&](int s, auto issue_tag, auto read_tag) __attribute__((always_inline)) {
        constexpr bool ISSUE = decltype(issue_tag)::value, READ = decltype(read_tag)::value;
        char *st_cur = smem + (s & 1) * C::STAGE_BYTES;
        const char *st_nxt = smem + ((s + 1) & 1) * C::STAGE_BYTES;
        // first k-step (its fragments are in registers), the second one's read behind it
        const Fetch none{};
        if (kb == 0) kstep(std::true_type{}, std::true_type{}, st_cur, 1, std::false_type{}, none, nullptr);
        else kstep(std::false_type{}, std::true_type{}, st_cur, 1, std::false_type{}, none, nullptr);
        // the tile's last block fetches the next tile's start values; they land
        // before this block's barrier (vmcnt(0))
        if (kb == nkb - 1 && ct + G < nct) fetch_init(ct + G, (tseq + 1) & 1);
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        // second k-step, the next block's first fragments and the requests for the block two ahead behind it
        if constexpr (ISSUE) {
            const Fetch f = fetch_of(pct, pkb);
            if (++pkb == nkb) {
                pkb = 0;
                pct += G;
            }
            kstep(std::false_type{}, std::true_type{}, st_nxt, 0, std::true_type{}, f, st_cur);
        } else if constexpr (READ) {
            kstep(std::false_type{}, std::true_type{}, st_nxt, 0, std::false_type{}, none, nullptr);
        } else {
            kstep(std::false_type{}, std::false_type{}, st_nxt, 0, std::false_type{}, none, nullptr);
        }
        if (++kb == nkb) {
            // a lane's scores come in ascending centroid order, so a strict '>'
            // keeps the lowest index among equal scores
            const int code0 = ct << 5;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        const float sc = acc[i][j][e];
                        const bool gt = sc > bestv[j];
                        bestv[j] = gt ? sc : bestv[j];
                        bestc[j] = gt ? code0 + (i * 4 + e) : bestc[j];
                    }
            kb = 0;
            ct += G;
            ++tseq;
        }
    };

    fetch_init(member, 0);
    issue(member, 0, smem);
    if (total > 1) {
        issue(nkb > 1 ? member : member + G, nkb > 1 ? 1 : 0, smem + C::STAGE_BYTES);
        wait_vm_then_barrier<2 * LOADS>();
    } else {
        wait_vm_then_barrier<0>();
    }
    {
        const int lo0 = lane_off(0);
#pragma unroll
        for (int i = 0; i < FM; ++i) read_a(smem, lo0, i);
#pragma unroll
        for (int j = 0; j < FN; ++j) read_b(smem, lo0, j);
    }
    int s = 0;
    for (; s < total - 2; ++s) body(s, std::true_type{}, std::true_type{});
    if (total > 1) {
        body(s, std::false_type{}, std::true_type{});
        ++s;
    }
    body(s, std::false_type{}, std::false_type{});
    __syncthreads();

    // position code -> centroid index; then merge the four lane groups (rows 4 * (lane / 16)
    // interleave) and the WM waves: higher score, else lower index
    int besti[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int c = bestc[j];
        besti[j] = (c >> 5) * C::BM + wm * C::WTM + 16 * ((c >> 2) & 7) + 4 * g + (c & 3);
#pragma unroll
        for (int sh = 16; sh <= 32; sh <<= 1) {
            const float ov = __shfl_xor(bestv[j], sh);
            const int oi = __shfl_xor(besti[j], sh);
            if (lex_less(-ov, oi, -bestv[j], besti[j])) {
                bestv[j] = ov;
                besti[j] = oi;
            }
        }
    }
    float *sv = reinterpret_cast<float *>(smem);
    int *si = reinterpret_cast<int *>(smem + C::WM * C::BN * 4);
    if (lane < 16) {
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int col = wn * C::WTN + j * 16 + lane;
            sv[wm * C::BN + col] = bestv[j];
            si[wm * C::BN + col] = besti[j];
        }
    }
    __syncthreads();
    for (int col = threadIdx.x; col < nq; col += C::NT) {
        float bv = sv[col];
        int bi = si[col];
#pragma unroll
        for (int w = 1; w < C::WM; ++w) {
            const float v = sv[w * C::BN + col];
            const int i = si[w * C::BN + col];
            if (lex_less(-v, i, -bv, bi)) {
                bv = v;
                bi = i;
            }
        }
        if (G == 1) {
            if (p.cid) p.cid[q0 + col] = bi;
            if (p.expert_ids) p.expert_ids[q0 + col] = p.slot ? p.slot[bi] : bi;
        } else if (bv > -__builtin_inff()) {
            // exact, order-independent merge across the group: smallest -score,
            // then lowest index; a score of -inf (excluded centroid, NaN) never enters
            atomicMin(&p.best[q0 + col], ((unsigned long long)float_order_key(-bv) << 32) | (unsigned)bi);
        }
    }
    // G > 1: route_unpack_kernel turns the packed winners into ids.  (Electing a
    // finishing workgroup here would need device-scope fences, and an acquire
    // fence drops the XCD's L2 contents -- the very thing the grouping protects.)
}

// Packed (score key, index) winners of the grouped streaming kernel -> ids.
__global__ __launch_bounds__(256) void route_unpack_kernel(const unsigned long long *best, int64_t N, int K,
                                                           const int *slot, int *cid, int *expert_ids)
{
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= N) return;
    const unsigned idx = (unsigned)(best[q] & 0xffffffffu);
    const int bi = (idx < (unsigned)K) ? (int)idx : 0;   // nothing won: centroid 0
    if (cid) cid[q] = bi;
    if (expert_ids) expert_ids[q] = slot ? slot[bi] : bi;
}

// Small batches: too few queries to fill the chip with 256-query workgroups, so
// the centroid range is split as well.  Workgroup (ct, qt) scores 64 centroids
// against 64 queries and merges its per-query minimum into best[] with a 64-bit
// atomic min on (score key << 32 | index): exact, order-independent, and the
// lowest index wins equal scores.  The workgroup that arrives last unpacks.
template <class C>
__global__ __launch_bounds__(C::NT) void route_small_kernel(RouteKParams p, int nqt)
{
    extern __shared__ __align__(16) char smem[];
    __shared__ int last_flag;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wn = wave % C::WN;
    const int qt = blockIdx.x % nqt, ct = blockIdx.x / nqt;
    const int q0 = qt * C::BN, c0 = ct * C::BM;
    const int nq = min(C::BN, (int)p.N - q0), nc = min(C::BM, p.K - c0);
    const uint32_t ld = (uint32_t)p.D * 2u;
    const int nkb = p.D / C::BK;
    const char *cb = p.cent + (int64_t)c0 * ld;
    const char *qb = p.emb + (int64_t)q0 * ld;
    const auto lc = C::template make_lanes<C::A_I>(nc);
    const auto lq = C::template make_lanes<C::B_I>(nq);

    typename C::Acc acc;
    C::zero(acc);
#pragma unroll
    for (int s = 0; s < C::NS - 1; ++s)
        if (s < nkb) C::issue(smem + s * C::STAGE_BYTES, cb, ld, lc, qb, ld, lq, (uint32_t)s * (C::BK * 2));
    int st = 0;
    for (int it = 0; it < nkb; ++it) {
        if (it + C::NS - 2 < nkb) wait_vm_then_barrier<(C::NS - 2) * C::LPB>();
        else wait_vm_then_barrier<0>();
        const int nb = it + C::NS - 1;
        const int ns = (st == 0) ? C::NS - 1 : st - 1;
        if (nb < nkb) C::issue(smem + ns * C::STAGE_BYTES, cb, ld, lc, qb, ld, lq, (uint32_t)nb * (C::BK * 2));
        C::compute_stage(smem + st * C::STAGE_BYTES, acc);
        st = (st + 1 == C::NS) ? 0 : st + 1;
    }

    float bestv[C::FN];
    int besti[C::FN];
#pragma unroll
    for (int j = 0; j < C::FN; ++j) {
        bestv[j] = __builtin_inff();
        besti[j] = 0;
    }
    fold_scores<C>(acc, p.cnorm + c0, c0, bestv, besti);
#pragma unroll
    for (int j = 0; j < C::FN; ++j) {
        const float ov = __shfl_xor(bestv[j], 32);
        const int oi = __shfl_xor(besti[j], 32);
        if (lex_less(ov, oi, bestv[j], besti[j])) {
            bestv[j] = ov;
            besti[j] = oi;
        }
        const int col = wn * C::WTN + j * 32 + lane;
        // a score that is not below +inf (excluded centroid, NaN) never wins
        if (lane < 32 && col < nq && bestv[j] < __builtin_inff())
            atomicMin(&p.best[q0 + col],
                      ((unsigned long long)float_order_key(bestv[j]) << 32) | (unsigned)besti[j]);
    }
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0)
        last_flag = (atomicAdd(p.arrivals, 1) == (int)gridDim.x - 1);
    __syncthreads();
    if (!last_flag) return;
    __threadfence();
    if (p.self_clean && p.counts) {   // (uniform) nobody zeroed the histogram ahead of this launch
        for (int k = threadIdx.x; k < p.K; k += C::NT) p.counts[k] = 0;
        __syncthreads();
    }
    if (p.self_clean && threadIdx.x == 0) *p.arrivals = 0;
    for (int q = threadIdx.x; q < (int)p.N; q += C::NT) {
        const unsigned long long key =
            __hip_atomic_load(&p.best[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (p.self_clean) p.best[q] = ~0ull;   // ready for the next call
        const unsigned idx = (unsigned)(key & 0xffffffffu);
        const int bi = (idx < (unsigned)p.K) ? (int)idx : 0;   // nothing won: centroid 0
        if (p.cid) p.cid[q] = bi;
        if (p.expert_ids) p.expert_ids[q] = p.slot ? p.slot[bi] : bi;
        if (p.counts) atomicAdd(&p.counts[bi], 1);
    }
    if constexpr (C::NT == PLAN_THREADS_SMALL) {
        if (p.with_plan) {
            // the ids this workgroup has just written are the plan's input
            __threadfence_block();
            __syncthreads();
            plan_body<PLAN_THREADS_SMALL>(p.plan, p.seq_offsets, p.expert_ids, p.rank_of_expert, p.err_word);
        }
    }
}

// ||c_k||^2 in fp32 (one wave per centroid), +inf for centroids left out of the
// search and for the padding up to a multiple of 256.  The same launch resets
// what the kernels after it accumulate into: the packed minima and arrival
// counter of the small-batch router, and the histogram.
__global__ __launch_bounds__(256) void centroid_norm_kernel(const char *cent, int K, int Kpad,
                                                            int D, int is_bf16, const int *slot,
                                                            int retained_only, float *cnorm,
                                                            float *cinit,
                                                            unsigned long long *best, int64_t nbest,
                                                            int *arrivals, int narrivals, int *counts)
{
    const int gid = blockIdx.x * 256 + threadIdx.x;
    const int gsz = gridDim.x * 256;
    for (int64_t i = gid; i < nbest; i += gsz) best[i] = ~0ull;
    if (counts)
        for (int i = gid; i < K; i += gsz) counts[i] = 0;
    for (int i = gid; i < narrivals; i += gsz) arrivals[i] = 0;

    const int lane = threadIdx.x & 63;
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (k >= Kpad) return;
    float acc = 0.f;
    if (k < K) {
        if (is_bf16) {
            const uint16_t *c = reinterpret_cast<const uint16_t *>(cent) + (int64_t)k * D;
            for (int j = lane; j < D; j += 64) {
                const float v = bf16_bits_to_f32(c[j]);
                acc = fmaf(v, v, acc);
            }
        } else {
            const float *c = reinterpret_cast<const float *>(cent) + (int64_t)k * D;
            for (int j = lane; j < D; j += 64) acc = fmaf(c[j], c[j], acc);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
        if (retained_only && slot[k] < 0) acc = __builtin_inff();
    } else {
        acc = __builtin_inff();
    }
    if (lane == 0) {
        cnorm[k] = acc;
        cinit[k] = -0.5f * acc;
    }
}

// fp32 embeddings: one wave per query, direct sum of squared differences.
// cnorm is only consulted for its +inf marks (centroids left out of the search).
__global__ __launch_bounds__(256) void route_f32_kernel(const float *emb, const float *cent,
                                                        const float *cnorm, int64_t N, int K, int D,
                                                        const int *slot, int *cid, int *expert_ids)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= N) return;
    const float *q = emb + i * D;
    float bv = __builtin_inff();
    int bi = 0;
    for (int k = 0; k < K; ++k) {
        const float *c = cent + (int64_t)k * D;
        float acc = 0.f;
        for (int j = lane; j < D; j += 64) {
            const float d = q[j] - c[j];
            acc = fmaf(d, d, acc);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
        if (cnorm[k] == __builtin_inff()) acc = __builtin_inff();
        if (acc < bv) {
            bv = acc;
            bi = k;
        }
    }
    if (lane == 0) {
        if (cid) cid[i] = bi;
        if (expert_ids) expert_ids[i] = slot ? slot[bi] : bi;
    }
}

// counts[k] = #{i : ids[i] == k}.  Workgroups tally a slice of ids in LDS and
// flush the non-zero bins with integer atomics (order-independent, exact).
constexpr int HIST_LDS_BINS = 16384;
__global__ __launch_bounds__(1024) void histogram_kernel(const int *ids, int64_t N, int K,
                                                         int *counts, int *err_word)
{
    __shared__ int bins[HIST_LDS_BINS];
    const bool use_lds = K <= HIST_LDS_BINS;
    if (use_lds) {
        for (int k = threadIdx.x; k < K; k += blockDim.x) bins[k] = 0;
        __syncthreads();
    }
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += stride) {
        const int id = ids[i];
        if (id < 0 || id >= K) {
            bad = true;
            continue;
        }
        if (use_lds) atomicAdd(&bins[id], 1);
        else atomicAdd(&counts[id], 1);
    }
    if (bad) atomicOr(err_word, ERR_BAD_ID);
    if (use_lds) {
        __syncthreads();
        for (int k = threadIdx.x; k < K; k += blockDim.x)
            if (bins[k]) atomicAdd(&counts[k], bins[k]);
    }
}

// The k nearest centroids of every query ("Future Works", creating new experts on the
// fly: a query on the boundary of several clusters may need several adapters).  A
// request-time call, not the bulk router: one wave per query, the squared distance
// written out as the sum of squared differences in fp32 (lanes split the dimension; the
// cross-lane sum ends in a uniform value, so every lane sees the same bits), centroids visited in index
// order and inserted behind their equals, so equal distances keep index order.
// Every lane carries the same list of ROUTE_TOPK_MAX entries in registers.
constexpr int ROUTE_TOPK_MAX = 8;
constexpr int ROUTE_TOPK_BATCH = 8;

template <bool BF16>
__global__ __launch_bounds__(256) void route_topk_kernel(const char *__restrict__ emb, const char *__restrict__ cent,
                                                         int64_t N, int K, int D, int k,
                                                         const int *__restrict__ slot, int retained_only,
                                                         int *__restrict__ cid, int *__restrict__ expert_ids,
                                                         float *__restrict__ d2)
{
    constexpr int VPC = BF16 ? 8 : 4;   // values per 16-byte chunk
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= N) return;
    const int64_t row_bytes = (int64_t)D * (16 / VPC);
    const char *q = emb + i * row_bytes;
    const int nch = D / VPC;
    float ld[ROUTE_TOPK_MAX];
    int li[ROUTE_TOPK_MAX];
#pragma unroll
    for (int m = 0; m < ROUTE_TOPK_MAX; ++m) {
        ld[m] = __builtin_inff();
        li[m] = -1;
    }
    // ROUTE_TOPK_BATCH centroids at a time: their loads are independent and in flight together
    for (int c0 = 0; c0 < K; c0 += ROUTE_TOPK_BATCH) {
        float acc[ROUTE_TOPK_BATCH];
#pragma unroll
        for (int u = 0; u < ROUTE_TOPK_BATCH; ++u) acc[u] = 0.f;
        for (int ch = lane; ch < nch; ch += 64) {
            const uint4 a = *reinterpret_cast<const uint4 *>(q + (int64_t)ch * 16);
            uint4 b[ROUTE_TOPK_BATCH];
#pragma unroll
            for (int u = 0; u < ROUTE_TOPK_BATCH; ++u)   // past the last centroid: the last one again, not inserted
                b[u] = *reinterpret_cast<const uint4 *>(cent + (int64_t)min(c0 + u, K - 1) * row_bytes + (int64_t)ch * 16);
            float x[8];
            if constexpr (BF16) {
                const uint32_t aw[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    x[2 * t] = bits_f32(aw[t] << 16);
                    x[2 * t + 1] = bits_f32(aw[t] & 0xFFFF0000u);
                }
            } else {
                x[0] = bits_f32(a.x); x[1] = bits_f32(a.y); x[2] = bits_f32(a.z); x[3] = bits_f32(a.w);
            }
#pragma unroll
            for (int u = 0; u < ROUTE_TOPK_BATCH; ++u) {
                float y[8];
                if constexpr (BF16) {
                    const uint32_t bw[4] = {b[u].x, b[u].y, b[u].z, b[u].w};
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        y[2 * t] = bits_f32(bw[t] << 16);
                        y[2 * t + 1] = bits_f32(bw[t] & 0xFFFF0000u);
                    }
                } else {
                    y[0] = bits_f32(b[u].x); y[1] = bits_f32(b[u].y); y[2] = bits_f32(b[u].z); y[3] = bits_f32(b[u].w);
                }
#pragma unroll
                for (int t = 0; t < VPC; ++t) {
                    const float df = x[t] - y[t];
                    acc[u] += df * df;
                }
            }
        }
        // The eight sums over the wave in 10 exchanges instead of 48: at distance 32 a lane hands
        // over the four partial sums its half does not keep, at 16 two, at 8 one; then three plain
        // butterfly steps.  Lane l ends with the sum of centroid 4 (l / 32) + 2 (l / 16 % 2) + l / 8 % 2,
        // and a uniform read of one lane of each group gives every lane all eight.
        static_assert(ROUTE_TOPK_BATCH == 8, "the exchange pattern below is written for eight sums");
        float v4[4], v2[2], v1;
        {
            const bool hi = lane & 32;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float keep = hi ? acc[4 + j] : acc[j], give = hi ? acc[j] : acc[4 + j];
                v4[j] = keep + __shfl_xor(give, 32);
            }
            const bool h16 = lane & 16;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float keep = h16 ? v4[2 + j] : v4[j], give = h16 ? v4[j] : v4[2 + j];
                v2[j] = keep + __shfl_xor(give, 16);
            }
            const bool h8 = lane & 8;
            const float keep = h8 ? v2[1] : v2[0], give = h8 ? v2[0] : v2[1];
            v1 = keep + __shfl_xor(give, 8);
#pragma unroll
            for (int off = 4; off > 0; off >>= 1) v1 += __shfl_xor(v1, off);
        }
#pragma unroll
        for (int u = 0; u < ROUTE_TOPK_BATCH; ++u) {
            acc[u] = bits_f32((uint32_t)__builtin_amdgcn_readlane(
                (int)__builtin_bit_cast(uint32_t, v1), ((u >> 2) & 1) * 32 + ((u >> 1) & 1) * 16 + (u & 1) * 8));
            const int c = c0 + u;
            // (the same for the whole wave) past the end, or a topic left out of the search
            if (c >= K || (retained_only && slot[c] < 0)) continue;
            const float d = acc[u];
            // (every lane holds the same list: the test is the same for the whole wave)
            if (!(d < ld[ROUTE_TOPK_MAX - 1])) continue;
            // behind its equals; a NaN compares false and never enters
#pragma unroll
            for (int m = ROUTE_TOPK_MAX - 1; m >= 0; --m) {
                const bool lt = d < ld[m];
                if (m + 1 < ROUTE_TOPK_MAX) {
                    ld[m + 1] = lt ? ld[m] : ld[m + 1];
                    li[m + 1] = lt ? li[m] : li[m + 1];
                }
                ld[m] = lt ? d : ld[m];
                li[m] = lt ? c : li[m];
            }
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int m = 0; m < ROUTE_TOPK_MAX; ++m)
            if (m < k) {
                const int c = li[m];
                if (cid) cid[i * k + m] = c;
                if (expert_ids) expert_ids[i * k + m] = c < 0 ? -1 : (slot ? slot[c] : c);
                if (d2) d2[i * k + m] = ld[m];
            }
    }
}

hipError_t launch_route_topk(const RouteArgs &a, int k, float *d2, hipStream_t stream)
{
    if (a.N <= 0) return hipSuccess;
    if (k < 1 || k > ROUTE_TOPK_MAX) return hipErrorInvalidValue;
    const int64_t grid = (a.N + 3) / 4;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.is_bf16)
        hipLaunchKernelGGL(route_topk_kernel<true>, dim3((unsigned)grid), dim3(256), 0, stream, (const char *)a.emb,
                           (const char *)a.cent, a.N, a.K, a.D, k, a.slot, a.retained_only, a.cid, a.expert_ids, d2);
    else
        hipLaunchKernelGGL(route_topk_kernel<false>, dim3((unsigned)grid), dim3(256), 0, stream, (const char *)a.emb,
                           (const char *)a.cent, a.N, a.K, a.D, k, a.slot, a.retained_only, a.cid, a.expert_ids, d2);
    return hipGetLastError();
}

// Plain fill: a memset node recorded into a captured graph is unreliable on
// this platform, a kernel is not.
__global__ __launch_bounds__(256) void fill_i32_kernel(int *dst, int n, int value)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = value;
}

template <class K>
static hipError_t allow_lds(K kern, int bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

hipError_t prepare_route_kernels()
{
    hipError_t e;
    if ((e = allow_lds(&route_kernel<CfgRoute>, CfgRoute::SMEM_BYTES)) != hipSuccess) return e;
    if ((e = allow_lds(&route_stream_kernel, CfgRouteDma::SMEM_BYTES + 2048)) != hipSuccess) return e;
    return allow_lds(&route_small_kernel<CfgRouteSmall>, CfgRouteSmall::SMEM_BYTES);
}

static bool use_small_route(const RouteArgs &a)
{
    return a.is_bf16 && a.D % 64 == 0 && a.N <= ROUTE_SMALL_MAX_N;
}

static bool use_stream_route(const RouteArgs &a) { return a.is_bf16 && a.D % 64 == 0 && !use_small_route(a); }

// Workgroups per query tile of the streaming kernel: prefers 4 (eight query
// tiles per XCD in flight), among the sizes that split the centroid tiles
// evenly or nearly so; 1 = no sharing (few centroid tiles).
int route_stream_group(int64_t N, int K, int D, int is_bf16)
{
    RouteArgs a{};
    a.N = N; a.K = K; a.D = D; a.is_bf16 = is_bf16;
    if (!use_stream_route(a)) return 1;
    const int nct = (K + CfgRouteDma::BM - 1) / CfgRouteDma::BM;
    const int pref[] = {4, 8, 2, 5, 3, 6, 7};
    int best_g = 1;
    double best_waste = 1.05;   // accept at most 5 % of idle tile slots over the plain scheme
    for (int g : pref) {
        if (g > nct) continue;
        const double waste = (double)((nct + g - 1) / g * g) / nct;
        if (waste < best_waste) {
            best_waste = waste;
            best_g = g;
            if (waste == 1.0) break;
        }
    }
    return best_g;
}

bool route_small_batch(int64_t N, int K, int D, int is_bf16)
{
    RouteArgs a{};
    a.N = N; a.K = K; a.D = D; a.is_bf16 = is_bf16;
    return use_small_route(a);
}

bool route_tallies_counts(const RouteArgs &a) { return a.N > 0 && a.counts != nullptr && use_small_route(a); }

hipError_t launch_centroid_norms(const RouteArgs &a, hipStream_t stream)
{
    const int Kpad = (a.K + 255) / 256 * 256;
    // a self-cleaning small-batch call needs the norms only
    const int64_t nbest = a.self_clean ? 0 : ((use_small_route(a) || a.group > 1) ? a.N : 0);
    const int narr = a.self_clean ? 0 : 1;
    hipLaunchKernelGGL(centroid_norm_kernel, dim3((Kpad + 3) / 4), dim3(256), 0, stream,
                       (const char *)a.cent, a.K, Kpad, a.D, a.is_bf16, a.slot, a.retained_only,
                       a.cnorm, a.cinit, a.best, nbest, a.arrivals, narr, a.self_clean ? nullptr : a.counts);
    return hipGetLastError();
}

hipError_t launch_route(const RouteArgs &a, hipStream_t stream)
{
    if (a.N <= 0) return hipSuccess;
    if (a.is_bf16) {
        RouteKParams p;
        p.emb = (const char *)a.emb; p.cent = (const char *)a.cent;
        p.cnorm = a.cnorm; p.cinit = a.cinit; p.slot = a.slot; p.cid = a.cid; p.expert_ids = a.expert_ids;
        p.best = a.best; p.arrivals = a.arrivals;
        p.counts = use_small_route(a) ? a.counts : nullptr;
        p.N = a.N; p.K = a.K; p.D = a.D;
        p.group = a.group > 1 ? a.group : 1;
        p.self_clean = use_small_route(a) ? a.self_clean : 0;
        static_assert(ROUTE_PLAN_FUSED_MAX_S <= 2 * PLAN_THREADS_SMALL && CfgRouteSmall::NT == PLAN_THREADS_SMALL,
                      "the grouping that rides in the small-batch launch is the four-wave one");
        if (a.plan && !(use_small_route(a) && a.self_clean && a.expert_ids && a.seq_offsets && a.err_word &&
                        a.N <= ROUTE_PLAN_FUSED_MAX_S && a.plan->S == (int)a.N))
            return hipErrorInvalidValue;
        p.with_plan = a.plan ? 1 : 0;
        if (p.with_plan) {
            p.plan = *a.plan;
            p.seq_offsets = a.seq_offsets; p.rank_of_expert = a.rank_of_expert; p.err_word = a.err_word;
        } else {
            p.plan = PlanView{};
            p.seq_offsets = p.rank_of_expert = nullptr; p.err_word = nullptr;
        }
        if (use_small_route(a)) {
            using C = CfgRouteSmall;
            const int nqt = (int)((a.N + C::BN - 1) / C::BN);
            const int64_t grid = (int64_t)nqt * ((a.K + C::BM - 1) / C::BM);
            if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
            hipLaunchKernelGGL(route_small_kernel<C>, dim3((unsigned)grid), dim3(C::NT),
                               C::SMEM_BYTES, stream, p, nqt);
            return hipGetLastError();
        }
        const int64_t grid = (a.N + CfgRoute::BN - 1) / CfgRoute::BN;
        if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
        if (a.D % 64 == 0) {
            // query tile t runs on XCD t % 8, its workgroups in consecutive slots there
            const int64_t sgrid = (grid + 7) / 8 * 8 * p.group;
            if (sgrid > 0x7fffffffLL) return hipErrorInvalidValue;
            hipLaunchKernelGGL(route_stream_kernel, dim3((unsigned)sgrid), dim3(CfgRouteDma::NT),
                               CfgRouteDma::SMEM_BYTES + 2048, stream, p);
            if (p.group > 1)
                hipLaunchKernelGGL(route_unpack_kernel, dim3((unsigned)((a.N + 255) / 256)), dim3(256), 0,
                                   stream, p.best, a.N, a.K, a.slot, a.cid, a.expert_ids);
        } else
            hipLaunchKernelGGL(route_kernel<CfgRoute>, dim3((unsigned)grid), dim3(CfgRoute::NT),
                               CfgRoute::SMEM_BYTES, stream, p);
    } else {
        const int64_t grid = (a.N + 3) / 4;
        if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(route_f32_kernel, dim3((unsigned)grid), dim3(256), 0, stream,
                           (const float *)a.emb, (const float *)a.cent, a.cnorm, a.N, a.K, a.D,
                           a.slot, a.cid, a.expert_ids);
    }
    return hipGetLastError();
}

hipError_t launch_histogram(const int *ids, int64_t N, int K, int *counts, int zero_first,
                            int *err_word, hipStream_t stream)
{
    if (zero_first) {
        hipLaunchKernelGGL(fill_i32_kernel, dim3((K + 255) / 256), dim3(256), 0, stream, counts, K, 0);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (N <= 0) return hipSuccess;
    int64_t blocks = (N + 1024 * 16 - 1) / (1024 * 16);
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(histogram_kernel, dim3((unsigned)blocks), dim3(1024), 0, stream, ids, N, K,
                       counts, err_word);
    return hipGetLastError();
}

}  // namespace moin
