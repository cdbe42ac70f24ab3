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
    int64_t n_virtual;    // streaming kernel: work items (query tiles rounded up to 8, times group)
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

// One (query tile, member of its group) per workgroup: 256 queries against every group-th tile of 256
// centroids, the blocks of all its centroid tiles forming one stream.  FOUR waves, one per SIMD, in the
// form of the prefill main kernel: 128 x 128 patches of 64 accumulators in AccVGPRs, MFMAs as assembly
// with the accumulator tied in and out, fragments of a k-step read under the MFMAs of the one before,
// and never more than one piece of other work (an LDS read, a request's address, the request) between
// two MFMAs.  argmin ||q - c||^2 is taken as argmax (q.c - ||c||^2 / 2): a tile's accumulators start
// from -||c||^2 / 2, and a finished tile is folded into the running best with a compare and two
// selects per score; the position inside the tile travels as a small code (tile, accumulator row
// block, element) that is the same for all lanes.
// An eight-wave form of this kernel (two waves per SIMD, 64 x 128 patches, accumulators in VGPRs) had
// the second wave to cover a wave's stalls, but both waves of a SIMD fold at the same time, and its
// registers were full: cycle stamps showed 3560 cycles per block of 128 MFMAs per SIMD and 12 000 at a
// tile's end, against 2700 per block in this form.
namespace r4 {
constexpr int BT = 256, BK = 64, ROWB = BK * 2, OP_BYTES = BT * ROWB, STAGE_BYTES = 2 * OP_BYTES;
constexpr int SMEM_STAGES = 2 * STAGE_BYTES;
constexpr int NW = 4, NT = NW * 64, FP = 8, FQ = 8, LOADS = 8;
constexpr int CBUF_BYTES = 2048;             // -||c||^2 / 2 of a centroid tile, two slots
constexpr int XCH_BYTES = 2 * BT * 8;        // winners of the two centroid halves, per query
constexpr int SMEM_BYTES = SMEM_STAGES + CBUF_BYTES + XCH_BYTES;
}  // namespace r4

__global__ __launch_bounds__(r4::NT) void route_stream4_kernel(RouteKParams p)
{
    using namespace r4;
    extern __shared__ __align__(16) char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = uniform(threadIdx.x >> 6);
    const int wp = wave >> 1, wq = wave & 1;
    // Work items: virtual workgroup v = (query tile, member of its group), query tile t on XCD t % 8 with
    // its G members in consecutive slots there.  The launch is persistent -- one workgroup per compute
    // unit, workgroup b takes v = b, b + gridDim, ... (gridDim is a multiple of 8 G, so the XCD and the
    // member stay the same) -- and the blocks of ALL its items form one stream: the first blocks of the
    // next item are requested under the last blocks of this one.  One launch per item left the matrix
    // core idle for a workgroup's dispatch and the 3.4 us from its start to its first block landed, once
    // per 90 us of work.
    const int G = p.group;
    const int member = (int)(blockIdx.x >> 3) % G;
    const int xcd = blockIdx.x & 7;
    // (gridDim = 8 G n: item `it` of this workgroup is query tile ((blockIdx >> 3) / G + it n) * 8 + xcd)
    const int64_t q0_first = ((int64_t)((blockIdx.x >> 3) / G) * 8 + xcd) * BT;
    const int64_t q0_step = (int64_t)(gridDim.x / (8 * G)) * 8 * BT;
    auto item_q0 = [&](int it) __attribute__((always_inline)) { return q0_first + (int64_t)it * q0_step; };
    int n_items = (int)((p.n_virtual - 1 - (int64_t)blockIdx.x) / gridDim.x) + 1;   // blockIdx.x < n_virtual
    while (n_items > 0 && item_q0(n_items - 1) >= p.N) --n_items;   // (only trailing items can lie past the batch)
    if (n_items == 0) return;
    const uint32_t ld = (uint32_t)p.D * 2u;
    const int nkb = p.D / BK;
    const int nct = (p.K + BT - 1) / BT;
    const int last_rows = p.K - (nct - 1) * BT;
    const int my_tiles = (nct - member + G - 1) / G;   // >= 1: G <= nct

    // requests of one block (centroid tile ct, contraction block kb): n = 0..7 centroid rows, 8..15 query
    // rows.  Per lane: the two chunk offsets and the eight source rows of its requests, clamped per
    // request to the operand's last valid row (a min and a multiply-add besides the request itself); the
    // block's position along k is in the uniform base pointers.
    const uint32_t c16a = (((uint32_t)lane & 7) ^ ((uint32_t)lane >> 4)) * 16, c16b = c16a ^ 64u;   // even j, odd j
    uint32_t rowu[LOADS];
#pragma unroll
    for (int n = 0; n < LOADS; ++n) rowu[n] = (uint32_t)(wave * (LOADS * 8)) + ((uint32_t)lane >> 3) + 8u * n;
    struct Fetch {
        const char *pp, *pq;
        uint32_t p_last, q_last;
    };
    // The fetch cursor: what the next block to request needs (operand pointers at its first k, the operands'
    // last valid rows), kept up to date step by step -- 128 bytes along both rows from block to block, new
    // pointers only where a tile or an item begins -- so that taking a block under the MFMAs costs a
    // handful of scalar instructions.  Past the stream's end it stays on the last block, which is then
    // requested again into the stage that is free anyway.
    int pit = 0, pct = member, pkb = 0;
    int pleft = n_items * my_tiles * nkb;   // blocks not yet taken
    const char *pqb = nullptr;              // the item's query rows at k = 0
    Fetch pf;
    auto cursor_tile = [&]() __attribute__((always_inline)) {
        pf.pp = p.cent + (int64_t)pct * BT * ld;
        pf.pq = pqb;
        pf.p_last = (uint32_t)((pct == nct - 1 ? last_rows : BT) - 1);
    };
    auto cursor_item = [&]() __attribute__((always_inline)) {
        const int64_t q0_ = item_q0(pit);
        pqb = p.emb + q0_ * (int64_t)ld;
        pf.q_last = (uint32_t)((int)min((int64_t)BT, p.N - q0_) - 1);
    };
    auto cursor_fetch = [&]() __attribute__((always_inline)) {
        const Fetch f = pf;
        if (pleft > 1) {
            --pleft;
            if (++pkb < nkb) {
                pf.pp += BK * 2;
                pf.pq += BK * 2;
            } else {
                pkb = 0;
                pct += G;
                if (pct >= nct) {
                    pct = member;
                    ++pit;
                    cursor_item();
                }
                cursor_tile();
            }
        }
        return f;
    };
    cursor_item();
    cursor_tile();
    auto issue_one = [&](const Fetch &f, char *stage, int n) __attribute__((always_inline)) {
        const int j = n & 7;
        const bool q = n >= LOADS;
        const uint32_t off = __umul24(min(rowu[j], q ? f.q_last : f.p_last), ld) + ((j & 1) ? c16b : c16a);
        __builtin_amdgcn_global_load_lds(MOIN_GPTR((q ? f.pq : f.pp) + off),
                                         MOIN_LPTR(stage + (q ? OP_BYTES : 0) + (wave * LOADS + j) * 1024), 16, 0, 0);
    };
    char *cbuf = smem + SMEM_STAGES;
    auto fetch_init = [&](int ct_, int slot_) __attribute__((always_inline)) {
        if (wave == 0)
            __builtin_amdgcn_global_load_lds(MOIN_GPTR(reinterpret_cast<const char *>(p.cinit + ct_ * BT) + lane * 16),
                                             MOIN_LPTR(cbuf + slot_ * 1024), 16, 0, 0);
    };
    // MFMA operand of a lane: row lane%16 of a 16-row block, logical 16-byte chunk 4 ks + lane/16 of the
    // row; k-step 1 is k-step 0's address ^ 64.  Fragment n = 0..7: centroid blocks, 8..15: query blocks.
    const int lo0 = ((lane & 15) * ROWB) | ((((lane >> 4) ^ ((lane & 15) >> 1)) & 7) * 16);
    const int lo1 = lo0 ^ 64;
    const int baseP = wp * (FP * 16) * ROWB, baseQ = OP_BYTES + wq * (FQ * 16) * ROWB;
    bf16x8_t fr[2][FP + FQ];
    auto read_one = [&](const char *stage, int lo_, int set, int n) __attribute__((always_inline)) {
        const int base_ = n < FP ? baseP + n * 16 * ROWB : baseQ + (n - FP) * 16 * ROWB;
        fr[set][n] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(stage + base_ + lo_));
    };
    // the order in which a k-step's fragments are read: the first MFMAs (centroid block 0 against query
    // blocks 0..7) need centroid block 0 and all query blocks, centroid block i only from MFMA 8 i
    auto frag_at = [](int k_) { return k_ == 0 ? 0 : (k_ <= FQ ? FP + k_ - 1 : k_ - FQ); };
    // acc[i][j]: centroid rows wp*128 + 16 i + 4 (lane / 16) + 0..3 of the tile, query wq*128 + 16 j + lane % 16
    f32x4_t acc[FP][FQ];
    auto mfma = [&](int set, int i, int j) __attribute__((always_inline)) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fr[set][i]), "v"(fr[set][FP + j]));
    };
    // A tile's first k-step takes -||c||^2 / 2 of the accumulator's four centroid rows as its addend.  The
    // eight accumulators of a row block share those four values: they are loaded into the block's first
    // accumulator only (one LDS read per row block instead of 256 register writes per tile, 5.6 cycles each
    // at one wave per SIMD), the other seven read it as their addend, and it takes its own MFMA last.
    auto mfma_first = [&](int i, int j) __attribute__((always_inline)) {
        if (j == 0)
            asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][0]) : "v"(fr[0][i]), "v"(fr[0][FP]));
        else
            asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %3"
                         : "=&a"(acc[i][j])
                         : "v"(fr[0][i]), "v"(fr[0][FP + j]), "a"(acc[i][0]));
    };

    float bestv[FQ];
    int bestc[FQ];   // (tile << 5) | (accumulator row block i << 2) | element

    // cm: where the lane's start values of the tile lie in LDS (first blocks only)
    auto body = [&](auto first_tag, int s, bool last_of_tile, int ct_next, int slot_next, const char *cm) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first_tag)::value;   // the tile's first block
        char *st_cur = smem + (s & 1) * STAGE_BYTES;
        const char *st_nxt = smem + ((s + 1) & 1) * STAGE_BYTES;
        Fetch f;
        // A first block loads the start values of row block i straight from LDS into the AccVGPRs of
        // accumulator (i, 0) -- one instruction, one register quad that the compiler has no reason to move
        // (four v_accvgpr_write results it assembled into a quad with copies, placed right in front of an
        // MFMA it cannot see) -- one row block ahead, and waits for it by count: behind that load come the
        // row block's fragment reads (four in each of the first four) and the next row block's load.
        const uint32_t cm_lds = (uint32_t)(size_t)MOIN_LPTR(cm);
        if constexpr (FIRST) asm volatile("ds_read_b128 %0, %1" : "=a"(acc[0][0]) : "v"(cm_lds) : "memory");
#pragma unroll
        for (int n = 0; n < FP * FQ; ++n) {
            if constexpr (FIRST) {
                if (n % FQ == 0) {
                    const int i = n / FQ;
                    if (i + 1 < FP)
                        asm volatile("ds_read_b128 %0, %1" : "=a"(acc[i + 1][0]) : "v"(cm_lds + (uint32_t)((i + 1) * 64)) : "memory");
                    constexpr int RPR = FQ / 2;   // fragment reads per row block of MFMAs, while there are any
                    const int behind = ((i >= 1 && (i - 1) * RPR < FP + FQ) ? RPR : 0) + (i + 1 < FP ? 1 : 0);
                    if (behind == 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    else if (behind == 1) asm volatile("s_waitcnt lgkmcnt(1)" ::: "memory");
                    else asm volatile("s_waitcnt lgkmcnt(5)" ::: "memory");
                    static_assert(RPR + 1 == 5, "the counted wait above");
                    __builtin_amdgcn_sched_barrier(0);
                }
                mfma_first(n / FQ, (n + 1) % FQ);   // 1..7, then 0
            } else {
                mfma(0, n / FQ, n % FQ);
            }
            if (n % 2 == 1 && n / 2 < FP + FQ) {
                read_one(st_cur, lo1, 1, frag_at(n / 2));
                __builtin_amdgcn_sched_barrier(0);
            }
            if (n == 36) {
                f = cursor_fetch();   // what the second half fetches
                __builtin_amdgcn_sched_barrier(0);
            }
            if (n == 44) {
                // the tile's last block fetches the next tile's start values; they land before this block's barrier
                if (last_of_tile && ct_next < nct) fetch_init(ct_next, slot_next);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
        for (int n = 0; n < FP * FQ; ++n) {
            mfma(1, n / FQ, n % FQ);
            if (n % 2 == 0 && n / 2 < FP + FQ) {   // all reads in the first half of the k-step: landed when the next block starts
                read_one(st_nxt, lo0, 0, frag_at(n / 2));
                __builtin_amdgcn_sched_barrier(0);
            }
            if (n % 4 == 1) {
                issue_one(f, st_cur, n / 4);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    fetch_init(member, 0);
    {
        const Fetch f0 = cursor_fetch();
#pragma unroll
        for (int n = 0; n < 2 * LOADS; ++n) issue_one(f0, smem, n);
        // (a stream of one block fetches it twice: the second copy is never read)
        const Fetch f1 = cursor_fetch();
#pragma unroll
        for (int n = 0; n < 2 * LOADS; ++n) issue_one(f1, smem + STAGE_BYTES, n);
    }
    wait_vm_then_barrier<2 * LOADS>();

    // the first block's leading fragments; every later block's are read under the block before it
#pragma unroll
    for (int n = 0; n < FP + FQ; ++n) read_one(smem, lo0, 0, n);
    const int g = lane >> 4;
    float *sv = reinterpret_cast<float *>(smem + SMEM_STAGES + CBUF_BYTES);
    int *si = reinterpret_cast<int *>(smem + SMEM_STAGES + CBUF_BYTES + 2 * BT * 4);
    int s = 0;    // blocks done so far (stage parity)
    int tt = 0;   // tiles done so far (parity of the start values' slot)
    for (int it = 0; it < n_items; ++it) {
    const int64_t q0 = item_q0(it);
    const int nq = (int)min((int64_t)BT, p.N - q0);
#pragma unroll
    for (int j = 0; j < FQ; ++j) {
        bestv[j] = -__builtin_inff();
        bestc[j] = 0;
    }
    int ct = member;
    for (int t = 0; t < my_tiles; ++t, ct += G, ++tt) {
        // the tile after this one: the item's next, or the next item's first, or none (nct)
        const int ct_next = t + 1 < my_tiles ? ct + G : (it + 1 < n_items ? member : nct);
        // start values: -||c||^2 / 2 of the lane's 32 centroid rows
        const char *cm = cbuf + (tt & 1) * 1024 + (wp * (FP * 16) + 4 * (lane >> 4)) * 4;
        body(std::true_type{}, s, nkb == 1, ct_next, (tt + 1) & 1, cm);
        ++s;
        for (int kb = 1; kb < nkb; ++kb, ++s) body(std::false_type{}, s, kb == nkb - 1, ct_next, (tt + 1) & 1, nullptr);
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // the last MFMAs' results before the fold reads them
        // A lane's scores come in ascending centroid order, so a strict '>' keeps the lowest index among
        // equals.  Every score is read out of its AccVGPR by an instruction of its own, in place (left to
        // the compiler, all 256 are copied out at once and push everything else out of the registers).
        // The compares of a lane's eight queries write eight scalar register pairs, the sixteen selects
        // follow: written as `sc > best ? ...` the compiler puts every compare's result in VCC and needs
        // two wait states before each select -- 23 cycles per score against 16 in a loop of nothing else
        // (one wave on the SIMD issues a vector instruction every 5.6 cycles).  A select reads its mask
        // seven or more instructions after the compare that wrote it, which is the distance the hardware
        // wants between a vector write of a scalar register and a vector read of it.
        const int code0 = ct << 5;
#pragma unroll
        for (int i = 0; i < FP; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float sc[FQ];
                unsigned long long gt[FQ];
                const int code = code0 + (i * 4 + e);
#pragma unroll
                for (int j = 0; j < FQ; ++j) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(sc[j]) : "a"(acc[i][j][e]));
#pragma unroll
                for (int j = 0; j < FQ; ++j) asm volatile("v_cmp_gt_f32_e64 %0, %1, %2" : "=s"(gt[j]) : "v"(sc[j]), "v"(bestv[j]));
#pragma unroll
                for (int j = 0; j < FQ; ++j) {
                    asm volatile("v_cndmask_b32_e64 %0, %0, %1, %2" : "+v"(bestv[j]) : "v"(sc[j]), "s"(gt[j]));
                    asm volatile("v_cndmask_b32_e64 %0, %0, %1, %2" : "+v"(bestc[j]) : "v"(code), "s"(gt[j]));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
    }
    // position code -> centroid index; merge the four lane groups (rows 4 * (lane / 16) interleave), then
    // the two waves that hold the other half of the tile's centroids: higher score, else lower index.
    // (The exchange area is written again only an item later, many block barriers after these reads.)
#pragma unroll
    for (int j = 0; j < FQ; ++j) {
        const int c = bestc[j];
        int bi = (c >> 5) * BT + wp * (FP * 16) + 16 * ((c >> 2) & 7) + 4 * g + (c & 3);
        float bv = bestv[j];
#pragma unroll
        for (int sh = 16; sh <= 32; sh <<= 1) {
            const float ov = __shfl_xor(bv, sh);
            const int oi = __shfl_xor(bi, sh);
            if (lex_less(-ov, oi, -bv, bi)) {
                bv = ov;
                bi = oi;
            }
        }
        if (lane < 16) {
            const int col = wq * (FQ * 16) + j * 16 + lane;
            sv[wp * BT + col] = bv;
            si[wp * BT + col] = bi;
        }
    }
    __syncthreads();
    for (int col = threadIdx.x; col < nq; col += NT) {
        float bv = sv[col];
        int bi = si[col];
        const float v = sv[BT + col];
        const int i = si[BT + col];
        if (lex_less(-v, i, -bv, bi)) {
            bv = v;
            bi = i;
        }
        if (G == 1) {
            if (p.cid) p.cid[q0 + col] = bi;
            if (p.expert_ids) p.expert_ids[q0 + col] = p.slot ? p.slot[bi] : bi;
        } else if (bv > -__builtin_inff()) {
            atomicMin(&p.best[q0 + col], ((unsigned long long)float_order_key(-bv) << 32) | (unsigned)bi);
        }
    }
    }   // items
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the requests repeated past the stream's end
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
    if ((e = allow_lds(&route_stream4_kernel, r4::SMEM_BYTES)) != hipSuccess) return e;
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
    const int nct = (K + r4::BT - 1) / r4::BT;
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
            // persistent: one workgroup per compute unit, a multiple of 8 * group so that a workgroup's
            // items all lie on its XCD and belong to its member of the group
            const int64_t unit = 8 * (int64_t)p.group;
            int64_t pgrid = (int64_t)compute_units() / unit * unit;
            if (pgrid < unit) pgrid = unit;
            if (pgrid > sgrid) pgrid = sgrid;
#ifdef MOIN_ROUTE_NONPERSISTENT
            pgrid = sgrid;
#endif
            p.n_virtual = sgrid;
            hipLaunchKernelGGL(route_stream4_kernel, dim3((unsigned)pgrid), dim3(r4::NT), r4::SMEM_BYTES, stream, p);
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
