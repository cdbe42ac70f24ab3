// Grouping of a batch by expert, as a device function (see plan.hip for what it computes).
#pragma once
#include "kernels.h"

namespace moin {

constexpr int PLAN_THREADS_MAX = 1024;   // large batches
constexpr int PLAN_THREADS_SMALL = 256;  // up to 512 sequences: four waves meet at a barrier much faster than sixteen
constexpr int PLAN_LDS_S = 2048;

// In-place exclusive prefix sum of data[0..n) by one workgroup; returns the total.
template <int PLAN_THREADS>
__device__ int block_exclusive_scan(int *data, int n, int *lds /* PLAN_THREADS + 1 ints */)
{
    const int tid = threadIdx.x;
    const int per = (n + PLAN_THREADS - 1) / PLAN_THREADS;
    const int lo = min(tid * per, n), hi = min(lo + per, n);
    int sum = 0;
    for (int i = lo; i < hi; ++i) sum += data[i];
    lds[tid] = sum;
    __syncthreads();
    // Hillis-Steele inclusive scan over the per-thread sums
    for (int off = 1; off < PLAN_THREADS; off <<= 1) {
        const int v = (tid >= off) ? lds[tid - off] : 0;
        __syncthreads();
        lds[tid] += v;
        __syncthreads();
    }
    const int total = lds[PLAN_THREADS - 1];
    int run = lds[tid] - sum;
    __syncthreads();
    for (int i = lo; i < hi; ++i) {
        const int v = data[i];
        data[i] = run;
        run += v;
    }
    __syncthreads();
    return total;
}

// The whole grouping, by ONE workgroup of PLAN_THREADS threads (all of them must call it).  A device
// function so that the kernel that routes a request-sized batch can go on to group it in the same launch.
template <int PLAN_THREADS>
__device__ __forceinline__ void plan_body(const PlanView &pv, const int *seq_offsets, const int *expert_ids,
                                          const int *rank_of_expert, int *err_word)
{
    // Rank of adapter slot e ("Future Works": adaptive rank per topic).  Multiples of 8,
    // like the stacks' own rank; anything else is rounded down and raises the sticky fault.
    auto rank_of = [&](int e) -> int {
        if (e < 0) return 0;
        if (!rank_of_expert) return RANK_FULL;
        int rk = rank_of_expert[e];
        if (rk < 0 || (rk & 7)) {
            atomicOr(err_word, ERR_BAD_RANK);
            rk = rk < 0 ? RANK_FULL : (rk & ~7);
        }
        return rk;
    };
    __shared__ int lds[PLAN_THREADS + 1];
    // batches of up to PLAN_LDS_S sequences sort and scan entirely in LDS (a
    // barrier-separated pass then costs tens of nanoseconds, not a round trip
    // to L2); larger ones use the plan's global scratch
    __shared__ unsigned long long lds_keys[PLAN_LDS_S];
    __shared__ int lds_tmp[4 * (PLAN_LDS_S + 1)];
    __shared__ int bad_offsets;
    const int tid = threadIdx.x;
    const int S = pv.S;
    const int T = (int)pv.T;
    int npow2 = 1;
    while (npow2 < S) npow2 <<= 1;
    const bool small = npow2 <= PLAN_LDS_S;
    unsigned long long *keys = small ? lds_keys : pv.keys;
    int *tmp = small ? lds_tmp : pv.tmp;

    int *lens = tmp;                  // [S]   length of each sequence (by sequence)
    int *a1 = tmp + (S + 1);          // [S+1] per sorted position: tile count -> tile base
    int *a2 = tmp + 2 * (S + 1);      // [S+1] per sorted position: length -> token base
    int *a3 = tmp + 3 * (S + 1);      // [S+1] per sorted position: group head flag -> group id

    // 1. validate, build sort keys (expert + 1 in the high word: -1 sorts first)
    int err = 0;
    if (tid == 0) bad_offsets = 0;
    __syncthreads();
    if (tid == 0 && (seq_offsets[0] != 0 || seq_offsets[S] != T)) err |= ERR_BAD_OFFSETS;
    for (int s = tid; s < npow2; s += PLAN_THREADS) {
        unsigned long long key = ~0ull;
        if (s < S) {
            int lo = seq_offsets[s], hi = seq_offsets[s + 1];
            int e = expert_ids[s];
            if (lo < 0 || hi > T || hi < lo) {
                err |= ERR_BAD_OFFSETS;
                lo = 0;
                hi = 0;
            }
            if (e < -1 || e >= pv.E) {
                err |= ERR_BAD_EXPERT;
                e = -1;
            }
            lens[s] = hi - lo;
            key = ((unsigned long long)(unsigned)(e + 1) << 32) | (unsigned)s;
        }
        keys[s] = key;
    }
    if (err) atomicOr(err_word, err);
    if (err & ERR_BAD_OFFSETS) bad_offsets = 1;
    for (int j = tid; j < pv.max_plain; j += PLAN_THREADS) {
        const int rows = min(TILE_M, T - j * TILE_M);
        pv.plain_row0[j] = j * TILE_M;
        pv.plain_rows[j] = max(rows, 0);
        pv.plain_expert[j] = -1;
        pv.plain_rank[j] = 0;
    }
    if (tid == 0 && pv.max_plain > 0) *pv.plain_n = min(pv.max_plain, (T + TILE_M - 1) / TILE_M);
    __syncthreads();
    if (bad_offsets) {
        // the sequences do not cover every token exactly once: one base-only
        // sequence over the whole batch instead
        const int nt = (T + TILE_M - 1) / TILE_M;   // <= max_tiles
        for (int j = tid; j < nt; j += PLAN_THREADS) {
            pv.tile_row0[j] = j * TILE_M;
            pv.tile_rows[j] = min(TILE_M, T - j * TILE_M);
            pv.tile_expert[j] = -1;
            pv.tile_rank[j] = 0;
        }
        if (tid == 0) *pv.n_tiles = nt;
        if (pv.decode) {
            for (int t = tid; t < T; t += PLAN_THREADS) pv.tok_sorted[t] = t;
            const int nc = min((T + GROUP_CHUNK - 1) / GROUP_CHUNK, pv.max_groups);
            if (tid == 0) *pv.n_groups = nc;
            for (int gi = tid; gi < pv.max_groups; gi += PLAN_THREADS)
                pv.grp_meta[gi] = gi < nc ? make_int4(-1, gi * GROUP_CHUNK, min(T, (gi + 1) * GROUP_CHUNK), 0)
                                          : make_int4(-1, 0, 0, 0);
        }
        return;
    }

    // 2. bitonic sort of the keys by the one workgroup.  Element i meets element i ^ j,
    // ascending where (i & k) == 0.  Up to PLAN_LDS_S keys everything happens in LDS.
    // Beyond, only the steps whose partners lie PLAN_LDS_S or more apart walk global
    // memory; all steps with j < PLAN_LDS_S stay inside an aligned chunk of PLAN_LDS_S
    // keys, which is brought into LDS once for a whole run of them.
    auto steps_in = [&](unsigned long long *buf, int n, int base, int k, int j_first) {
        for (int j = j_first; j > 0; j >>= 1) {
            for (int i = tid; i < n; i += PLAN_THREADS) {
                const int l = i ^ j;
                if (l > i) {
                    const unsigned long long a = buf[i], b = buf[l];
                    const bool up = ((base + i) & k) == 0;
                    if ((a > b) == up) {
                        buf[i] = b;
                        buf[l] = a;
                    }
                }
            }
            __syncthreads();
        }
    };
    if (small) {
        for (int k = 2; k <= npow2; k <<= 1) steps_in(keys, npow2, 0, k, k >> 1);
    } else {
        auto chunk_run = [&](int c, int k_first, int k_last, int j_first_of_last) {
            // chunk c through LDS: whole stages k_first..k_last / 2 and, of stage k_last, the steps from j_first_of_last down
            unsigned long long *g = keys + (size_t)c * PLAN_LDS_S;
            for (int i = tid; i < PLAN_LDS_S; i += PLAN_THREADS) lds_keys[i] = g[i];
            __syncthreads();
            for (int k = k_first; k < k_last; k <<= 1) steps_in(lds_keys, PLAN_LDS_S, c * PLAN_LDS_S, k, k >> 1);
            steps_in(lds_keys, PLAN_LDS_S, c * PLAN_LDS_S, k_last, j_first_of_last);
            for (int i = tid; i < PLAN_LDS_S; i += PLAN_THREADS) g[i] = lds_keys[i];
            __syncthreads();
        };
        const int n_chunks = npow2 / PLAN_LDS_S;
        for (int c = 0; c < n_chunks; ++c) chunk_run(c, 2, PLAN_LDS_S, PLAN_LDS_S >> 1);
        for (int k = 2 * PLAN_LDS_S; k <= npow2; k <<= 1) {
            for (int j = k >> 1; j >= PLAN_LDS_S; j >>= 1) {
                for (int i = tid; i < npow2; i += PLAN_THREADS) {
                    const int l = i ^ j;
                    if (l > i) {
                        const unsigned long long a = keys[i], b = keys[l];
                        const bool up = (i & k) == 0;
                        if ((a > b) == up) {
                            keys[i] = b;
                            keys[l] = a;
                        }
                    }
                }
                __syncthreads();
            }
            for (int c = 0; c < n_chunks; ++c) chunk_run(c, k, k, PLAN_LDS_S >> 1);
        }
    }

    // 3. per sorted position: tile count, token count, group-head flag
    for (int p = tid; p < S; p += PLAN_THREADS) {
        const unsigned long long key = keys[p];
        const int s = (int)(key & 0xffffffffu);
        const int len = lens[s];
        a1[p] = (len + TILE_M - 1) / TILE_M;
        a2[p] = len;
        const bool head = (p == 0) || ((keys[p - 1] >> 32) != (key >> 32));
        a3[p] = head ? 1 : 0;
    }
    __syncthreads();
    const int n_tiles = block_exclusive_scan<PLAN_THREADS>(a1, S, lds);
    if (tid == 0) *pv.n_tiles = min(n_tiles, pv.max_tiles);
    int n_groups = 0, n_tok = 0;
    if (pv.decode) {
        n_tok = block_exclusive_scan<PLAN_THREADS>(a2, S, lds);
        n_groups = block_exclusive_scan<PLAN_THREADS>(a3, S, lds);   // a3[p] = groups before p
        if (tid == 0) pv.grp_start[n_groups] = min(n_tok, T);
    }

    // 4. emit
    for (int p = tid; p < S; p += PLAN_THREADS) {
        const unsigned long long key = keys[p];
        const int s = (int)(key & 0xffffffffu);
        const int e = (int)(key >> 32) - 1;
        const int lo = seq_offsets[s];
        const int len = lens[s];
        const int tb = a1[p];
        const int rk = rank_of(e);
        for (int j = 0, left = len; left > 0 && tb + j < pv.max_tiles; ++j, left -= TILE_M) {
            pv.tile_row0[tb + j] = lo + j * TILE_M;
            pv.tile_rows[tb + j] = min(left, TILE_M);
            pv.tile_expert[tb + j] = e;
            pv.tile_rank[tb + j] = rk;
        }
        if (pv.decode) {
            const int base = min(a2[p], T);
            const bool head = (p == 0) || ((keys[p - 1] >> 32) != (key >> 32));
            if (head) {
                const int gi = a3[p];   // exclusive count of heads before p
                pv.grp_tmp[gi] = make_int2(e, rk);
                pv.grp_start[gi] = base;
            }
        }
    }
    if (pv.decode) {
        // tokens in sorted order, one per thread and step whatever the sequences' lengths:
        // position t belongs to the last sorted sequence that starts at or before it
        for (int t = tid; t < min(n_tok, T); t += PLAN_THREADS) {
            int first = 0, last = S - 1;
            while (first < last) {
                const int mid = (first + last + 1) >> 1;
                if (a2[mid] <= t) first = mid;
                else last = mid - 1;
            }
            const int s = (int)(keys[first] & 0xffffffffu);
            pv.tok_sorted[t] = seq_offsets[s] + (t - a2[first]);
        }
    }
    if (pv.decode) {
        // A group ends where the next one starts.  It is cut into records of at most
        // GROUP_CHUNK tokens: the decode kernels hand a record to one column of
        // workgroups, and a hot expert's tokens must not all queue behind one column.
        __syncthreads();   // grp_start / grp_tmp are complete, a1 is free
        for (int gi = tid; gi < n_groups; gi += PLAN_THREADS)
            a1[gi] = (pv.grp_start[gi + 1] - pv.grp_start[gi] + GROUP_CHUNK - 1) / GROUP_CHUNK;
        __syncthreads();
        const int n_rec = min(block_exclusive_scan<PLAN_THREADS>(a1, n_groups, lds), pv.max_groups);
        for (int gi = tid; gi < n_groups; gi += PLAN_THREADS) {
            const int2 er = pv.grp_tmp[gi];
            const int ge = pv.grp_start[gi + 1];
            int rec = a1[gi];
            for (int t = pv.grp_start[gi]; t < ge && rec < pv.max_groups; t += GROUP_CHUNK, ++rec)
                pv.grp_meta[rec] = make_int4(er.x, t, min(t + GROUP_CHUNK, ge), er.y);
        }
        if (tid == 0) *pv.n_groups = n_rec;
        // unused records read as empty groups, so the decode kernels need not
        // fetch the group count before their own record
        for (int gi = n_rec + tid; gi < pv.max_groups; gi += PLAN_THREADS) pv.grp_meta[gi] = make_int4(-1, 0, 0, 0);
    }
}


}  // namespace moin
