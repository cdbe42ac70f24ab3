// Decode path of the routed LoRA linear layer: a handful of tokens per
// sequence, hundreds of distinct adapters per batch, so the time goes into
// streaming W_a and W_b of every distinct adapter from HBM once (Section 1:
// many small adapters served together; Section 3.2: y = W x + W_b (W_a x)).
//
// Tokens arrive grouped by expert (plan).  One workgroup handles one
// (expert, slab of adapter rows): it streams the slab with 16-byte lane loads
// straight into MFMA operands -- no LDS staging, each adapter byte is used by
// exactly one wave -- and multiplies it against the (at most a few) tokens of
// that expert with v_mfma_f32_16x16x32_bf16, whose 16 columns are 16 tokens.
// Idle MFMA columns cost nothing here: the kernels are HBM-bound, and what
// decides their speed is how many independent loads are in flight, so every
// wave issues all loads of a batch before the first MFMA that consumes them
// and the grid is shaped for several resident workgroups per compute unit.
//
//   base   : ybase[s] = x[:, range s] W[:, range s]^T   (fp32, linear.hip)
//   shrink : ug[pos, :] = scale * A_e x_tok             (bf16 high part + remainder)
//   expand : y[tok, :]  = sum_s ybase[s][tok, :] + B_e ug[pos]
#include <algorithm>

#include "gemm_core.h"
#include "kernels.h"
#include "linear_tile.h"

namespace moin {

// 16-byte operand fragment at row + k*2 bytes.  Past the row end (k >= klen)
// the load is redirected to k = 0 and the data zeroed, so no branch is needed.
// Lanes whose row is only padding pass any in-bounds row: an MFMA output
// depends on its own row and column only, and padded outputs are not stored.
__device__ __forceinline__ bf16x8_t ldg_frag(const char *row, int k, int klen)
{
    const bool ok = k < klen;
    const uint32_t m = ok ? 0xFFFFFFFFu : 0u;
    uint4 v = *reinterpret_cast<const uint4 *>(row + (ok ? k : 0) * 2);
    v.x &= m; v.y &= m; v.z &= m; v.w &= m;
    return __builtin_bit_cast(bf16x8_t, v);
}

// Group records and the first token indices of a group come through the scalar
// cache: a scalar load does not queue behind the compute unit's vector-memory
// traffic, so a workgroup knows its adapter and its tokens a few hundred
// nanoseconds after it starts and can then issue ALL of its vector loads at once --
// one trip to memory per workgroup instead of a chain of three.  (Under load
// every dependent vector load costs a full queueing delay of several
// microseconds, which is what kept these kernels at half the streaming rate.)
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x16_t __attribute__((ext_vector_type(16)));
__device__ __forceinline__ i32x4_t sload_x4(const void *p)   // p: uniform, 4-byte aligned
{
    i32x4_t v;
    asm volatile("s_load_dwordx4 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(p) : "memory");
    return v;
}
__device__ __forceinline__ i32x16_t sload_x16(const void *p)
{
    i32x16_t v;
    asm volatile("s_load_dwordx16 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(p) : "memory");
    return v;
}
// Element (lane % 16) of sixteen wave-uniform values.
__device__ __forceinline__ int pick16(const i32x16_t &t, int lane)
{
    const int i = lane & 15;
    int v = t[0];
#pragma unroll
    for (int k = 1; k < 16; ++k) v = (i == k) ? t[k] : v;
    return v;
}

// ldg_frag in two halves, so that a kernel can first issue every load it will need
// and only then touch the data (a scheduling barrier between the two keeps the
// compiler from waiting on one load before it has issued the next).
__device__ __forceinline__ uint4 ldg_raw(const char *row, int k, int klen)
{
    return *reinterpret_cast<const uint4 *>(row + (k < klen ? k : 0) * 2);
}
__device__ __forceinline__ bf16x8_t frag_of(uint4 v, int k, int klen)
{
    const uint32_t m = k < klen ? 0xFFFFFFFFu : 0u;
    v.x &= m; v.y &= m; v.z &= m; v.w &= m;
    return __builtin_bit_cast(bf16x8_t, v);
}

constexpr int SHRINK_WAVES = 8;   // waves of a workgroup split the d_in range
constexpr int SHRINK_BATCH = 8;   // k-steps (of 32) whose loads are issued together

struct ShrinkDParams {
    const char *x, *A_stack;
    char *ug_hi, *ug_lo;
    const int *tok_sorted;
    const int4 *grp_meta;
    const int *n_groups;
    int d_in, r;
    float scale;
    int act;
};

// One (expert group g, 16-row slab of A_e) of the decode shrink; `red` is the
// workgroup's [SHRINK_WAVES][64][4] floats of LDS.
// KS_HOLD > 0 (batches beyond the small-batch size, whose group records hold up
// to GROUP_CHUNK tokens: several blocks of 16): a wave's share of the slab is at
// most KS_HOLD k-steps and stays in registers for all of the record's token
// blocks, instead of being fetched again for each.
template <int UNR, int KS_HOLD = 0>
__device__ __forceinline__ void decode_shrink_slab(const ShrinkDParams &p, int slab, int g,
                                                   float (*red)[64][4])
{
    constexpr int NW = SHRINK_WAVES;
    const char *__restrict__ x = p.x;
    const char *__restrict__ A_stack = p.A_stack;
    char *__restrict__ ug_hi = p.ug_hi;
    char *__restrict__ ug_lo = p.ug_lo;
    const int *__restrict__ tok_sorted = p.tok_sorted;
    const int4 *__restrict__ grp_meta = p.grp_meta;
    const int *__restrict__ n_groups = p.n_groups;
    const int d_in = p.d_in;
    const float scale = p.scale;
    (void)n_groups;   // records past the group count are empty
    const i32x4_t gm = sload_x4(grp_meta + g);
    const int e = gm.x;
    if (e < 0) return;
    const int gs = gm.y, ge = gm.z;
    if (ge <= gs) return;
    // the expert's own rank (a multiple of 8): slabs beyond it are never read, u is
    // stored [pos, p.r] and only its first r columns are written and later read
    const int r = min(p.r, gm.w);
    const int ldr = p.r;
    if (slab * 16 >= r) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // tokens of the first block of 16 positions (entries past the group's end are read --
    // the list is followed by more of the plan -- and not used)
    const i32x16_t toks = sload_x16(tok_sorted + gs);
    const int tok_first = pick16(toks, lane);
    const int tok_gs = toks[0];   // lanes past the group's end take its first token (in bounds, result unused)
    const int j0 = slab * 16;
    const int jrow = j0 + (lane & 15);
    const int kq = (lane >> 4) * 8;               // element offset of this lane's k-group
    const int64_t ld = (int64_t)d_in * 2;
    const char *arow = A_stack + ((int64_t)e * ldr + (jrow < r ? jrow : 0)) * ld;
    // each wave owns a contiguous run of k-steps: its 16 rows are read as 16
    // contiguous segments
    const int nks = (d_in + 31) / 32;
    const int per = (nks + NW - 1) / NW;
    const int ks_beg = wave * per;
    const int ks_end = min(nks, ks_beg + per);
    const int klen = min(d_in, ks_end * 32);

    bf16x8_t held[KS_HOLD > 0 ? KS_HOLD : 1];
    if constexpr (KS_HOLD > 0) {
#pragma unroll
        for (int u = 0; u < KS_HOLD; ++u) held[u] = ldg_frag(arow, (ks_beg + u) * 32 + kq, klen);   // past the range: zero
    }
    for (int t0 = gs; t0 < ge; t0 += 16) {
        const int pos = t0 + (lane & 15);
        const bool tvalid = pos < ge;
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
        int tok = tvalid ? tok_first : tok_gs;
        if (t0 != gs) tok = tok_sorted[tvalid ? pos : gs];
        const char *xrow = x + (int64_t)tok * ld;
        if constexpr (KS_HOLD > 0) {
#pragma unroll
            for (int u0 = 0; u0 < KS_HOLD; u0 += UNR) {
                if (ks_beg + u0 < ks_end) {   // the same for the whole wave
                    bf16x8_t b[UNR];
#pragma unroll
                    for (int u = 0; u < UNR; ++u) b[u] = ldg_frag(xrow, (ks_beg + u0 + u) * 32 + kq, klen);
#pragma unroll
                    for (int u = 0; u < UNR; ++u)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(held[u0 + u], b[u], acc, 0, 0, 0);
                }
            }
        } else
        for (int ks0 = ks_beg; ks0 < ks_end; ks0 += UNR) {
            // every load of the batch is issued before the first one is used
            uint4 ra[UNR], rb[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) ra[u] = ldg_raw(arow, (ks0 + u) * 32 + kq, klen);
#pragma unroll
            for (int u = 0; u < UNR; ++u) rb[u] = ldg_raw(xrow, (ks0 + u) * 32 + kq, klen);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int k = (ks0 + u) * 32 + kq;   // past the wave's range: zero
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag_of(ra[u], k, klen), frag_of(rb[u], k, klen), acc,
                                                              0, 0, 0);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) red[wave][lane][i] = acc[i];
        __syncthreads();
        if (wave == 0) {
            // lane holds u[token = lane % 16][j0 + 4 * (lane / 16) + i]; the
            // partial sums are added in wave order, so runs repeat bit for bit
            uint32_t h[4], l[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float f = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) f += red[w][lane][i];
                f = adapter_act(f, p.act) * scale;
                h[i] = f32_to_bf16_bits(f);
                l[i] = f32_to_bf16_bits(f - bf16_bits_to_f32(h[i]));
            }
            const int jj = j0 + 4 * (lane >> 4);
            if (tvalid && jj < r) {   // r % 8 == 0, so a group of 4 is all in or all out
                const int64_t off = ((int64_t)pos * ldr + jj) * 2;
                *reinterpret_cast<uint2 *>(ug_hi + off) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                *reinterpret_cast<uint2 *>(ug_lo + off) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
            }
        }
        __syncthreads();
    }
}

// What differs between the projections of one call that read the same x (gate, up; q, k, v): they
// share the token groups, d_in, r, the scale and the number of base parts, so their base tiles, their
// shrink slabs and their expand blocks stand side by side in the call's two launches and the
// launches' ramp and tail are paid once.  Entry 0 repeats what the plain parameter blocks hold.
struct DecodeMore {
    int n;                          // projections of the call (1..MAX_SHARED_X)
    int base_first[MAX_SHARED_X];   // first base-role workgroup of each (multiples of 8)
    int xb_first[MAX_SHARED_X];     // first expand row block of each
    const char *W[MAX_SHARED_X], *A_stack[MAX_SHARED_X], *B_stack[MAX_SHARED_X];
    char *ug_hi[MAX_SHARED_X], *ug_lo[MAX_SHARED_X], *y[MAX_SHARED_X];
    float *ybase[MAX_SHARED_X];
    int d_out[MAX_SHARED_X], n_tiles_n[MAX_SHARED_X];
};

// grid (ceil(r / 16), max_groups): the slabs of one expert are neighbours in
// dispatch order, so its rows of A_e stream from HBM as one contiguous run.
template <int KS_HOLD>
__global__ __launch_bounds__(SHRINK_WAVES * 64) void decode_shrink_kernel(ShrinkDParams p)
{
    __shared__ float red[SHRINK_WAVES][64][4];
    decode_shrink_slab<SHRINK_BATCH, KS_HOLD>(p, (int)blockIdx.x, (int)blockIdx.y, red);
}

// Base GEMM tiles and shrink slabs in one launch: the two are independent, the
// shrink is bound by HBM and the base GEMM by the latency of its short serial
// loops, so side by side the base GEMM costs little time of its own.  The
// first `n_base` workgroups take base tiles (dispatched first, they run
// longest), the others one shrink slab each.
static_assert(CfgDecodeBase::NT == SHRINK_WAVES * 64, "both roles share one workgroup size");
// With several projections in the call (`m`): the base tiles of all of them first, then the slabs of
// all of them, `slabs_per_proj` each.
__global__ __launch_bounds__(SHRINK_WAVES * 64) void decode_base_shrink_kernel(LinearKParams lp, ShrinkDParams sp,
                                                                             DecodeMore m, int n_base, int n_slabs,
                                                                             int slabs_per_proj)
{
    extern __shared__ __align__(16) char smem[];
    if ((int)blockIdx.x < n_base) {
        int first = 0;
        // (picked by comparison, not by indexing: indexing the parameter arrays would put them in scratch)
#pragma unroll
        for (int i = 1; i < MAX_SHARED_X; ++i)
            if (i < m.n && (int)blockIdx.x >= m.base_first[i]) {
                first = m.base_first[i];
                lp.W = m.W[i];
                lp.y = reinterpret_cast<char *>(m.ybase[i]);
                lp.d_out = m.d_out[i];
                lp.n_tiles_n = m.n_tiles_n[i];
            }
        linear_tile<CfgDecodeBase>(lp, (int)blockIdx.x - first, smem);
    } else {
        // (the shrink role keeps its partial sums where the base role keeps its stages)
        int idx = (int)blockIdx.x - n_base;
#pragma unroll
        for (int i = 1; i < MAX_SHARED_X; ++i)
            if (i < m.n && idx >= slabs_per_proj) {
                idx -= slabs_per_proj;
                sp.A_stack = m.A_stack[i];
                sp.ug_hi = m.ug_hi[i];
                sp.ug_lo = m.ug_lo[i];
            }
        decode_shrink_slab<SHRINK_BATCH>(sp, idx % n_slabs, idx / n_slabs,
                                         reinterpret_cast<float(*)[64][4]>(smem));
    }
}

struct ExpandKParams {
    const char *B_stack, *ug_hi, *ug_lo;
    const float *ybase;        // [k_splits, T, d_out]
    char *y;
    const int *tok_sorted;
    const int4 *grp_meta;
    const int *n_groups;
    int64_t T;
    int d_out, r, k_splits, y_f32;
};

constexpr int EXPAND_WAVES = 4;

__device__ __forceinline__ void store_out(const ExpandKParams &p, int tok, int o, f32x4_t v)
{
    const int64_t at = (int64_t)tok * p.d_out + o;
    if (p.y_f32) {
        *reinterpret_cast<f32x4_t *>(p.y + at * 4) = v;
    } else {
        *reinterpret_cast<uint2 *>(p.y + at * 2) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
    }
}

// One (expert group, slab of EXPAND_WAVES * RB * 16 output rows).  KS_HOLD > 0:
// r <= 32 * KS_HOLD, the wave's RB x KS_HOLD fragments of B_e are requested at once
// and held across the group's token blocks; KS_HOLD == 0: any r, fragment by
// fragment.  The accumulators start from the base result, so y leaves in one pass.
// FULL (wave-uniform): the expert's rank is exactly 32 * KS_HOLD, so no fragment
// needs its tail cut off: loads take constant offsets from a few row addresses and
// nothing is masked.
// BY_POS: the rows of the base partial planes follow the by-expert token order (the
// small-batch base product gathers its rows that way), so nothing a workgroup
// loads depends on another load: adapter rows, u, base sums and token indices are
// all requested at once, and the token index is needed only to place the result.
// Phase 1 of a token block issues every load (for the first block also B_e, the HBM
// traffic); phase 2 consumes them; a scheduling barrier between the two keeps all
// loads ahead of the first wait.
template <int KS_HOLD, int NSPLIT, bool BY_POS, int RB, bool FULL>
__device__ __forceinline__ void expand_item(const ExpandKParams &p, int slab, int e, int gs, int ge, int r)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int o_base = (slab * EXPAND_WAVES + wave) * (RB * 16);
    const int d_out = p.d_out;
    if (o_base >= d_out) return;
    const int kq = (lane >> 4) * 8;
    // rows of B_e and u are p.r long; the expert's own rank r (a multiple of 8) says how
    // much of them exists -- fragments past it are zero-filled, not read
    const int64_t ldb = (int64_t)p.r * 2;
    const char *bexp = p.B_stack + (int64_t)(e < 0 ? 0 : e) * d_out * ldb;
    const bool lora = e >= 0 && r > 0;
    constexpr int KH = KS_HOLD > 0 ? KS_HOLD : 1;
    auto ld_frag = [&](const char *row, int ks) __attribute__((always_inline)) -> uint4 {
        if constexpr (FULL) return *reinterpret_cast<const uint4 *>(row + ks * 64);   // row already at kq
        else return ldg_raw(row, ks * 32 + kq, r);
    };
    auto as_frag = [&](uint4 v, int ks) __attribute__((always_inline)) -> bf16x8_t {
        if constexpr (FULL) return __builtin_bit_cast(bf16x8_t, v);
        else return frag_of(v, ks * 32 + kq, r);
    };
    const int koff = FULL ? kq * 2 : 0;

    uint4 a[RB][KH];
    if constexpr (KS_HOLD > 0) {
        if (lora) {
#pragma unroll
            for (int c = 0; c < RB; ++c) {
                const int orow = o_base + c * 16 + (lane & 15);
                const char *brow = bexp + (int64_t)(orow < d_out ? orow : 0) * ldb + koff;
#pragma unroll
                for (int ks = 0; ks < KS_HOLD; ++ks) a[c][ks] = ld_frag(brow, ks);
            }
        }
    }

    for (int t0 = gs; t0 < ge; t0 += 16) {
        const int pos = t0 + (lane & 15);
        const bool tvalid = pos < ge;
        const int ps = tvalid ? pos : gs;
        const int tok = p.tok_sorted[ps];
        int brow_idx = ps;
        if constexpr (!BY_POS) brow_idx = tok;
        // lane holds y[token = lane % 16][o_base + c*16 + 4*(lane/16) + i]; rows
        // past d_out read (and never store) the last valid group of four
        f32x4_t part[RB][NSPLIT];
        {
            const int64_t plane = p.T * (int64_t)d_out;
#pragma unroll
            for (int c = 0; c < RB; ++c) {
                const int oo = min(o_base + c * 16 + 4 * (lane >> 4), d_out - 4);
                const float *src = p.ybase + (int64_t)brow_idx * d_out + oo;
#pragma unroll
                for (int sp = 0; sp < NSPLIT; ++sp) part[c][sp] = *reinterpret_cast<const f32x4_t *>(src + sp * plane);
            }
        }
        const char *uh = p.ug_hi + (int64_t)ps * ldb + koff;
        const char *ul = p.ug_lo + (int64_t)ps * ldb + koff;
        uint4 rh[KH], rl[KH];
        if constexpr (KS_HOLD > 0) {
            if (lora) {
#pragma unroll
                for (int ks = 0; ks < KS_HOLD; ++ks) {
                    rh[ks] = ld_frag(uh, ks);
                    rl[ks] = ld_frag(ul, ks);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        f32x4_t acc[RB];
#pragma unroll
        for (int c = 0; c < RB; ++c) {
            acc[c] = part[c][0];   // parts are added in order: repeatable
#pragma unroll
            for (int sp = 1; sp < NSPLIT; ++sp) acc[c] += part[c][sp];
        }
        if (lora) {
            if constexpr (KS_HOLD > 0) {
#pragma unroll
                for (int ks = 0; ks < KS_HOLD; ++ks) {
                    const bf16x8_t fh = as_frag(rh[ks], ks), fl = as_frag(rl[ks], ks);
#pragma unroll
                    for (int c = 0; c < RB; ++c) {
                        const bf16x8_t fa = as_frag(a[c][ks], ks);
                        acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fh, acc[c], 0, 0, 0);
                        acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fl, acc[c], 0, 0, 0);
                    }
                }
            } else {
                const int nks = (r + 31) / 32;
#pragma unroll
                for (int c = 0; c < RB; ++c) {
                    const int orow = o_base + c * 16 + (lane & 15);
                    const char *brow = bexp + (int64_t)(orow < d_out ? orow : 0) * ldb;
                    for (int ks = 0; ks < nks; ++ks) {
                        const int k = ks * 32 + kq;
                        const bf16x8_t ab = ldg_frag(brow, k, r);
                        const bf16x8_t bh = ldg_frag(p.ug_hi + (int64_t)ps * ldb, k, r);
                        const bf16x8_t bl = ldg_frag(p.ug_lo + (int64_t)ps * ldb, k, r);
                        acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab, bh, acc[c], 0, 0, 0);
                        acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab, bl, acc[c], 0, 0, 0);
                    }
                }
            }
        }
#pragma unroll
        for (int c = 0; c < RB; ++c) {
            const int oo = o_base + c * 16 + 4 * (lane >> 4);
            if (tvalid && oo < d_out) store_out(p, tok, oo, acc[c]);   // d_out % 4 == 0
        }
    }
}

// grid (ceil(d_out / (EXPAND_WAVES * RB * 16)), max_groups)
// With several projections in the call (`m`): grid.x holds the row blocks of all of them.
template <int KS_HOLD, int NSPLIT, bool BY_POS, int RB>
__global__ __launch_bounds__(EXPAND_WAVES * 64) void decode_expand_kernel(ExpandKParams p, DecodeMore m)
{
    const i32x4_t gm = sload_x4(p.grp_meta + blockIdx.y);   // records past the group count are empty
    const int e = gm.x, gs = gm.y, ge = gm.z;
    if (ge <= gs) return;
    const int r = min(p.r, gm.w);
    int first = 0;
#pragma unroll
    for (int i = 1; i < MAX_SHARED_X; ++i)
        if (i < m.n && (int)blockIdx.x >= m.xb_first[i]) {
            first = m.xb_first[i];
            p.B_stack = m.B_stack[i];
            p.ug_hi = m.ug_hi[i];
            p.ug_lo = m.ug_lo[i];
            p.ybase = m.ybase[i];
            p.y = m.y[i];
            p.d_out = m.d_out[i];
        }
    const int slab = (int)blockIdx.x - first;
    if (KS_HOLD > 0 && r == KS_HOLD * 32)
        expand_item<KS_HOLD, NSPLIT, BY_POS, RB, true>(p, slab, e, gs, ge, r);
    else
        expand_item<KS_HOLD, NSPLIT, BY_POS, RB, false>(p, slab, e, gs, ge, r);
}

static ShrinkDParams shrink_params(const PlanView &pv, const DecodeArgs &d)
{
    const LinearArgs &a = d.lin;
    ShrinkDParams p;
    p.x = (const char *)a.x; p.A_stack = (const char *)a.A_stack;
    p.ug_hi = (char *)d.ug_hi; p.ug_lo = (char *)d.ug_lo;
    p.tok_sorted = pv.tok_sorted; p.grp_meta = pv.grp_meta; p.n_groups = pv.n_groups;
    p.d_in = a.d_in; p.r = a.r; p.scale = a.scale; p.act = a.act;
    return p;
}

hipError_t launch_decode_shrink(const PlanView &pv, const DecodeArgs &d, hipStream_t stream)
{
    const LinearArgs &a = d.lin;
    if (a.r <= 0 || pv.max_groups <= 0) return hipSuccess;
    dim3 grid((unsigned)((a.r + 15) / 16), (unsigned)pv.max_groups);
    // k-steps of 32 per wave
    const int per = ((a.d_in + 31) / 32 + SHRINK_WAVES - 1) / SHRINK_WAVES;
    const ShrinkDParams p = shrink_params(pv, d);
    // holding 24 k-steps costs occupancy: worth it only where records tend to span several token
    // blocks, i.e. not with about one token per group (4 tokens per possible group on average is
    // where it began to pay on the 5632-wide projection)
    const bool several_blocks = pv.T >= 4 * std::min<int64_t>(pv.S, (int64_t)pv.E + 1);
    if (pv.T > DECODE_MAX_T && per <= 8)
        hipLaunchKernelGGL(decode_shrink_kernel<8>, grid, dim3(SHRINK_WAVES * 64), 0, stream, p);
    else if (pv.T > DECODE_MAX_T && per <= 24 && several_blocks)
        hipLaunchKernelGGL(decode_shrink_kernel<24>, grid, dim3(SHRINK_WAVES * 64), 0, stream, p);
    else
        hipLaunchKernelGGL(decode_shrink_kernel<0>, grid, dim3(SHRINK_WAVES * 64), 0, stream, p);
    return hipGetLastError();
}

bool decode_base_shrink_fits(const PlanView &pv, const DecodeArgs &d)
{
    return d.lin.r > 0 && pv.max_groups > 0 && pv.T > 0 &&
           decode_base_shape(pv.T, d.lin.d_in, d.lin.d_out).dma;
}

hipError_t prepare_decode_kernels()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&decode_base_shrink_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, CfgDecodeBase::SMEM_BYTES);
}

// True when the n projections of a call that share x can share its two launches: the same input,
// contraction length, rank, scale, activation, output type and number of base parts.
bool decode_shared_fits(const PlanView &pv, const DecodeArgs *d, int n)
{
    if (n < 1 || n > MAX_SHARED_X) return false;
    for (int i = 0; i < n; ++i) {
        if (!decode_base_shrink_fits(pv, d[i])) return false;
        const LinearArgs &a = d[i].lin, &a0 = d[0].lin;
        if (a.x != a0.x || a.d_in != a0.d_in || a.r != a0.r || a.scale != a0.scale || a.act != a0.act ||
            a.y_f32 != a0.y_f32 || d[i].k_splits != d[0].k_splits || d[i].ybase_by_pos != d[0].ybase_by_pos)
            return false;
    }
    return true;
}

static DecodeMore decode_more(const DecodeArgs *d, int n)
{
    DecodeMore m;
    m.n = n;
    for (int i = 0; i < MAX_SHARED_X; ++i) {
        const DecodeArgs &q = d[i < n ? i : 0];
        m.base_first[i] = m.xb_first[i] = 0;
        m.W[i] = (const char *)q.lin.W; m.A_stack[i] = (const char *)q.lin.A_stack;
        m.B_stack[i] = (const char *)q.lin.B_stack;
        m.ug_hi[i] = (char *)q.ug_hi; m.ug_lo[i] = (char *)q.ug_lo; m.y[i] = (char *)q.lin.y;
        m.ybase[i] = q.ybase;
        m.d_out[i] = q.lin.d_out; m.n_tiles_n[i] = 0;
    }
    return m;
}

hipError_t launch_decode_base_shrink_shared(const PlanView &pv, const DecodeArgs *d, int n, hipStream_t stream)
{
    if (!decode_shared_fits(pv, d, n)) return hipErrorInvalidValue;
    const LinearArgs &a = d[0].lin;
    DecodeMore m = decode_more(d, n);
    int64_t n_base = 0;
    LinearKParams lp{};
    for (int i = 0; i < n; ++i) {
        const DecodeBaseShape sh = decode_base_shape(pv.T, a.d_in, d[i].lin.d_out);
        if (!sh.dma || sh.k_splits != d[i].k_splits) return hipErrorInvalidValue;
        if (i == 0) lp = decode_base_params(pv, a, d[0].ybase, 1, sh, pv.tok_sorted);   // rows in by-expert order
        m.base_first[i] = (int)n_base;
        m.n_tiles_n[i] = sh.n_tiles_n;
        n_base += sh.grid;   // (a multiple of 8: every projection's tiles keep their place in the XCD rotation)
    }
    const int n_slabs = (a.r + 15) / 16;
    const int64_t per_proj = (int64_t)n_slabs * pv.max_groups;
    const int64_t grid = n_base + per_proj * n;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(decode_base_shrink_kernel, dim3((unsigned)grid), dim3(SHRINK_WAVES * 64),
                       CfgDecodeBase::SMEM_BYTES, stream, lp, shrink_params(pv, d[0]), m, (int)n_base, n_slabs,
                       (int)per_proj);
    return hipGetLastError();
}

hipError_t launch_decode_base_shrink(const PlanView &pv, const DecodeArgs &d, hipStream_t stream)
{
    return launch_decode_base_shrink_shared(pv, &d, 1, stream);
}

hipError_t launch_decode_expand_shared(const PlanView &pv, const DecodeArgs *d, int n, hipStream_t stream)
{
    if (n < 1 || n > MAX_SHARED_X) return hipErrorInvalidValue;
    if (pv.max_groups <= 0) return hipSuccess;
    const LinearArgs &a = d[0].lin;
    for (int i = 1; i < n; ++i)
        if (d[i].lin.r != a.r || d[i].k_splits != d[0].k_splits || d[i].lin.y_f32 != a.y_f32 ||
            d[i].ybase_by_pos != d[0].ybase_by_pos)
            return hipErrorInvalidValue;
    ExpandKParams p;
    p.B_stack = (const char *)a.B_stack; p.ug_hi = (const char *)d[0].ug_hi; p.ug_lo = (const char *)d[0].ug_lo;
    p.ybase = d[0].ybase; p.y = (char *)a.y;
    p.tok_sorted = pv.tok_sorted; p.grp_meta = pv.grp_meta; p.n_groups = pv.n_groups;
    p.T = pv.T; p.d_out = a.d_out; p.r = a.r; p.k_splits = d[0].k_splits; p.y_f32 = a.y_f32;
    constexpr int RB = 4;   // 16-row blocks per wave: 64 KB of B_e per workgroup and rank-128 adapter
    const int rows = EXPAND_WAVES * RB * 16;
    DecodeMore m = decode_more(d, n);
    int64_t xb = 0;
    for (int i = 0; i < n; ++i) {
        m.xb_first[i] = (int)xb;
        xb += (d[i].lin.d_out + rows - 1) / rows;
    }
    if (xb > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)xb, (unsigned)pv.max_groups);
    const int nks = (a.r + 31) / 32;
#define MOIN_EXPAND_R(KS, NS, BP) \
    hipLaunchKernelGGL((decode_expand_kernel<KS, NS, BP, RB>), grid, dim3(EXPAND_WAVES * 64), 0, stream, p, m)
#define MOIN_EXPAND_S(KS, NS)                                                                                  \
    do {                                                                                                       \
        if (d[0].ybase_by_pos) MOIN_EXPAND_R(KS, NS, true);                                                    \
        else MOIN_EXPAND_R(KS, NS, false);                                                                     \
    } while (0)
#define MOIN_EXPAND(KS)                                  \
    switch (d[0].k_splits) {                             \
    case 1: MOIN_EXPAND_S(KS, 1); break;                 \
    case 2: MOIN_EXPAND_S(KS, 2); break;                 \
    case 3: MOIN_EXPAND_S(KS, 3); break;                 \
    case 4: MOIN_EXPAND_S(KS, 4); break;                 \
    default: return hipErrorInvalidValue;                \
    }
    if (nks <= 1) MOIN_EXPAND(1)
    else if (nks <= 2) MOIN_EXPAND(2)
    else if (nks <= 4) MOIN_EXPAND(4)
    else MOIN_EXPAND(0)
#undef MOIN_EXPAND
#undef MOIN_EXPAND_S
#undef MOIN_EXPAND_R
    return hipGetLastError();
}

hipError_t launch_decode_expand(const PlanView &pv, const DecodeArgs &d, hipStream_t stream)
{
    return launch_decode_expand_shared(pv, &d, 1, stream);
}

}  // namespace moin
