// The tiled linear kernel shared by the prefill fallback, the decode base GEMM
// and the decode kernel that runs base tiles and shrink slabs side by side.
#pragma once
#include "gemm_core.h"
#include "kernels.h"

namespace moin {

struct LinearKParams {
    const char *x, *W, *B_stack;
    const char *u_hi, *u_lo;
    char *y;
    const int *tile_row0, *tile_rows, *tile_expert, *tile_rank, *n_tiles;
    int64_t T;
    int d_in, d_out, r;
    int n_tiles_n;
    int y_f32;
    int plain_tiles;         // 1: tiles are the regular grid over T, no adapters in-kernel
    const int *gather;       // plain tiles only, or null: row i of the product is x[gather[i]] W^T (the
                             // decode path's tokens in their by-expert order)
    int k_splits;            // plain tiles only: parts of the contraction range, one output plane each
    int kb_per_split;        // BK blocks per part
};

// One output tile: `bid` is the workgroup's index in a grid of (tiles rounded
// up to a multiple of 8) workgroups, `smem` its C::SMEM_BYTES of LDS.
template <class C>
__device__ __forceinline__ void linear_tile(const LinearKParams &p, int bid, char *smem)
{
    int ntm, row0, rows, e;
    int re = 0;   // the tile's adapter rank (at most p.r)
    int id;
    int kb_lo = 0, kb_hi = (p.d_in + C::BK - 1) / C::BK;   // BK blocks of the base contraction
    int split = 0;
    if (p.plain_tiles) {
        // id = ((n tile * k_splits + part) * ntm + m tile): the tiles that share a
        // slab of W are neighbours
        ntm = (int)((p.T + C::BM - 1) / C::BM);
        const int raw = xcd_band_id(bid, ntm * p.n_tiles_n * p.k_splits);
        if (raw < 0) return;
        const int tm = uniform(raw % ntm);
        const int rest = uniform(raw / ntm);
        split = rest % p.k_splits;
        id = tm * p.n_tiles_n + rest / p.k_splits;
        row0 = tm * C::BM;
        rows = (int)min((int64_t)C::BM, p.T - row0);
        e = -1;
        kb_lo = split * p.kb_per_split;
        kb_hi = min(kb_hi, kb_lo + p.kb_per_split);
    } else {
        // plan tiles are TILE_M rows; this kernel's BM divides TILE_M
        constexpr int SUB = TILE_M / C::BM;
        ntm = uniform(*p.n_tiles) * SUB;
        id = xcd_band_id(bid, ntm * p.n_tiles_n);
        if (id < 0) return;
        const int tm = uniform(id / p.n_tiles_n);
        const int t = tm / SUB, sub = tm % SUB;
        rows = uniform(p.tile_rows[t]) - sub * C::BM;
        if (rows <= 0) return;
        rows = min(rows, C::BM);
        row0 = uniform(p.tile_row0[t]) + sub * C::BM;
        e = uniform(p.tile_expert[t]);
        re = min(p.r, uniform(p.tile_rank[t]));
    }
    const int tn = uniform(id % p.n_tiles_n);
    const int n0 = tn * C::BN;
    const int ncols = min(C::BN, p.d_out - n0);

    const uint32_t ldx = (uint32_t)p.d_in * 2u, ldu = (uint32_t)p.r * 2u;
    const bool lora = (e >= 0) && re > 0;
    const int nkb0 = kb_hi - kb_lo;
    // adapter blocks up to the expert's own rank (the shrink wrote zeros from there to the block end)
    const int nkb1 = lora ? (re + C::BK - 1) / C::BK : 0;
    // adapter operands are harmless aliases of x / W when the tile has no adapter
    const char *uh = lora ? p.u_hi + (int64_t)row0 * ldu : p.x;
    const char *ul = lora ? p.u_lo + (int64_t)row0 * ldu : p.x;
    const char *be = lora ? p.B_stack + ((int64_t)e * p.d_out + n0) * ldu : p.W;

    typename C::Acc acc;
    C::zero(acc);
    if constexpr (C::IS_DMA) {
        const char *xa = p.x + (int64_t)row0 * ldx;
        const char *wb = p.W + (int64_t)n0 * ldx;
        auto la = C::template make_lanes<C::A_I>(rows);
        const auto lb = C::template make_lanes<C::B_I>(ncols);
        if (p.plain_tiles && p.gather) {
            // each lane's tile row becomes the token that stands at that position
#pragma unroll
            for (int j = 0; j < C::A_I; ++j) la.row[j] = (uint32_t)p.gather[row0 + (int)la.row[j]];
            xa = p.x;
        }
        // Block sequence: base blocks first, then the adapter blocks (the high
        // part of u, then the remainder); only uniform scalars differ between
        // them.  Written out here rather than through a callable: the operand
        // choice then stays a select of register values.
        const int total = nkb0 + 2 * nkb1;
#define MOIN_ISSUE_BLOCK(blk, stage)                                                      \
    do {                                                                                  \
        const int b_ = (blk);                                                             \
        const bool base_ = b_ < nkb0;                                                     \
        const int j_ = b_ - nkb0;                                                         \
        const bool hi_ = j_ < nkb1;                                                       \
        const char *pa_ = base_ ? xa : (hi_ ? uh : ul);                                   \
        const char *pb_ = base_ ? wb : be;                                                \
        const uint32_t ld_ = base_ ? ldx : ldu;                                           \
        const int kb_ = base_ ? b_ + kb_lo : (hi_ ? j_ : j_ - nkb1);                      \
        C::issue((stage), pa_, ld_, la, pb_, ld_, lb, (uint32_t)kb_ * (C::BK * 2));       \
    } while (0)
#pragma unroll
        for (int s = 0; s < C::NS - 1; ++s)
            if (s < total) MOIN_ISSUE_BLOCK(s, smem + s * C::STAGE_BYTES);
        int st = 0;
        for (int it = 0; it < total; ++it) {
            if (it + C::NS - 2 < total) wait_vm_then_barrier<(C::NS - 2) * C::LPB>();
            else wait_vm_then_barrier<0>();
            const int nb = it + C::NS - 1;
            const int ns = (st == 0) ? C::NS - 1 : st - 1;
            if (nb < total) MOIN_ISSUE_BLOCK(nb, smem + ns * C::STAGE_BYTES);
            C::compute_stage(smem + st * C::STAGE_BYTES, acc);
            st = (st + 1 == C::NS) ? 0 : st + 1;
        }
        __syncthreads();
#undef MOIN_ISSUE_BLOCK
    } else {
        auto vx = C::template make_view<C::A_CH>(p.x + (int64_t)row0 * ldx, ldx, rows);
        if (p.plain_tiles && p.gather) {
            vx.base = p.x;
#pragma unroll
            for (int i = 0; i < C::A_CH; ++i)
                vx.rowoff[i] = (uint32_t)p.gather[row0 + (int)(vx.rowoff[i] / ldx)] * ldx;
        }
        const auto vw = C::template make_view<C::B_CH>(p.W + (int64_t)n0 * ldx, ldx, ncols);
        const auto vuh = C::template make_view<C::A_CH>(uh, ldu, rows);
        const auto vul = C::template make_view<C::A_CH>(ul, ldu, rows);
        const auto vb = C::template make_view<C::B_CH>(be, ldu, ncols);
        auto issue = [=](int it, typename C::Stage &g) __attribute__((always_inline)) {
            if (it < nkb0) {
                C::load_stage(g, vx, vw, (uint32_t)(it + kb_lo) * (C::BK * 2), ldx);
            } else if (it < nkb0 + nkb1) {
                C::load_stage(g, vuh, vb, (uint32_t)(it - nkb0) * (C::BK * 2), ldu);
            } else {
                C::load_stage(g, vul, vb, (uint32_t)(it - nkb0 - nkb1) * (C::BK * 2), ldu);
            }
        };
        pipelined_blocks<C>(smem, nkb0 + 2 * nkb1, issue, acc);
    }

    const int64_t ldy = (int64_t)p.d_out * (p.y_f32 ? 4 : 2);
    char *yb = p.y + ((int64_t)split * p.T + row0) * ldy;
    C::epilogue(smem, acc, [&](int row, int col, float(&v)[8]) {
        if (row >= rows || col >= ncols) return;
        const int gc = n0 + col;
        if (p.y_f32) {
            float *dst = reinterpret_cast<float *>(yb + (int64_t)row * ldy) + gc;
            *reinterpret_cast<f32x4_t *>(dst) = f32x4_t{v[0], v[1], v[2], v[3]};
            *reinterpret_cast<f32x4_t *>(dst + 4) = f32x4_t{v[4], v[5], v[6], v[7]};
        } else {
            uint4 o;
            o.x = pack_bf16x2(v[0], v[1]);
            o.y = pack_bf16x2(v[2], v[3]);
            o.z = pack_bf16x2(v[4], v[5]);
            o.w = pack_bf16x2(v[6], v[7]);
            *reinterpret_cast<uint4 *>(yb + (int64_t)row * ldy + (int64_t)gc * 2) = o;
        }
    });
}

template <class C>
__global__ __launch_bounds__(C::NT) void linear_kernel(LinearKParams p)
{
    extern __shared__ __align__(16) char smem[];
    linear_tile<C>(p, (int)blockIdx.x, smem);
}

// Decode base GEMM, contraction length a multiple of 64: 8 waves, wave patch
// 64 x 32, four 16 KB stages.  64 KB of LDS lets two workgroups share a compute
// unit, and the workgroup size matches the decode shrink's, so both kinds of
// workgroup can live in one launch.
using CfgDecodeBase = DmaCore<128, 128, 32, 2, 4, 4>;
using CfgThin = GemmCore<128, 64, 64, 2, 2>;         // decode base GEMM, any contraction length: 4 waves, 64 x 32

// How the decode base GEMM of a shape is cut up.
struct DecodeBaseShape {
    int dma;            // 1: CfgDecodeBase, 0: CfgThin
    int k_splits, kb_per_split;
    int n_tiles_n;
    int64_t m_tiles;
    int grid;           // workgroups, a multiple of 8
};
DecodeBaseShape decode_base_shape(int64_t T, int d_in, int d_out);
// gather: null, or the plan's token order (rows of the result then follow that order)
LinearKParams decode_base_params(const PlanView &pv, const LinearArgs &a, void *out, int out_f32,
                                 const DecodeBaseShape &sh, const int *gather);

}  // namespace moin
