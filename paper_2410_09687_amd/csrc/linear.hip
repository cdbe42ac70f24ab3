// Prefill path of the routed LoRA linear layer (Section 3.2:
// y = W x + W_b (W_a x), one adapter per sequence).
//
//   shrink : u = scale * x A_e^T, written as a bf16 pair (u_hi + u_lo) so the
//            expand product sees ~16 significant bits of u.
//   linear : y = x W^T + u_hi B_e^T + u_lo B_e^T  -- the adapter term is simply
//            2r more contraction steps appended to the base GEMM of the same
//            output tile, so y is written once, from one fp32 accumulator.
// Tiles come from the plan: no tile spans two sequences, hence one adapter per
// tile.  The same linear kernel, in a smaller tile shape and over a regular
// grid of tiles, is the decode path's base GEMM; there the contraction range
// may be cut into several parts, each writing its own fp32 partial result.
#include "gemm_core.h"
#include "kernels.h"
#include "linear_tile.h"

namespace moin {


struct ShrinkKParams {
    const char *x, *A_stack;
    char *u_hi, *u_lo;
    // projections that share x: column tile tn belongs to projection tn / tiles_per_proj
    // (A_stack / u_hi / u_lo above are then those of projection 0)
    int n_proj, tiles_per_proj;
    const char *A_more[MAX_SHARED_X - 1];
    char *uh_more[MAX_SHARED_X - 1], *ul_more[MAX_SHARED_X - 1];
    const int *tile_row0, *tile_rows, *tile_expert, *tile_rank, *n_tiles;
    int d_in, r;
    int n_tiles_n;
    float scale;
    int act;
    // QUANT only: MXFP8 codes [T, d_in] and scale bytes [d_in / 128, T, 4] of x
    char *xq, *xs;
    int64_t T;
};

// MXFP8 quantisation of one thread's 8 consecutive values of x (w: four words of
// two bf16 each) whose block of 32 lies in four neighbouring lanes: the block's
// scale byte E = max(0, exponent field of the largest magnitude - 8), 127 for a
// block of zeros; elements = value / 2^(E - 127), clamped to +-448, rounded to
// nearest even ("Future Works", quantising the base model; OCP Microscaling
// format).  Returns the 8 codes; E through `scale_byte`.
__device__ __forceinline__ uint2 mx_quantize8(const uint4 &v, int &scale_byte)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t m = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        m = max(m, w[i] & 0x7FFFu);
        m = max(m, (w[i] >> 16) & 0x7FFFu);
    }
    m = max(m, (uint32_t)__shfl_xor((int)m, 1));
    m = max(m, (uint32_t)__shfl_xor((int)m, 2));
    const int E = m == 0 ? 127 : max(0, (int)(m >> 7) - 8);
    const float inv = bits_f32((uint32_t)(254 - E) << 23);   // 2^(127 - E)
    float f[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = fminf(fmaxf(bits_f32(w[i] << 16) * inv, -448.f), 448.f);
        f[2 * i + 1] = fminf(fmaxf(bits_f32(w[i] & 0xFFFF0000u) * inv, -448.f), 448.f);
    }
    int lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], 0, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
    int hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], 0, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
    scale_byte = E;
    return make_uint2((uint32_t)lo, (uint32_t)hi);
}

// QUANT (register-staged tile shapes with BK = 64, d_in a multiple of 128): the
// pass over x also writes x in MXFP8 for the quantised-base layer, so that x
// comes from HBM once for both.  The workgroups of the first column tile do it,
// also for tiles without an adapter, which the plain shrink skips.
template <class C, bool QUANT = false>
__global__ __launch_bounds__(C::NT) void shrink_kernel(ShrinkKParams p)
{
    extern __shared__ __align__(16) char smem[];
    constexpr int SUB = TILE_M / C::BM;
    const int ntm = uniform(*p.n_tiles) * SUB;
    // neighbouring sub-tiles share A_e: keep them on one XCD so that its L2
    // fetches each adapter slab from HBM once
    const int id = xcd_band_id(blockIdx.x, ntm * p.n_tiles_n);
    if (id < 0) return;
    const int tm = uniform(id / p.n_tiles_n), tn = uniform(id % p.n_tiles_n);
    const int t = tm / SUB, sub = tm % SUB;
    const int e = uniform(p.tile_expert[t]);
    int rows = uniform(p.tile_rows[t]) - sub * C::BM;
    const bool quant = QUANT && tn == 0;
    if (rows <= 0 || (e < 0 && !quant)) return;
    rows = min(rows, C::BM);
    const int row0 = uniform(p.tile_row0[t]) + sub * C::BM;
    const int proj = tn / p.tiles_per_proj;
    const int n0 = (tn - proj * p.tiles_per_proj) * C::BN;
    const char *A_stack = p.A_stack;
    char *u_hi = p.u_hi, *u_lo = p.u_lo;
#pragma unroll
    for (int i = 1; i < MAX_SHARED_X; ++i)
        if (proj == i) {   // (selected one by one: indexing the arrays would put the parameters in scratch)
            A_stack = p.A_more[i - 1];
            u_hi = p.uh_more[i - 1];
            u_lo = p.ul_more[i - 1];
        }
    // the expert's own rank: rows of A_e beyond it do not exist; the main kernel
    // reads u in blocks of 64 columns, so the rest of the last block is written as zeros
    const int re = e < 0 ? 0 : min(p.r, uniform(p.tile_rank[t]));
    const int r_read = min(p.r, (re + 63) & ~63);
    const bool shrink = n0 < r_read;
    if (!shrink && !quant) return;
    const int ncols = max(1, min(C::BN, re - n0));      // rows of A_e to fetch (at least one, in bounds)
    const int ncols_out = min(C::BN, r_read - n0);      // columns of u to write

    const uint32_t ldx = (uint32_t)p.d_in * 2u;
    const char *xa = p.x + (int64_t)row0 * ldx;
    // (a walk for the quantiser alone puts x in A_e's place: valid addresses, unused products)
    const char *ae = shrink ? A_stack + ((int64_t)e * p.r + n0) * ldx : xa;
    const int nkb = (p.d_in + C::BK - 1) / C::BK;

    // Workgroups that start together would all ask for the same 128 bytes of their rows, one row
    // pitch (4 KB and up) apart from the next: requests that pile up on a few memory channels.  Each
    // 256-row tile therefore starts its walk over the contraction at another block and wraps round
    // (the sub-tiles of a tile, and the projections that share x, keep one phase so that they meet
    // in L2): 88 -> 70 us for a 65536 x 2048 pass at rank 128.  The phase comes from the tile's
    // position in the batch, not from its place in the by-expert order, and is the same in every
    // variant of this kernel, so that a row's sum depends neither on how the experts are numbered
    // nor on which variant ran.
    const int k_first = (int)(((uint32_t)(row0 - sub * C::BM) / (uint32_t)TILE_M * 5u) % (uint32_t)nkb);
    auto block_of = [=](int it) __attribute__((always_inline)) {
        const int kb = it + k_first;
        return kb >= nkb ? kb - nkb : kb;
    };

    typename C::Acc acc;
    C::zero(acc);
    if constexpr (C::IS_DMA) {
        const auto la = C::template make_lanes<C::A_I>(rows);
        const auto lb = C::template make_lanes<C::B_I>(ncols);
        auto issue = [=](int it, char *stage) __attribute__((always_inline)) {
            C::issue(stage, xa, ldx, la, ae, ldx, lb, (uint32_t)block_of(it) * (C::BK * 2));
        };
        dma_pipelined_blocks<C>(smem, nkb, issue, acc, [](int) {});
    } else {
        const auto vx = C::template make_view<C::A_CH>(xa, ldx, rows);
        const auto va = C::template make_view<C::B_CH>(ae, ldx, shrink ? ncols : rows);
        auto issue = [=](int it, typename C::Stage &g) __attribute__((always_inline)) {
            C::load_stage(g, vx, va, (uint32_t)block_of(it) * (C::BK * 2), ldx);
        };
        if constexpr (C::PF > 1) {
            static_assert(!QUANT || C::BK == 64, "a block of 32 values in four neighbouring lanes, two per row");
            const int qrow = threadIdx.x / C::KCH, kc = threadIdx.x % C::KCH;
            pipelined_blocks_deep<C, C::PF>(smem, nkb, issue, acc, [&](int it, const typename C::Stage &g)
                                                                       __attribute__((always_inline)) {
                if constexpr (QUANT) {
                    if (!quant) return;
#pragma unroll
                    for (int i = 0; i < C::A_CH; ++i) {
                        int E;
                        const uint2 codes = mx_quantize8(g.a[i], E);
                        // the two scale bytes of a row's 64 values, into the row's first thread
                        const uint32_t pair = (uint32_t)E | ((uint32_t)__shfl_down(E, 4) << 8);
                        const int row = qrow + i * C::RPP;
                        if (row < rows) {
                            const int k0 = block_of(it) * 64;
                            *reinterpret_cast<uint2 *>(p.xq + (int64_t)(row0 + row) * p.d_in + k0 + kc * 8) = codes;
                            if (kc == 0)
                                *reinterpret_cast<uint16_t *>(p.xs + ((int64_t)(k0 >> 7) * p.T + row0 + row) * 4 +
                                                              ((k0 >> 5) & 3)) = (uint16_t)pair;
                        }
                    }
                }
            });
        } else {
            pipelined_blocks<C>(smem, nkb, issue, acc);
        }
    }
    if (!shrink) return;

    const int64_t ldu = (int64_t)p.r * 2;
    char *uh = u_hi + (int64_t)row0 * ldu;
    char *ul = u_lo + (int64_t)row0 * ldu;
    const float s = p.scale;
    const int act = p.act;
    C::epilogue(smem, acc, [&](int row, int col, float(&v)[8]) {
        if (row >= rows || col >= ncols_out) return;
        uint32_t h[8], l[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const float f = (n0 + col + q < re) ? adapter_act(v[q], act) * s : 0.f;
            h[q] = f32_to_bf16_bits(f);
            l[q] = f32_to_bf16_bits(f - bf16_bits_to_f32(h[q]));
        }
        uint4 oh, ol;
        oh.x = h[0] | (h[1] << 16); oh.y = h[2] | (h[3] << 16);
        oh.z = h[4] | (h[5] << 16); oh.w = h[6] | (h[7] << 16);
        ol.x = l[0] | (l[1] << 16); ol.y = l[2] | (l[3] << 16);
        ol.z = l[4] | (l[5] << 16); ol.w = l[6] | (l[7] << 16);
        const int64_t off = (int64_t)row * ldu + (int64_t)(n0 + col) * 2;
        *reinterpret_cast<uint4 *>(uh + off) = oh;
        *reinterpret_cast<uint4 *>(ul + off) = ol;
    });
}

// Tile shapes.  The *Dma variants need the contraction length to be a multiple
// of BK = 64; the register-staged ones take any multiple of 8.  CfgMain is the
// prefill fallback for shapes the streaming kernel (linear_stream.hip) does not
// take.
using CfgMain = GemmCore<256, 256, 64, 4, 2>;        // 8 waves, wave patch 64 x 128
using CfgShrink = GemmCore<64, 64, 64, 2, 2>;        // 4 waves, wave patch 32 x 32
using CfgShrinkDma = DmaCore<64, 64, 64, 2, 2, 4>;
// ranks from 65 to 128: the whole rank in one tile, so x streams from HBM once
using CfgShrinkR128 = DmaCore<128, 128, 64, 2, 4, 2>;   // (two stages of 64 steps: 5632-deep rows 15 % faster than four of 32)
// the quantising variant: register-staged (the quantiser works on the registers on
// their way to LDS), the loads of four blocks in flight per thread
template <int BM, int BN, int BK, int WM, int WN, int PF_>
struct DeepCore : GemmCore<BM, BN, BK, WM, WN> {
    static constexpr int PF = PF_;
};
using CfgShrinkDeep = DeepCore<128, 128, 64, 2, 4, 4>;   // ranks 65..128
using CfgShrinkDeep64 = DeepCore<128, 64, 64, 4, 2, 4>;  // ranks up to 64, and above 128 in column tiles

template <class K>
static hipError_t allow_lds(K kern, int bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

hipError_t prepare_stream_kernel();
bool stream_kernel_fits(const LinearArgs &a);
hipError_t launch_linear_stream(const PlanView &pv, const LinearArgs &a, int n_cus, hipStream_t stream);
hipError_t launch_linear_stream_shared(const PlanView &pv, const LinearArgs *a, int n, int n_cus, hipStream_t stream);

hipError_t prepare_linear_kernels()
{
    hipError_t e;
    if ((e = prepare_stream_kernel()) != hipSuccess) return e;
    if ((e = allow_lds(&linear_kernel<CfgMain>, CfgMain::SMEM_BYTES)) != hipSuccess) return e;
    if ((e = allow_lds(&linear_kernel<CfgThin>, CfgThin::SMEM_BYTES)) != hipSuccess) return e;
    if ((e = allow_lds(&linear_kernel<CfgDecodeBase>, CfgDecodeBase::SMEM_BYTES)) != hipSuccess) return e;
    if ((e = allow_lds(&shrink_kernel<CfgShrink>, CfgShrink::SMEM_BYTES)) != hipSuccess) return e;
    if ((e = allow_lds(&shrink_kernel<CfgShrinkR128>, CfgShrinkR128::SMEM_BYTES)) != hipSuccess) return e;
    if ((e = allow_lds(&shrink_kernel<CfgShrinkDma>, CfgShrinkDma::SMEM_BYTES)) != hipSuccess) return e;
    if ((e = allow_lds(&shrink_kernel<CfgShrinkDeep, true>, CfgShrinkDeep::SMEM_BYTES)) != hipSuccess) return e;
    return allow_lds(&shrink_kernel<CfgShrinkDeep64, true>, CfgShrinkDeep64::SMEM_BYTES);
}

static inline int round_up8(int v) { return (v + 7) & ~7; }

// Compute units of the current device (queried once per device).
int compute_units()
{
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

// xq / xs: the quantising variant's outputs
struct SharedX {
    int n;
    const void *const *A_stack;
    void *const *u_hi, *const *u_lo;
};

template <class C, bool QUANT = false>
static hipError_t launch_shrink_as(const PlanView &pv, const LinearArgs &a, hipStream_t stream, void *xq = nullptr,
                                   void *xs = nullptr, const SharedX *shared = nullptr)
{
    ShrinkKParams p;
    p.xq = (char *)xq; p.xs = (char *)xs; p.T = pv.T;
    p.x = (const char *)a.x; p.A_stack = (const char *)a.A_stack;
    p.u_hi = (char *)a.u_hi; p.u_lo = (char *)a.u_lo;
    p.tile_row0 = pv.tile_row0; p.tile_rows = pv.tile_rows; p.tile_expert = pv.tile_expert;
    p.tile_rank = pv.tile_rank;
    p.n_tiles = pv.n_tiles;
    p.d_in = a.d_in; p.r = a.r; p.scale = a.scale; p.act = a.act;
    p.tiles_per_proj = (a.r + C::BN - 1) / C::BN;
    p.n_proj = shared ? shared->n : 1;
    for (int i = 1; i < MAX_SHARED_X; ++i) {
        const bool on = shared && i < shared->n;
        p.A_more[i - 1] = on ? (const char *)shared->A_stack[i] : nullptr;
        p.uh_more[i - 1] = on ? (char *)shared->u_hi[i] : nullptr;
        p.ul_more[i - 1] = on ? (char *)shared->u_lo[i] : nullptr;
    }
    if (shared) {
        p.A_stack = (const char *)shared->A_stack[0];
        p.u_hi = (char *)shared->u_hi[0];
        p.u_lo = (char *)shared->u_lo[0];
    }
    p.n_tiles_n = p.tiles_per_proj * p.n_proj;
    const int64_t grid = (int64_t)pv.max_tiles * (TILE_M / C::BM) * p.n_tiles_n;
    if (grid > 0x7ffffff0LL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((shrink_kernel<C, QUANT>), dim3((unsigned)round_up8((int)grid)), dim3(C::NT),
                       C::SMEM_BYTES, stream, p);
    return hipGetLastError();
}

// The prefill shrink and the MXFP8 quantisation of x in one pass over x (r >= 1,
// d_in a multiple of 128).
hipError_t launch_prefill_shrink_quant(const PlanView &pv, const LinearArgs &a, void *xq, void *xs,
                                       hipStream_t stream)
{
    if (pv.max_tiles <= 0) return hipSuccess;
    if (a.r <= 0 || a.d_in % 128) return hipErrorInvalidValue;
    if (a.r > 64 && a.r <= 128) return launch_shrink_as<CfgShrinkDeep, true>(pv, a, stream, xq, xs);
    return launch_shrink_as<CfgShrinkDeep64, true>(pv, a, stream, xq, xs);
}

static hipError_t launch_prefill_shrink_any(const PlanView &pv, const LinearArgs &a, const SharedX *shared,
                                            hipStream_t stream)
{
    if (a.r <= 0 || pv.max_tiles <= 0) return hipSuccess;
    if (a.d_in % 64 == 0 && a.r > 64 && a.r <= 128)
        return launch_shrink_as<CfgShrinkR128>(pv, a, stream, nullptr, nullptr, shared);
    if (a.d_in % 64 == 0) return launch_shrink_as<CfgShrinkDma>(pv, a, stream, nullptr, nullptr, shared);
    return launch_shrink_as<CfgShrink>(pv, a, stream, nullptr, nullptr, shared);
}

hipError_t launch_prefill_shrink(const PlanView &pv, const LinearArgs &a, hipStream_t stream)
{
    return launch_prefill_shrink_any(pv, a, nullptr, stream);
}

hipError_t launch_prefill_shrink_shared(const PlanView &pv, const LinearArgs &a, int n, const void *const *A_stack,
                                        void *const *u_hi, void *const *u_lo, hipStream_t stream)
{
    if (n < 1 || n > MAX_SHARED_X) return hipErrorInvalidValue;
    const SharedX sh{n, A_stack, u_hi, u_lo};
    return launch_prefill_shrink_any(pv, a, &sh, stream);
}

template <class C>
static hipError_t launch_linear_as(const LinearKParams &p0, int64_t m_tiles, hipStream_t stream)
{
    LinearKParams p = p0;
    p.n_tiles_n = (p.d_out + C::BN - 1) / C::BN;
    const int64_t total = m_tiles * p.n_tiles_n;
    if (total > 0x7ffffff0LL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(linear_kernel<C>, dim3((unsigned)round_up8((int)total)), dim3(C::NT),
                       C::SMEM_BYTES, stream, p);
    return hipGetLastError();
}

hipError_t launch_prefill_linear_shared(const PlanView &pv, const LinearArgs *a, int n, hipStream_t stream)
{
    if (pv.max_tiles <= 0) return hipSuccess;
    return launch_linear_stream_shared(pv, a, n, compute_units(), stream);
}

hipError_t launch_prefill_linear(const PlanView &pv, const LinearArgs &a, hipStream_t stream)
{
    if (pv.max_tiles <= 0) return hipSuccess;
    if (stream_kernel_fits(a)) return launch_linear_stream(pv, a, compute_units(), stream);
    LinearKParams p;
    p.x = (const char *)a.x; p.W = (const char *)a.W; p.B_stack = (const char *)a.B_stack;
    p.u_hi = (const char *)a.u_hi; p.u_lo = (const char *)a.u_lo;
    p.y = (char *)a.y;
    p.tile_row0 = pv.tile_row0; p.tile_rows = pv.tile_rows; p.tile_expert = pv.tile_expert;
    p.tile_rank = pv.tile_rank;
    p.n_tiles = pv.n_tiles;
    p.T = pv.T;
    p.d_in = a.d_in; p.d_out = a.d_out; p.r = a.r;
    p.n_tiles_n = 0;
    p.y_f32 = a.y_f32;
    p.plain_tiles = 0;
    p.gather = nullptr;
    p.k_splits = 1; p.kb_per_split = 0;
    return launch_linear_as<CfgMain>(p, pv.max_tiles, stream);
}

// The decode base GEMM has few output tiles (T <= 1024 rows); cutting the
// contraction range gives the chip enough workgroups to keep many loads in
// flight.  The parts are summed, in order, by the expand kernel.
constexpr int DECODE_BASE_TARGET_WGS = 512;
constexpr int DECODE_BASE_MAX_SPLITS = 4;   // the expand kernel sums up to four parts
constexpr int DECODE_BASE_MIN_BLOCKS = 4;   // BK blocks per part at least
constexpr int DECODE_BASE_SPLIT_BLOCKS = 32;

template <class C>
static void shape_for(int64_t T, int d_in, int d_out, bool may_split, DecodeBaseShape *sh)
{
    sh->m_tiles = (T + C::BM - 1) / C::BM;
    sh->n_tiles_n = (d_out + C::BN - 1) / C::BN;
    const int64_t tiles = sh->m_tiles * sh->n_tiles_n;
    const int nkb = (d_in + C::BK - 1) / C::BK;
    int want = may_split ? (int)((DECODE_BASE_TARGET_WGS + tiles - 1) / (tiles > 0 ? tiles : 1)) : 1;
    if (want > DECODE_BASE_MAX_SPLITS) want = DECODE_BASE_MAX_SPLITS;
    // every part costs a plane of fp32 partial sums written and read back: no more
    // parts than it takes to keep a tile's serial loop to about DECODE_BASE_SPLIT_BLOCKS blocks
    const int by_len = (nkb + DECODE_BASE_SPLIT_BLOCKS - 1) / DECODE_BASE_SPLIT_BLOCKS;
    if (want > by_len) want = by_len;
    if (want > nkb / DECODE_BASE_MIN_BLOCKS) want = nkb / DECODE_BASE_MIN_BLOCKS;
    if (want < 1) want = 1;
    const int per = (nkb + want - 1) / want;
    sh->kb_per_split = per;
    sh->k_splits = (nkb + per - 1) / per;   // no empty part
    sh->grid = round_up8((int)(tiles * sh->k_splits));
}

static DecodeBaseShape base_shape(int64_t T, int d_in, int d_out, bool may_split)
{
    DecodeBaseShape sh;
    sh.dma = (d_in % 64 == 0);
    if (sh.dma) shape_for<CfgDecodeBase>(T, d_in, d_out, may_split, &sh);
    else shape_for<CfgThin>(T, d_in, d_out, may_split, &sh);
    return sh;
}

DecodeBaseShape decode_base_shape(int64_t T, int d_in, int d_out) { return base_shape(T, d_in, d_out, true); }

int decode_base_splits(int64_t T, int d_in, int d_out) { return decode_base_shape(T, d_in, d_out).k_splits; }

LinearKParams decode_base_params(const PlanView &pv, const LinearArgs &a, void *out, int out_f32,
                                 const DecodeBaseShape &sh, const int *gather)
{
    LinearKParams p;
    p.x = (const char *)a.x; p.W = (const char *)a.W; p.B_stack = nullptr;
    p.u_hi = nullptr; p.u_lo = nullptr;
    p.y = (char *)out;
    p.tile_row0 = nullptr; p.tile_rows = nullptr; p.tile_expert = nullptr; p.tile_rank = nullptr;
    p.n_tiles = nullptr;
    p.T = pv.T;
    p.d_in = a.d_in; p.d_out = a.d_out; p.r = 0;
    p.n_tiles_n = sh.n_tiles_n;
    p.y_f32 = out_f32;
    p.plain_tiles = 1;
    p.gather = gather;
    p.k_splits = sh.k_splits; p.kb_per_split = sh.kb_per_split;
    return p;
}

static hipError_t launch_plain(const PlanView &pv, const LinearArgs &a, void *out, int out_f32,
                               const DecodeBaseShape &sh, const int *gather, hipStream_t stream)
{
    if (pv.T <= 0) return hipSuccess;
    const LinearKParams p = decode_base_params(pv, a, out, out_f32, sh, gather);
    if (sh.dma)
        hipLaunchKernelGGL(linear_kernel<CfgDecodeBase>, dim3((unsigned)sh.grid), dim3(CfgDecodeBase::NT),
                           CfgDecodeBase::SMEM_BYTES, stream, p);
    else
        hipLaunchKernelGGL(linear_kernel<CfgThin>, dim3((unsigned)sh.grid), dim3(CfgThin::NT),
                           CfgThin::SMEM_BYTES, stream, p);
    return hipGetLastError();
}

hipError_t launch_decode_base(const PlanView &pv, const DecodeArgs &d, hipStream_t stream)
{
    const DecodeBaseShape sh = decode_base_shape(pv.T, d.lin.d_in, d.lin.d_out);
    if (sh.k_splits != d.k_splits) return hipErrorInvalidValue;
    return launch_plain(pv, d.lin, d.ybase, 1, sh, pv.tok_sorted, stream);   // partial sums in by-expert order
}

hipError_t launch_decode_base_only(const PlanView &pv, const LinearArgs &a, hipStream_t stream)
{
    return launch_plain(pv, a, a.y, a.y_f32, base_shape(pv.T, a.d_in, a.d_out, false), nullptr, stream);
}

}  // namespace moin
