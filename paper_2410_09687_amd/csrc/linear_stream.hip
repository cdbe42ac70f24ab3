// Prefill main kernel of the routed LoRA linear layer (Section 3.2:
// y = W x + W_b (W_a x), one adapter per sequence):
//   y tile = x W^T + u_hi B_e^T + u_lo B_e^T
// with the adapter term appended to the base GEMM as 2r more contraction steps.
//
// Shape of the kernel (gfx950):
//  * one persistent workgroup per compute unit walks a list of 256 x 256 output
//    tiles; the operand blocks of all its tiles form one stream, so the loads
//    of the next tile are already in flight while the current one finishes;
//  * operands reach LDS directly (global_load_lds), two stages of 64
//    contraction steps, rows XOR-swizzled in 16-byte chunks;
//  * MFMA fragments are read from LDS one k-step ahead; the per-block barrier
//    sits before the block's last k-step, whose fragments are in registers by
//    then, and the first fragments of the next block are read during that
//    k-step: no wave waits on LDS right after a barrier;
//  * W / B_e rows are the MFMA row operand and tokens the column operand, so a
//    lane ends up with four consecutive outputs of one token; the epilogue
//    regroups them through 4 KB of LDS per wave that lie outside the stages,
//    so it runs while the next tile's first blocks are landing.
// Contraction lengths (d_in, r) must be multiples of 64 and d_in >= 128.
#include <type_traits>

#include "gemm_core.h"
#include "kernels.h"
#include "stream_epilogue.h"

namespace moin {

namespace stream {

constexpr int BT = 256;              // tile edge, both ways
constexpr int BK = 64;
constexpr int NW = 8, NT = NW * 64;
constexpr int WQ = 2;                // waves along tokens (Q); NW / WQ along outputs (P)
constexpr int FP = 2, FQ = 4;        // 32 x 32 accumulators per wave: 64 outputs x 128 tokens
constexpr int ROWB = BK * 2;         // LDS row pitch
constexpr int OP_BYTES = BT * ROWB;  // one operand tile: 32 KB
constexpr int STAGE_BYTES = 2 * OP_BYTES;
constexpr int SMEM_STAGES = 2 * STAGE_BYTES;
constexpr int SCR_BYTES = 4096;      // per-wave epilogue scratch
constexpr int SMEM_BYTES = SMEM_STAGES + NW * SCR_BYTES;   // 160 KB: all of a compute unit's LDS
constexpr int LOADS = 4;             // DMA instructions per wave per operand per block
constexpr int KSTEPS = BK / 16;

struct Params {
    const char *x, *W, *B_stack, *u_hi, *u_lo;
    char *y;
    const int *tile_row0, *tile_rows, *tile_expert, *tile_rank, *n_tiles;
    int d_in, d_out, r;
    int n_tiles_n;
    int y_f32;
};

// Everything a tile needs, all wave-uniform.
struct Tile {
    const char *q0, *p0;       // x rows / W rows of the tile at k = 0
    const char *uh, *ul, *be;  // adapter operands (aliases of q0 / p0 without adapter)
    int q_rows, p_rows;        // valid tokens / outputs (1..256)
    int nkb1;                  // adapter blocks per half (0: no adapter)
    int total;                 // blocks of the tile: nkb0 + 2 * nkb1
    int row0, n0;
    int valid;
};

__device__ __forceinline__ Tile load_tile(const Params &p, int id, int n_work)
{
    Tile t;
    t.valid = id < n_work;
    const int cid = t.valid ? id : 0;
    const int tm = cid / p.n_tiles_n, tn = cid - tm * p.n_tiles_n;
    const int e = uniform(p.tile_expert[tm]);
    t.row0 = uniform(p.tile_row0[tm]);
    t.q_rows = uniform(p.tile_rows[tm]);
    t.n0 = tn * BT;
    t.p_rows = min(BT, p.d_out - t.n0);
    const int64_t ldx = (int64_t)p.d_in * 2, ldu = (int64_t)p.r * 2;
    t.q0 = p.x + (int64_t)t.row0 * ldx;
    t.p0 = p.W + (int64_t)t.n0 * ldx;
    // adapter blocks up to the expert's own rank (the shrink wrote zeros from there to the block end)
    const int re = min(p.r, uniform(p.tile_rank[tm]));
    const bool lora = e >= 0 && re > 0;
    t.nkb1 = lora ? (re + BK - 1) / BK : 0;
    t.total = p.d_in / BK + 2 * t.nkb1;
    t.uh = lora ? p.u_hi + (int64_t)t.row0 * ldu : t.q0;
    t.ul = lora ? p.u_lo + (int64_t)t.row0 * ldu : t.q0;
    t.be = lora ? p.B_stack + ((int64_t)e * p.d_out + t.n0) * ldu : t.p0;
    return t;
}

}  // namespace stream

__global__ __launch_bounds__(stream::NT) void linear_stream_kernel(stream::Params p)
{
    using namespace stream;
    extern __shared__ __align__(16) char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = uniform(threadIdx.x >> 6);
    const int wp = wave / WQ, wq = wave % WQ;
    const int r = lane & 31, h = lane >> 5;

    // work list of this workgroup: the 8 XCDs take workgroups round-robin, each
    // XCD owns one contiguous band of tile ids, and its workgroups stride
    // through the band together (neighbouring ids share W or x panels in L2)
    const int n_work = uniform(*p.n_tiles) * p.n_tiles_n;
    const int per = (n_work + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, nslot = gridDim.x >> 3;
    const int band_end = min((xcd + 1) * per, n_work);
    int id = xcd * per + slot;
    if (id >= band_end) return;

    const int nkb0 = p.d_in / BK;
    const uint32_t ldx = (uint32_t)p.d_in * 2u, ldu = (uint32_t)p.r * 2u;

    // DMA mapping: instruction j of a wave fills LDS rows (wave*4 + j)*8 .. +8 of
    // an operand tile; the lane fetches logical 16-byte chunk (lane%8) ^ swz(row)
    const uint32_t dma_row = (uint32_t)(wave * (LOADS * 8) + (lane >> 3));   // + 8 * j
    uint32_t dma_c16[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) dma_c16[j] = (uint32_t)(((lane & 7) ^ (((j * 8 + (lane >> 3)) >> 1) & 7)) * 16);
    // swz(row) = (row >> 1) & 7 with row = wave*32 + j*8 + lane/8: only j's parity matters

    // Starts the loads of block b of tile t into `stage`.
    auto issue = [&](const Tile &t, int b, char *stage) __attribute__((always_inline)) {
        const bool base = b < nkb0;
        const int jb = b - nkb0;
        const bool hi = jb < t.nkb1;
        const char *pq = base ? t.q0 : (hi ? t.uh : t.ul);
        const char *pp = base ? t.p0 : t.be;
        const uint32_t ld = base ? ldx : ldu;
        const int kb = base ? b : (hi ? jb : jb - t.nkb1);
        const uint32_t kbyte = (uint32_t)kb * (BK * 2);
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const uint32_t row = min(dma_row + 8u * j, (uint32_t)(t.p_rows - 1));
            const uint32_t off = __umul24(row, ld) + dma_c16[j & 1] + kbyte;
            __builtin_amdgcn_global_load_lds(MOIN_GPTR(pp + off), MOIN_LPTR(stage + (wave * LOADS + j) * 1024),
                                             16, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const uint32_t row = min(dma_row + 8u * j, (uint32_t)(t.q_rows - 1));
            const uint32_t off = __umul24(row, ld) + dma_c16[j & 1] + kbyte;
            __builtin_amdgcn_global_load_lds(MOIN_GPTR(pq + off),
                                             MOIN_LPTR(stage + OP_BYTES + (wave * LOADS + j) * 1024), 16, 0, 0);
        }
    };

    // fragment addresses: patch bases are multiples of 32 rows, so the swizzle
    // depends on r only
    const int f = (r >> 1) & 7;
    const int offP = (wp * (FP * 32) + r) * ROWB;
    const int offQ = OP_BYTES + (wq * (FQ * 32) + r) * ROWB;
    bf16x8_t fp[2][FP], fq[2][FQ];
    auto read_frags = [&](const char *stage, int ks, int slot_) __attribute__((always_inline)) {
        const int o = (((ks * 2 + h) ^ f) & 7) * 16;
#pragma unroll
        for (int i = 0; i < FP; ++i)
            fp[slot_][i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(stage + offP + i * 32 * ROWB + o));
#pragma unroll
        for (int j = 0; j < FQ; ++j)
            fq[slot_][j] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(stage + offQ + j * 32 * ROWB + o));
    };
    f32x16_t acc[FP][FQ];
    auto mfmas = [&](int slot_) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < FP; ++i)
#pragma unroll
            for (int j = 0; j < FQ; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fp[slot_][i], fq[slot_][j], acc[i][j], 0, 0, 0);
    };

    Tile cur = load_tile(p, id, band_end);
    id += nslot;
    Tile nxt = load_tile(p, id, band_end);

    // fetch cursor: tile and block index of the next block to request
    Tile pft = cur;
    int pfb = 2;

    // One block of the stream.  ISSUE: a block two positions ahead exists and is
    // fetched into the stage this block frees; READ: a next block exists.
    auto body = [&](int s, auto issue_tag, auto read_tag) __attribute__((always_inline)) {
        constexpr bool ISSUE = decltype(issue_tag)::value, READ = decltype(read_tag)::value;
        char *st_cur = smem + (s & 1) * STAGE_BYTES;
        const char *st_nxt = smem + ((s + 1) & 1) * STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < KSTEPS - 1; ++ks) {
            read_frags(st_cur, ks + 1, (ks + 1) & 1);
            mfmas(ks & 1);
            // one MFMA, one LDS read, ...: the next k-step's fragments trickle in
            // under this k-step's MFMAs
#pragma unroll
            for (int n = 0; n < FP + FQ; ++n) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, FP * FQ - (FP + FQ), 0);
        }
        // own share of block s+1 has landed and every fragment of block s is in
        // registers; past the barrier that holds for all waves
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if constexpr (ISSUE) {
            // the fetch cursor runs two blocks ahead; when it has used up its tile
            // it moves to the tile after the one being computed (checked here, not
            // when the cursor advances: by now `nxt` is that tile in every case)
            if (pfb == pft.total) {
                pft = nxt;
                pfb = 0;
            }
            issue(pft, pfb, st_cur);
            ++pfb;
        }
        if constexpr (READ) read_frags(st_nxt, 0, 0);
        mfmas((KSTEPS - 1) & 1);
        if constexpr (ISSUE && READ) {
#pragma unroll
            for (int n = 0; n < FP * FQ; ++n) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                if (n < FP + FQ) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        } else if constexpr (READ) {
#pragma unroll
            for (int n = 0; n < FP + FQ; ++n) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
    };

    // prologue of the stream: two blocks in flight, the first one's leading fragments read
    issue(cur, 0, smem);
    issue(cur, 1, smem + STAGE_BYTES);   // every tile has at least two blocks
    wait_vm_then_barrier<2 * LOADS>();
    read_frags(smem, 0, 0);

    int s = 0;
    for (;;) {
#pragma unroll
        for (int i = 0; i < FP; ++i)
#pragma unroll
            for (int j = 0; j < FQ; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

        const int total = cur.total;
        if (nxt.valid) {
            for (int b = 0; b < total; ++b, ++s) body(s, std::true_type{}, std::true_type{});
        } else {
            int b = 0;
            for (; b < total - 2; ++b, ++s) body(s, std::true_type{}, std::true_type{});
            body(s, std::false_type{}, std::true_type{});
            ++s;
            body(s, std::false_type{}, std::false_type{});
            ++s;
        }

        // epilogue through the wave's private 4 KB of LDS beyond the two stages
        // (which the next tile's loads are already filling)
        // (the lane id goes in through an opaque copy: the epilogue's per-lane
        // addresses are then recomputed per tile instead of being kept, and
        // spilled, across the main loop; a reload between two stores would wait
        // for the first store to complete)
        int lane_e = lane;
        asm volatile("; lane id, rematerialised" : "+v"(lane_e));
        stream_epilogue<FP, FQ>(smem + SMEM_STAGES + wave * SCR_BYTES, acc, p.y, p.y_f32, p.d_out, cur.row0,
                                cur.n0, cur.q_rows, cur.p_rows, wp, wq, lane_e);
        if (!nxt.valid) break;
        cur = nxt;
        id += nslot;
        nxt = load_tile(p, id, band_end);
    }
}

hipError_t prepare_stream_kernel()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&linear_stream_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, stream::SMEM_BYTES);
}

bool stream_kernel_fits(const LinearArgs &a)
{
    return a.d_in % 64 == 0 && a.r % 64 == 0 && a.d_in >= 128;
}

hipError_t launch_linear_stream(const PlanView &pv, const LinearArgs &a, int n_cus, hipStream_t stream_)
{
    stream::Params p;
    p.x = (const char *)a.x; p.W = (const char *)a.W; p.B_stack = (const char *)a.B_stack;
    p.u_hi = (const char *)a.u_hi; p.u_lo = (const char *)a.u_lo;
    p.y = (char *)a.y;
    p.tile_row0 = pv.tile_row0; p.tile_rows = pv.tile_rows; p.tile_expert = pv.tile_expert;
    p.tile_rank = pv.tile_rank;
    p.n_tiles = pv.n_tiles;
    p.d_in = a.d_in; p.d_out = a.d_out; p.r = a.r;
    p.n_tiles_n = (a.d_out + stream::BT - 1) / stream::BT;
    p.y_f32 = a.y_f32;
    // one workgroup per compute unit (the LDS footprint allows no more), fewer
    // when the batch has fewer tiles than that; always a multiple of 8
    const int64_t max_work = (int64_t)pv.max_tiles * p.n_tiles_n;
    int64_t grid = n_cus > 0 ? n_cus : 256;
    if (grid > max_work) grid = max_work;
    grid = (grid + 7) / 8 * 8;
    hipLaunchKernelGGL(linear_stream_kernel, dim3((unsigned)grid), dim3(stream::NT), stream::SMEM_BYTES,
                       stream_, p);
    return hipGetLastError();
}

}  // namespace moin
