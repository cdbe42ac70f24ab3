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
//  * four waves, one per SIMD: 128 x 128 patches of v_mfma_f32_16x16x32_bf16
//    accumulators; the fragments of a k-step are read from LDS under the
//    MFMAs of the k-step before, the block's barrier sits between its two
//    k-steps, and the requests for the block two ahead go out under the second;
//  * W / B_e rows are the MFMA row operand and tokens the column operand, so a
//    lane ends up with four consecutive outputs of one token; the epilogue
//    regroups them through 8 KB of LDS per wave that lie outside the stages,
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
constexpr int ROWB = BK * 2;         // LDS row pitch
constexpr int OP_BYTES = BT * ROWB;  // one operand tile: 32 KB
constexpr int STAGE_BYTES = 2 * OP_BYTES;
constexpr int SMEM_STAGES = 2 * STAGE_BYTES;

// Up to MAX_SHARED_X projections that read the same x (q, k, v; gate, up) in one launch: the column
// tiles of projection i follow those of projection i - 1, so a narrow projection's tiles (k, v: one
// column of tiles) ride in the wide one's stream and share its x panels in L2.
struct Params {
    const char *x;
    const char *W[MAX_SHARED_X], *B_stack[MAX_SHARED_X], *u_hi[MAX_SHARED_X], *u_lo[MAX_SHARED_X];
    char *y[MAX_SHARED_X];
    int d_out[MAX_SHARED_X];
    int tn_start[MAX_SHARED_X];   // first column tile of each projection (tn_start[0] = 0)
    int n_proj;
    const int *tile_row0, *tile_rows, *tile_expert, *tile_rank, *n_tiles;
    int d_in, r;
    int n_tiles_n;                // column tiles of all projections together
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
    char *y;                   // the projection's output and its width
    int d_out;
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
    // the projection of this column tile (picked by comparison, not by indexing: indexing the
    // parameter arrays would put them in scratch)
    const char *W = p.W[0], *B_stack = p.B_stack[0], *u_hi = p.u_hi[0], *u_lo = p.u_lo[0];
    int tn0 = 0;
    t.y = p.y[0];
    t.d_out = p.d_out[0];
#pragma unroll
    for (int i = 1; i < MAX_SHARED_X; ++i)
        if (i < p.n_proj && tn >= p.tn_start[i]) {
            W = p.W[i]; B_stack = p.B_stack[i]; u_hi = p.u_hi[i]; u_lo = p.u_lo[i];
            t.y = p.y[i];
            t.d_out = p.d_out[i];
            tn0 = p.tn_start[i];
        }
    t.n0 = (tn - tn0) * BT;
    t.p_rows = min(BT, t.d_out - t.n0);
    const int64_t ldx = (int64_t)p.d_in * 2, ldu = (int64_t)p.r * 2;
    t.q0 = p.x + (int64_t)t.row0 * ldx;
    t.p0 = W + (int64_t)t.n0 * ldx;
    // adapter blocks up to the expert's own rank (the shrink wrote zeros from there to the block end)
    const int re = min(p.r, uniform(p.tile_rank[tm]));
    const bool lora = e >= 0 && re > 0;
    t.nkb1 = lora ? (re + BK - 1) / BK : 0;
    t.total = p.d_in / BK + 2 * t.nkb1;
    t.uh = lora ? u_hi + (int64_t)t.row0 * ldu : t.q0;
    t.ul = lora ? u_lo + (int64_t)t.row0 * ldu : t.q0;
    t.be = lora ? B_stack + ((int64_t)e * t.d_out + t.n0) * ldu : t.p0;
    return t;
}

}  // namespace stream

// Four waves, one per SIMD, each with the full 512 registers: a 128 x 128 patch of the tile per
// wave (64 accumulators of 16 outputs x 16 tokens, v_mfma_f32_16x16x32_bf16), so a k-step of 32
// takes 8 + 8 fragment reads for 64 MFMAs.  An earlier form of this kernel ran eight waves with
// 64 x 128 patches of 32 x 32 x 16 MFMAs (2 + 4 reads per 8 MFMAs): half more LDS bytes per flop
// and twice the accumulator registers moved per flop -- both count where the limit is power -- and
// it was 8-9 % slower on N(0,1) data (241 against 213 us on the 2048 -> 2048 prefill shape), though
// a little faster on all-zero data, where a second wave per SIMD hides this kernel's barrier.
namespace s16 {
using stream::BK;
using stream::BT;
using stream::OP_BYTES;
using stream::ROWB;
using stream::SMEM_STAGES;
using stream::STAGE_BYTES;
constexpr int NW = 4, NT = NW * 64;
constexpr int FP = 8, FQ = 8;          // 16 x 16 accumulators per wave: 128 outputs x 128 tokens
constexpr int LOADS = 8;               // DMA instructions per wave per operand per block
constexpr int SCR_BYTES = 8192;        // per-wave epilogue scratch: 16 tokens x 128 outputs, fp32
constexpr int SMEM_BYTES = SMEM_STAGES + NW * SCR_BYTES;   // 160 KB
}  // namespace s16

template <bool Y_F32>
__global__ __launch_bounds__(s16::NT) void linear_stream_kernel(stream::Params p)
{
    using namespace s16;
    using stream::Tile;
    extern __shared__ __align__(16) char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = uniform(threadIdx.x >> 6);
    const int wp = wave >> 1, wq = wave & 1;

    const int n_work = uniform(*p.n_tiles) * p.n_tiles_n;
    const int per = (n_work + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, nslot = gridDim.x >> 3;
    const int band_end = min((xcd + 1) * per, n_work);
    int id = xcd * per + slot;
    if (id >= band_end) return;

    const int nkb0 = p.d_in / BK;
    const uint32_t ldx = (uint32_t)p.d_in * 2u, ldu = (uint32_t)p.r * 2u;

    // DMA: instruction j of a wave fills LDS rows (wave*8 + j)*8 .. +8 of an operand tile; the lane
    // fetches logical 16-byte chunk (lane%8) ^ swz(row), swz(row) = (row >> 1) & 7, which for
    // row = wave*64 + j*8 + lane/8 is ((j & 1) * 4 + lane/16) & 7.  A block's requests are issued
    // one by one (issue_one, n = 0..15: eight for the output rows, eight for the tokens) so that
    // they can be placed between the MFMAs.  What a request needs per lane is kept in registers
    // for the tile being fetched (its 16 source rows, clamped to the tile's last row) and for the
    // kernel (the two chunk offsets); the block's position along k goes into the uniform base
    // pointers, so a request costs one multiply-add besides itself.
    const uint32_t c16a = (((uint32_t)lane & 7) ^ ((uint32_t)lane >> 4)) * 16, c16b = c16a ^ 64u;   // even j, odd j
    uint32_t rowc[2 * LOADS];
    auto rows_of = [&](const Tile &t) __attribute__((always_inline)) {
        const uint32_t dma_row = (uint32_t)(wave * (LOADS * 8)) + ((uint32_t)lane >> 3);
#pragma unroll
        for (int n = 0; n < 2 * LOADS; ++n)
            rowc[n] = min(dma_row + 8u * (n & 7), (uint32_t)((n >= LOADS ? t.q_rows : t.p_rows) - 1));
    };
    struct Fetch {
        const char *pp, *pq;   // the operands' rows 0 at the block's first k
        uint32_t ld;
    };
    auto fetch_of = [&](const Tile &t, int b) __attribute__((always_inline)) {
        Fetch f;
        const bool base = b < nkb0;
        const int jb = b - nkb0;
        const bool hi = jb < t.nkb1;
        const int kb = base ? b : (hi ? jb : jb - t.nkb1);
        f.pq = (base ? t.q0 : (hi ? t.uh : t.ul)) + kb * (BK * 2);
        f.pp = (base ? t.p0 : t.be) + kb * (BK * 2);
        f.ld = base ? ldx : ldu;
        return f;
    };
    auto issue_one = [&](const Fetch &f, char *stage, int n) __attribute__((always_inline)) {
        const int j = n & 7;
        const bool q = n >= LOADS;
        const uint32_t off = __umul24(rowc[n], f.ld) + ((j & 1) ? c16b : c16a);
        __builtin_amdgcn_global_load_lds(MOIN_GPTR((q ? f.pq : f.pp) + off),
                                         MOIN_LPTR(stage + (q ? OP_BYTES : 0) + (wave * LOADS + j) * 1024), 16, 0, 0);
    };
    auto issue = [&](const Tile &t, int b, char *stage) __attribute__((always_inline)) {
        const Fetch f = fetch_of(t, b);
#pragma unroll
        for (int n = 0; n < 2 * LOADS; ++n) issue_one(f, stage, n);
    };

    // MFMA operand of a lane: row lane%16 of a 16-row block, elements 8 (lane/16) .. + 8 of the
    // k-step's 32, i.e. logical chunk 4 ks + lane/16 of the row; the swizzle of a row inside a
    // 16-row block depends on lane%16 only ((row >> 1) & 7 = (lane%16) >> 1), and k-step 1 is
    // k-step 0's address ^ 64.  Fragment n = 0..7: output blocks, 8..15: token blocks.
    const int lo0 = ((lane & 15) * ROWB) | ((((lane >> 4) ^ ((lane & 15) >> 1)) & 7) * 16);
    const int lo1 = lo0 ^ 64;
    const int baseP = wp * (FP * 16) * ROWB, baseQ = OP_BYTES + wq * (FQ * 16) * ROWB;
    bf16x8_t fr[2][FP + FQ];
    auto read_one = [&](const char *stage, int lo_, int set, int n) __attribute__((always_inline)) {
        const int base_ = n < FP ? baseP + n * 16 * ROWB : baseQ + (n - FP) * 16 * ROWB;
        fr[set][n] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(stage + base_ + lo_));
    };
    // The order in which a k-step's fragments are read: the first MFMAs (output block 0 against
    // token blocks 0..7) need output block 0 and all token blocks, output block i only from MFMA 8 i.
    auto frag_at = [](int k) { return k == 0 ? 0 : (k <= FQ ? FP + k - 1 : k - FQ); };
    // The MFMAs are written as assembly with the accumulator tied in and out as an AccVGPR operand:
    // the compiler's own selection for 64 four-register accumulators goes through the VGPR form and
    // wraps every MFMA in copies.  What its hazard checks cannot see is taken care of by hand: an
    // accumulator is touched again only 64 MFMAs later, its operands come from LDS reads (waited for by
    // the compiler: they are inputs of the statement), and the epilogue waits before it reads.
    f32x4_t acc[FP][FQ];
    auto mfma = [&](int set, int i, int j) __attribute__((always_inline)) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fr[set][i]), "v"(fr[set][FP + j]));
    };
    // a tile's first MFMA on an accumulator takes a constant zero as its addend: the accumulators are never
    // cleared (256 register writes per tile, and with one wave on the SIMD a vector instruction issues
    // every 5.6 cycles)
    auto mfma_first = [&](int i, int j) __attribute__((always_inline)) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, 0" : "=a"(acc[i][j]) : "v"(fr[0][i]), "v"(fr[0][FP + j]));
    };

    Tile cur = stream::load_tile(p, id, band_end);
    id += nslot;
    Tile nxt = stream::load_tile(p, id, band_end);
    Tile pft = cur;
    int pfb = 2;
    rows_of(cur);

    // One block of the stream: k-step 0 (its fragments were read during the block before) with the
    // reads of k-step 1 between its MFMAs; barrier; k-step 1 with the requests for the block two
    // ahead and the first fragments of the next block between its MFMAs.  A wave issues in order and
    // an MFMA keeps the matrix core busy for 16 cycles, 4 of them its own issue: whatever stands
    // between two MFMAs and takes longer than the other 12 delays the second one.  So the other work
    // is spread thin -- one LDS read, or one request's address, or the request itself (the longest:
    // about 20 cycles) after an MFMA, never two of them -- and the order below IS the instruction
    // order (scheduling barriers after every piece).  Measured with cycle stamps around the barrier,
    // a block of 128 MFMAs took 3050 cycles with read, address and request together after every
    // fourth MFMA, 2570 without the requests, 2480 without requests and reads.  No branch after the
    // barrier: past the stream's end the fetch repeats the last block into the free stage and the
    // reads take stale bytes that nothing uses.
    auto body = [&](int s, auto first_tag) __attribute__((always_inline)) {
        char *st_cur = smem + (s & 1) * STAGE_BYTES;
        const char *st_nxt = smem + ((s + 1) & 1) * STAGE_BYTES;
        Fetch f;
#pragma unroll
        for (int n = 0; n < FP * FQ; ++n) {
            if constexpr (decltype(first_tag)::value) mfma_first(n / FQ, n % FQ);   // the tile's first block
            else mfma(0, n / FQ, n % FQ);
            if (n % 2 == 1 && n / 2 < FP + FQ) {
                read_one(st_cur, lo1, 1, frag_at(n / 2));
                __builtin_amdgcn_sched_barrier(0);
            }
            if (n == 36) {
                // what the second half fetches, worked out here so that the matrix core has work
                // again the moment the barrier opens
                if (pfb == pft.total) {
                    if (nxt.valid) {
                        pft = nxt;
                        pfb = 0;
                        rows_of(pft);
                    } else {
                        pfb = pft.total - 1;
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (n == 40) {
                f = fetch_of(pft, pfb);
                ++pfb;
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

    issue(cur, 0, smem);
    issue(cur, 1, smem + STAGE_BYTES);   // every tile has at least two blocks
    wait_vm_then_barrier<2 * LOADS>();

    int s = 0;
    for (;;) {
        // leading fragments of the tile's first block (landed: the prologue, or the previous
        // tile's last barrier, waited for it); not held across the epilogue
        {
#pragma unroll
            for (int n = 0; n < FP + FQ; ++n) read_one(smem + (s & 1) * STAGE_BYTES, lo0, 0, n);
        }
        const int total = cur.total;   // >= 2
        body(s, std::true_type{});
        ++s;
        for (int b = 1; b < total; ++b, ++s) body(s, std::false_type{});
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // the last MFMAs' results before the epilogue reads them

        // Epilogue through the wave's private 8 KB beyond the stages (which the next tile's loads are
        // already filling).  A lane holds, per accumulator (i, j), token 16 j + lane%16 and outputs
        // 16 i + 4 (lane/16) + 0..3.  One 16-token block at a time: every lane parks its 32 outputs of
        // the block's token in the scratch row of that token (slots of four outputs, the slot index
        // XORed with twice the token so that the 16 tokens of a write hit different banks), then the
        // wave reads the block back 16 bytes per lane and stores whole 128-byte lines.  All reads of a
        // block are issued before its first store (one wait per block, not one per read), a lane's
        // store address is a 32-bit offset worked out once per tile plus a wave-uniform base, and a
        // bf16 block takes half the scratch, so blocks alternate between the halves.
        {
            int ln = lane;
            asm volatile("; lane id, rematerialised" : "+v"(ln));
            char *scr = smem + SMEM_STAGES + wave * SCR_BYTES;
            const int t16 = ln & 15, kg = ln >> 4;
            constexpr int EB = Y_F32 ? 4 : 2;           // bytes per output
            constexpr int SLOT = 4 * EB;                // four outputs
            constexpr int ROW = 128 * EB;               // a token's 128 outputs
            constexpr int CPR = ROW / 16;               // 16-byte chunks per token row (16 bf16 / 32 fp32)
            constexpr int SPC = 16 / SLOT;              // slots per chunk (2 / 1)
            constexpr int NPS = 16 * CPR / 64;          // read-back instructions per block (4 / 8)
            constexpr int TPP = 64 / CPR;               // tokens per read-back instruction (4 / 2)
            constexpr int BLOCK = 16 * ROW;             // scratch bytes of a block (4 KB / 8 KB)
            constexpr bool TWO = 2 * BLOCK <= SCR_BYTES;
            const int tl = ln / CPR, ch = ln % CPR;     // read-back: token ps * TPP + tl of the block, chunk ch
            const int n = wp * (FP * 16) + ch * (16 / EB);
            const bool n_ok = n < cur.p_rows;           // d_out % 8 == 0: a chunk is all in or all out
            const uint32_t ldy = (uint32_t)cur.d_out * EB;
            char *ybase = cur.y + (int64_t)(cur.row0 + wq * (FQ * 16)) * ldy + (int64_t)cur.n0 * EB;   // wave-uniform
            const uint32_t voff = (uint32_t)tl * ldy + (uint32_t)n * EB;
            const int m_lane = wq * (FQ * 16) + tl;
#pragma unroll
            for (int j = 0; j < FQ; ++j) {
                char *blk = scr + (TWO ? (j & 1) * BLOCK : 0);
#pragma unroll
                for (int i = 0; i < FP; ++i) {
                    const int slot_ = (i * 4 + kg) ^ (2 * t16);
                    // (read in place: left to itself the compiler may copy all 256 accumulators out first)
                    f32x4_t a;
#pragma unroll
                    for (int e = 0; e < 4; ++e) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a[e]) : "a"(acc[i][j][e]));
                    if constexpr (Y_F32)
                        *reinterpret_cast<f32x4_t *>(blk + t16 * ROW + slot_ * SLOT) = a;
                    else
                        *reinterpret_cast<uint2 *>(blk + t16 * ROW + slot_ * SLOT) =
                            make_uint2(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]));
                }
                lds_order();
                auto rd = [&](int ps) {
                    const int tt = ps * TPP + tl;
                    const int pslot = (ch * SPC) ^ (2 * tt);       // XOR with an even number keeps slot pairs adjacent
                    return *reinterpret_cast<const uint4 *>(blk + tt * ROW + pslot * SLOT);
                };
                auto st = [&](int ps, const uint4 &v) {
                    const int m = m_lane + j * 16 + ps * TPP;
                    if (n_ok && m < cur.q_rows)
                        *reinterpret_cast<uint4 *>(ybase + (uint32_t)(j * 16 + ps * TPP) * ldy + voff) = v;
                };
                static_assert(NPS == 4 || NPS == 8, "read-back steps per block");
                const uint4 v0 = rd(0), v1 = rd(1), v2 = rd(2), v3 = rd(3);
                if constexpr (NPS == 8) {
                    const uint4 v4 = rd(4), v5 = rd(5), v6 = rd(6), v7 = rd(7);
                    st(0, v0), st(1, v1), st(2, v2), st(3, v3);
                    st(4, v4), st(5, v5), st(6, v6), st(7, v7);
                } else {
                    st(0, v0), st(1, v1), st(2, v2), st(3, v3);
                }
                lds_order();
            }
        }
        if (!nxt.valid) break;
        cur = nxt;
        id += nslot;
        nxt = stream::load_tile(p, id, band_end);
    }
}

hipError_t prepare_stream_kernel()
{
    hipError_t e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(&linear_stream_kernel<false>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, s16::SMEM_BYTES)) != hipSuccess)
        return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&linear_stream_kernel<true>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, s16::SMEM_BYTES);
}

bool stream_kernel_fits(const LinearArgs &a)
{
    return a.d_in % 64 == 0 && a.r % 64 == 0 && a.d_in >= 128;
}

// n projections that share x, d_in, r and the output type (a[i]: W, B_stack, u_hi, u_lo, y, d_out of
// projection i; a[0] also x, d_in, r, y_f32)
hipError_t launch_linear_stream_shared(const PlanView &pv, const LinearArgs *a, int n, int n_cus, hipStream_t stream_)
{
    if (n < 1 || n > MAX_SHARED_X) return hipErrorInvalidValue;
    stream::Params p;
    p.x = (const char *)a[0].x;
    p.n_proj = n;
    int tn = 0;
    for (int i = 0; i < MAX_SHARED_X; ++i) {
        const LinearArgs &ai = a[i < n ? i : 0];
        p.W[i] = (const char *)ai.W; p.B_stack[i] = (const char *)ai.B_stack;
        p.u_hi[i] = (const char *)ai.u_hi; p.u_lo[i] = (const char *)ai.u_lo;
        p.y[i] = (char *)ai.y;
        p.d_out[i] = ai.d_out;
        p.tn_start[i] = tn;
        if (i < n) tn += (ai.d_out + stream::BT - 1) / stream::BT;
    }
    p.tile_row0 = pv.tile_row0; p.tile_rows = pv.tile_rows; p.tile_expert = pv.tile_expert;
    p.tile_rank = pv.tile_rank;
    p.n_tiles = pv.n_tiles;
    p.d_in = a[0].d_in; p.r = a[0].r;
    p.n_tiles_n = tn;
    p.y_f32 = a[0].y_f32;
    // one workgroup per compute unit (the LDS footprint allows no more), fewer
    // when the batch has fewer tiles than that; always a multiple of 8
    const int64_t max_work = (int64_t)pv.max_tiles * p.n_tiles_n;
    if (max_work > 0x7fffffffLL) return hipErrorInvalidValue;
    int64_t grid = n_cus > 0 ? n_cus : 256;
    if (grid > max_work) grid = max_work;
    grid = (grid + 7) / 8 * 8;
    if (p.y_f32)
        hipLaunchKernelGGL(linear_stream_kernel<true>, dim3((unsigned)grid), dim3(s16::NT), s16::SMEM_BYTES, stream_, p);
    else
        hipLaunchKernelGGL(linear_stream_kernel<false>, dim3((unsigned)grid), dim3(s16::NT), s16::SMEM_BYTES, stream_, p);
    return hipGetLastError();
}

hipError_t launch_linear_stream(const PlanView &pv, const LinearArgs &a, int n_cus, hipStream_t stream_)
{
    return launch_linear_stream_shared(pv, &a, 1, n_cus, stream_);
}

}  // namespace moin
