// Routed LoRA linear layer on a quantised base ("Future Works", quantising the
// base model: an aggressively quantised base whose loss the full-precision
// experts recover).  The base operands are in the OCP Microscaling MXFP8 format:
// blocks of 32 contraction steps share a power-of-two scale (one E8M0 byte) and
// hold FP8 E4M3 elements.
//
//   mx_quantize_kernel      bf16 -> codes + scales (the weight once, the
//                           activations per call);
//   linear_mx_stream_kernel y tile = xq Wq^T (block-scaled FP8 MFMA)
//                                    + u_hi B_e^T + u_lo B_e^T (bf16 MFMA),
//                           all into the same fp32 accumulators.
//
// The main kernel is the streaming prefill kernel with another block format: an
// operand row of a block is still 128 bytes, which now are 128 FP8 contraction
// steps of the base product, or 64 bf16 ones of the adapter term.
// v_mfma_scale_f32_32x32x64_f8f6f4 takes, per lane, 16 + 16 bytes of an operand
// row: bytes [16 h, 16 h + 16) of the first and of the second 32-step block of a
// 64-step slice (h = lane / 32), and the scale byte of the first block from the
// lanes with h = 0, of the second from those with h = 1.  Read as bf16 the same
// two 16-byte pieces are the operands of two v_mfma_f32_32x32x16_bf16, so both
// block kinds share one LDS read pattern.
#include <type_traits>

#include "gemm_core.h"
#include "kernels.h"
#include "stream_epilogue.h"

namespace moin {

typedef int i32x8_t __attribute__((ext_vector_type(8)));

// ---- quantiser -----------------------------------------------------------

// One thread per 8 consecutive values, four threads per block of 32.  All the
// arithmetic is exact until the final rounding: the shared scale is the power
// of two 2^(floor(log2 amax) - 8) (byte E = exponent field of amax - 8, at
// least 0; 127 for a block of zeros), the quotient value / scale is a product
// with a power of two, magnitudes above 448 clamp to 448, and the conversion
// rounds to nearest even.
//
// Scale bytes go out row-major ([rows, cols / 32], BLOCKED = false) or in the
// order the main kernel fetches them (BLOCKED = true, cols a multiple of 128):
// [cols / 128, rows, 4], i.e. the four bytes of a row's 128 consecutive values as
// one word, words of consecutive rows adjacent, so that 32 lanes holding 32
// consecutive rows fetch one 128-byte line.
template <bool BLOCKED>
__global__ __launch_bounds__(256) void mx_quantize_kernel(const uint4 *__restrict__ src, uint2 *__restrict__ codes,
                                                          uint8_t *__restrict__ scales, int64_t n8, int64_t rows,
                                                          int cols8)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < n8; t += stride) {
        const uint4 v = src[t];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        uint32_t m = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            m = max(m, w[i] & 0x7FFFu);
            m = max(m, (w[i] >> 16) & 0x7FFFu);
        }
        // n8 is a multiple of 4 and the stride of 64: the four lanes of a block are active together
        m = max(m, (uint32_t)__shfl_xor((int)m, 1));
        m = max(m, (uint32_t)__shfl_xor((int)m, 2));
        const int E = m == 0 ? 127 : max(0, (int)(m >> 7) - 8);
        const float inv = bits_f32((uint32_t)(254 - E) << 23);   // 2^(127 - E), a normal number for E <= 246
        float f[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = bits_f32(w[i] << 16) * inv;
            f[2 * i + 1] = bits_f32(w[i] & 0xFFFF0000u) * inv;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = fminf(fmaxf(f[i], -448.f), 448.f);
        int lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], 0, false);
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
        int hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], 0, false);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
        codes[t] = make_uint2((uint32_t)lo, (uint32_t)hi);
        if constexpr (BLOCKED) {
            // n8 is a multiple of 16 here: the 16 lanes of a row's 128 values are active together
            uint32_t word = (uint32_t)E;
            word |= (uint32_t)__shfl_down(E, 4) << 8;
            word |= (uint32_t)__shfl_down(E, 8) << 16;
            word |= (uint32_t)__shfl_down(E, 12) << 24;
            if ((t & 15) == 0) {
                const int64_t row = t / cols8, kb = (t - row * cols8) >> 4;
                reinterpret_cast<uint32_t *>(scales)[kb * rows + row] = word;
            }
        } else {
            if ((t & 3) == 0) scales[t >> 2] = (uint8_t)E;
        }
    }
}

hipError_t launch_mx_quantize(const void *src, int64_t rows, int64_t cols, void *codes, void *scales,
                              int blocked, hipStream_t stream)
{
    const int64_t n8 = rows * cols / 8;
    if (n8 <= 0) return hipSuccess;
    if (blocked && cols % 128) return hipErrorInvalidValue;
    int64_t grid = (n8 + 255) / 256;
    if (grid > 256 * 32) grid = 256 * 32;
    if (blocked)
        hipLaunchKernelGGL(mx_quantize_kernel<true>, dim3((unsigned)grid), dim3(256), 0, stream,
                           reinterpret_cast<const uint4 *>(src), reinterpret_cast<uint2 *>(codes),
                           reinterpret_cast<uint8_t *>(scales), n8, rows, (int)(cols / 8));
    else
        hipLaunchKernelGGL(mx_quantize_kernel<false>, dim3((unsigned)grid), dim3(256), 0, stream,
                           reinterpret_cast<const uint4 *>(src), reinterpret_cast<uint2 *>(codes),
                           reinterpret_cast<uint8_t *>(scales), n8, rows, (int)(cols / 8));
    return hipGetLastError();
}

// ---- main kernel -----------------------------------------------------------

namespace mxs {

constexpr int BT = 256;              // tile edge, both ways
constexpr int ROWB = 128;            // bytes of one operand row per block
constexpr int KB16 = 64;             // contraction steps of an adapter block (bf16)
constexpr int NW = 4, NT = NW * 64;  // one wave per SIMD: 512 registers each
constexpr int WQ = 2;                // waves along tokens (Q); NW / WQ along outputs (P)
constexpr int FP = 4, FQ = 4;        // 32 x 32 accumulators per wave: 128 outputs x 128 tokens
constexpr int OP_BYTES = BT * ROWB;  // one operand tile: 32 KB
constexpr int STAGE_BYTES = 2 * OP_BYTES;
constexpr int SMEM_STAGES = 2 * STAGE_BYTES;
constexpr int SC_BYTES = 2 * BT * 4; // scale words of a block: 256 output rows, then 256 tokens
constexpr int SMEM_SCALES = 2 * SC_BYTES;
constexpr int SCR_BYTES = 4096;      // per-wave epilogue scratch
constexpr int SMEM_BYTES = SMEM_STAGES + SMEM_SCALES + NW * SCR_BYTES;   // 148 KB
constexpr int LOADS = 8;             // DMA instructions per wave per operand per block
constexpr int NSC = FP + FQ;         // scale words a lane needs per block

struct Params {
    const char *xq, *Wq;             // FP8 codes [T, d_in], [d_out, d_in]
    const char *xs, *Ws;             // scale words [d_in / 128, T], [d_in / 128, d_out] (four bytes each)
    int64_t T;
    const char *B_stack, *u_hi, *u_lo;
    char *y;
    const int *tile_row0, *tile_rows, *tile_expert, *tile_rank, *n_tiles;
    int d_in, d_out, r;
    int n_tiles_n;
    int y_f32;
    // plain mode (decode-sized batches: the base product alone, for all tokens, no
    // plan): tiles_m row tiles of 256 tokens, the contraction range cut into k_splits
    // parts of kb_per_split blocks, part s written to y + s * plane_bytes
    int plain, tiles_m, k_splits, kb_per_split;
    int64_t plane_bytes;
};

// Everything a tile needs, all wave-uniform.
struct Tile {
    const char *q0, *p0;       // code rows of the tile's tokens / outputs at k = 0
    const char *uh, *ul, *be;  // adapter operands (aliases of q0 / p0 without adapter)
    int q_rows, p_rows;        // valid tokens / outputs (1..256)
    int nkb1;                  // adapter blocks per half (0: no adapter)
    int total;                 // blocks of the tile: nkb0 + 2 * nkb1
    int row0, n0;
    int kb0;                   // first contraction block (plain mode: the part's; else 0)
    int64_t y_off;             // byte offset of the output plane (plain mode)
    int valid;
};

template <bool MX>
__device__ __forceinline__ Tile load_tile(const Params &p, int id, int n_work)
{
    constexpr int EB = MX ? 1 : 2;   // bytes per base operand element
    Tile t;
    t.valid = id < n_work;
    const int cid = t.valid ? id : 0;
    const int64_t ldq = (int64_t)p.d_in * EB, ldu = (int64_t)p.r * 2;
    if (p.plain) {
        const int per_part = p.tiles_m * p.n_tiles_n;
        const int part = cid / per_part, rem = cid - part * per_part;
        const int tm = rem / p.n_tiles_n, tn = rem - tm * p.n_tiles_n;
        t.row0 = tm * BT;
        t.q_rows = (int)min((int64_t)BT, p.T - t.row0);
        t.n0 = tn * BT;
        t.p_rows = min(BT, p.d_out - t.n0);
        t.kb0 = part * p.kb_per_split;
        t.y_off = (int64_t)part * p.plane_bytes;
        t.q0 = p.xq + (int64_t)t.row0 * ldq + (int64_t)t.kb0 * ROWB;
        t.p0 = p.Wq + (int64_t)t.n0 * ldq + (int64_t)t.kb0 * ROWB;
        t.nkb1 = 0;
        t.total = min(p.kb_per_split, p.d_in * EB / ROWB - t.kb0);
        t.uh = t.ul = t.q0;
        t.be = t.p0;
        return t;
    }
    const int tm = cid / p.n_tiles_n, tn = cid - tm * p.n_tiles_n;
    const int e = uniform(p.tile_expert[tm]);
    t.row0 = uniform(p.tile_row0[tm]);
    t.q_rows = uniform(p.tile_rows[tm]);
    t.n0 = tn * BT;
    t.p_rows = min(BT, p.d_out - t.n0);
    t.kb0 = 0;
    t.y_off = 0;
    t.q0 = p.xq + (int64_t)t.row0 * ldq;
    t.p0 = p.Wq + (int64_t)t.n0 * ldq;
    const int re = min(p.r, uniform(p.tile_rank[tm]));
    const bool lora = e >= 0 && re > 0;
    t.nkb1 = lora ? (re + KB16 - 1) / KB16 : 0;
    t.total = p.d_in * EB / ROWB + 2 * t.nkb1;
    t.uh = lora ? p.u_hi + (int64_t)t.row0 * ldu : t.q0;
    t.ul = lora ? p.u_lo + (int64_t)t.row0 * ldu : t.q0;
    t.be = lora ? p.B_stack + ((int64_t)e * p.d_out + t.n0) * ldu : t.p0;
    return t;
}

typedef int i32x4_t __attribute__((ext_vector_type(4)));
// One MFMA operand of a lane: 16 + 16 bytes of a row (see the head of the file).
typedef i32x8_t Frag;

}  // namespace mxs

// Shape of the kernel: one persistent workgroup of four waves per compute unit
// (one wave per SIMD, so each has the full 512 registers: 256 of accumulators for
// its 128 x 128 patch and two complete sets of MFMA operands), walking a list of
// 256 x 256 output tiles whose operand blocks form one stream through two LDS
// stages.  Codes, adapter operands and scale words all reach LDS directly
// (global_load_lds); the loop itself has no load into registers from global
// memory, so the only wait on the memory counter is the one in front of the
// per-block barrier.
//
// MX = false runs the same stream on a bf16 base (xq / Wq then hold x and W, there
// are no scales, and every block takes the bf16 MFMAs); it is not instantiated:
// measured against the eight-wave bf16 kernel on the 2048 -> 2048 prefill shape it
// took 262 us against 252 us on the same device.
template <bool MX, bool Y_F32>
__global__ __launch_bounds__(mxs::NT) void linear_stream4_kernel(mxs::Params p)
{
    using namespace mxs;
    constexpr int EB = MX ? 1 : 2;
    extern __shared__ __align__(16) char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = uniform(threadIdx.x >> 6);
    const int wp = wave / WQ, wq = wave % WQ;

    // work list of this workgroup: the 8 XCDs take workgroups round-robin, each
    // XCD owns one contiguous band of tile ids, and its workgroups stride
    // through the band together (neighbouring ids share W or x panels in L2)
    const int n_work = p.plain ? p.tiles_m * p.n_tiles_n * p.k_splits : uniform(*p.n_tiles) * p.n_tiles_n;
    const int per = (n_work + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, nslot = gridDim.x >> 3;
    const int band_end = min((xcd + 1) * per, n_work);
    int id = xcd * per + slot;
    if (id >= band_end) return;

    const int nkb0 = p.d_in * EB / ROWB;
    const uint32_t ldq = (uint32_t)p.d_in * EB, ldu = (uint32_t)p.r * 2u;

    // Requests of one block.  DMA mapping: instruction j of a wave fills LDS rows (wave*8 + j)*8 .. +8 of an
    // operand tile; the lane fetches logical 16-byte chunk (lane%8) ^ swz(row), swz(row) = (row >> 1) & 7
    // with row = wave*64 + j*8 + lane/8, which is lane/16 for even j and lane/16 + 4 for odd j.  With them
    // come the block's scale words: 64 rows of either operand per wave, one word per lane.  Per lane and
    // kernel: its first source row and the two chunk offsets; per block, uniform: the operand pointers at
    // the block's first k, the pitch, the operands' last valid rows.  A request (issue_one, n = 0..7 output
    // rows, 8..15 tokens, 16 / 17 the scale words) then costs an add, a min and a multiply-add, and goes
    // out behind an MFMA of its own.
    const uint32_t dma_row = (uint32_t)(wave * (LOADS * 8)) + ((uint32_t)lane >> 3);   // + 8 * j
    const uint32_t c16a = (((uint32_t)lane & 7) ^ ((uint32_t)lane >> 4)) * 16, c16b = c16a ^ 64u;   // even j, odd j
    struct Fetch {
        const char *pp, *pq, *ps, *qs;
        uint32_t ld, p_last, q_last;
    };
    auto fetch_of = [&](const Tile &t, int b) __attribute__((always_inline)) {
        Fetch f;
        const bool base = b < nkb0;
        const int jb = b - nkb0;
        const bool hi = jb < t.nkb1;
        const int kb = base ? b : (hi ? jb : jb - t.nkb1);
        f.pq = (base ? t.q0 : (hi ? t.uh : t.ul)) + kb * ROWB;
        f.pp = (base ? t.p0 : t.be) + kb * ROWB;
        f.ld = base ? ldq : ldu;
        f.p_last = (uint32_t)(t.p_rows - 1);
        f.q_last = (uint32_t)(t.q_rows - 1);
        f.ps = f.qs = nullptr;
        if constexpr (MX) {
            // (an adapter block has no scales; it repeats the loads of the tile's first
            // block, so that the body needs no branch)
            const int sb = base ? b : 0;
            f.ps = p.Ws + ((int64_t)(t.kb0 + sb) * p.d_out + t.n0) * 4;
            f.qs = p.xs + ((int64_t)(t.kb0 + sb) * p.T + t.row0) * 4;
        }
        return f;
    };
    auto issue_one = [&](const Fetch &f, int st, int n) __attribute__((always_inline)) {
        char *stage = smem + st * STAGE_BYTES;
        if (n < 2 * LOADS) {
            const int j = n & (LOADS - 1);
            const bool q = n >= LOADS;
            const uint32_t row = min(dma_row + 8u * j, q ? f.q_last : f.p_last);
            const uint32_t off = __umul24(row, f.ld) + ((j & 1) ? c16b : c16a);
            __builtin_amdgcn_global_load_lds(MOIN_GPTR((q ? f.pq : f.pp) + off),
                                             MOIN_LPTR(stage + (q ? OP_BYTES : 0) + (wave * LOADS + j) * 1024), 16, 0, 0);
        } else if constexpr (MX) {
            char *sc_ = smem + SMEM_STAGES + st * SC_BYTES;
            const bool q = n == 2 * LOADS + 1;
            const uint32_t row = min((uint32_t)(wave * 64) + (uint32_t)lane, q ? f.q_last : f.p_last);
            __builtin_amdgcn_global_load_lds(MOIN_GPTR((q ? f.qs : f.ps) + row * 4u),
                                             MOIN_LPTR(sc_ + (q ? BT * 4 : 0) + wave * 256), 4, 0, 0);
        }
    };
    auto issue = [&](const Tile &t, int b, int st) __attribute__((always_inline)) {
        const Fetch f = fetch_of(t, b);
#pragma unroll
        for (int n = 0; n < 2 * LOADS + (MX ? 2 : 0); ++n) issue_one(f, st, n);
    };

    // fragment addresses: byte (16 h) ^ (16 f) of the lane's row in the first patch of
    // each operand, f = (r >> 1) & 7; the row offsets are multiples of 128, so chunk
    // c = 4 ks + 2 * half of that row is at (this address) ^ (16 c)
    const int lo_ = ((lane & 31) * ROWB) | ((((lane >> 5) ^ (lane >> 1)) & 7) * 16);   // r * ROWB + ((h ^ f) & 7) * 16
    const int baseP = wp * (FP * 32) * ROWB, baseQ = OP_BYTES + wq * (FQ * 32) * ROWB;   // wave-uniform
    Frag fp[2][FP], fq[2][FQ];
    auto read_frag = [&](Frag &g, const char *stage_, int row, int ks) __attribute__((always_inline)) {
        const i32x4_t lo = *reinterpret_cast<const i32x4_t *>(stage_ + (row ^ (ks * 64)));
        const i32x4_t hi = *reinterpret_cast<const i32x4_t *>(stage_ + (row ^ (ks * 64 + 32)));
        g = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    // fragment n of a k-step: 0..3 output blocks, 4..7 token blocks
    auto read_frag_n = [&](const char *stage, int ks, int n) __attribute__((always_inline)) {
        if (n < FP) read_frag(fp[ks][n], stage, baseP + lo_ + n * 32 * ROWB, ks);
        else read_frag(fq[ks][n - FP], stage, baseQ + lo_ + (n - FP) * 32 * ROWB, ks);
    };
    auto read_frags = [&](const char *stage, int ks) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < FP + FQ; ++n) read_frag_n(stage, ks, n);
    };
    // scale words of this lane's rows, as they lie in LDS (sc_raw: the four bytes of
    // a row's 128 steps) and regrouped (sc: word n holds, for fragments 2n and 2n + 1,
    // the bytes this lane feeds the MFMAs of k-steps 0 and 1; a lane supplies the
    // scale of the first 32-step block of a 64-step slice if h = 0, of the second if 1)
    uint32_t sc_raw[NSC], sc[NSC / 2];
    auto read_scale_n = [&](const char *area, int n) __attribute__((always_inline)) {
        const int r = lane & 31;
        if (n < FP) sc_raw[n] = *reinterpret_cast<const uint32_t *>(area + (wp * (FP * 32) + n * 32 + r) * 4);
        else sc_raw[n] = *reinterpret_cast<const uint32_t *>(area + (BT + wq * (FQ * 32) + (n - FP) * 32 + r) * 4);
    };
    auto read_scales = [&](const char *area) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < NSC; ++n) read_scale_n(area, n);
    };
    auto regroup = [&]() __attribute__((always_inline)) {
        const uint32_t pick = 0x06040200u + (uint32_t)(lane >> 5) * 0x01010101u;   // h = 1: 0x07050301
#pragma unroll
        for (int n = 0; n < NSC / 2; ++n) sc[n] = __builtin_amdgcn_perm(sc_raw[2 * n + 1], sc_raw[2 * n], pick);
    };

    f32x16_t acc[FP][FQ];
    auto lo16 = [](const Frag &g) __attribute__((always_inline)) {
        return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(g, g, 0, 1, 2, 3));
    };
    auto hi16 = [](const Frag &g) __attribute__((always_inline)) {
        return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(g, g, 4, 5, 6, 7));
    };
    // acc[I][J] += fragment pair: one scaled FP8 MFMA on a base block, two bf16
    // MFMAs on an adapter block
    // (ZERO: the tile's first MFMA on this accumulator takes a constant zero as its addend, so the
    // accumulators are never cleared: 256 register writes per tile, 5.6 cycles each at one wave per SIMD)
    auto mfma_one = [&](auto base_tag, auto ks_tag, auto i_tag, auto j_tag, auto zero_tag) __attribute__((always_inline)) {
        constexpr bool BASE = decltype(base_tag)::value, ZERO = decltype(zero_tag)::value;
        constexpr int KS = decltype(ks_tag)::value, I = decltype(i_tag)::value, J = decltype(j_tag)::value;
        const f32x16_t c0 = ZERO ? f32x16_t{} : acc[I][J];
        if constexpr (BASE) {
            acc[I][J] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                fp[KS][I], fq[KS][J], c0, 0, 0, (I & 1) * 2 + KS, (int)sc[I / 2], (J & 1) * 2 + KS,
                (int)sc[FP / 2 + J / 2]);
        } else {
            acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo16(fp[KS][I]), lo16(fq[KS][J]), c0, 0, 0, 0);
            acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi16(fp[KS][I]), hi16(fq[KS][J]), acc[I][J], 0, 0, 0);
        }
    };
    static_assert(FP == 4 && FQ == 4 && LOADS == 8, "the steps below are written out for 4 x 4 accumulators");

    Tile cur = load_tile<MX>(p, id, band_end);
    id += nslot;
    Tile nxt = load_tile<MX>(p, id, band_end);

    // fetch cursor: tile and block index of the next block to request
    Tile pft = cur;
    int pfb = 2;
    Fetch fsecond;   // what the second half of the block under way requests

    // One block of the stream: k-step 0 (its fragments were read during the block before) with the reads
    // of k-step 1 between its MFMAs; barrier (own share of block s+1 has landed and every fragment of
    // block s is in registers; past the barrier that holds for all waves); k-step 1 with the requests for
    // the block two ahead -- into the stage this block frees -- and the next block's scales and leading
    // fragments between its MFMAs.  One wave per SIMD: an MFMA keeps the matrix core busy for 64 cycles
    // (32 on an adapter block), 4 of them its own issue, and whatever stands between two MFMAs and takes
    // longer than the rest delays the second.  So the other work is dealt out one piece per MFMA -- a
    // fragment (two LDS reads), a request with its three address instructions (about 40 cycles together),
    // a scale word -- and the source order IS the instruction order (a scheduling barrier after every
    // step).  With the steps left to the scheduler's group barriers a block of 32 MFMAs took 3500 cycles.
    // BASE: kind of this block.  At the stream's end the requests and reads are repeated requests and
    // stale bytes of LDS that nothing uses: no branch after the barrier.
    // (An MFMA has no side effects, so only data flow keeps it in its place: its accumulator and the
    // output-rows fragment of the NEXT step's MFMA pass through an empty assembly statement that also
    // stands for a memory access -- the MFMA cannot sink below it, the next one cannot rise above it, and
    // no LDS read or request crosses it.)
    auto first_half_step = [&](auto base_tag, auto first_tag, auto n_tag, int s) __attribute__((always_inline)) {
        constexpr int n = decltype(n_tag)::value;
        using std::integral_constant;
        mfma_one(base_tag, integral_constant<int, 0>{}, integral_constant<int, n / FQ>{}, integral_constant<int, n % FQ>{}, first_tag);
        if constexpr (n + 1 < FP * FQ) asm volatile("" : "+a"(acc[n / FQ][n % FQ]), "+v"(fp[0][(n + 1) / FQ]) : : "memory");
        else asm volatile("" : "+a"(acc[n / FQ][n % FQ]) : : "memory");
        if (n < FP + FQ) read_frag_n(smem + (s & 1) * STAGE_BYTES, 1, n);
        if (n == 10) {
            // The fetch cursor runs two blocks ahead; when it has used up its tile it moves to the tile
            // after the one being computed (by now `nxt` is that tile in every case); past the last
            // tile it requests that tile's last block again, into the stage that is free anyway.
            if (pfb == pft.total) {
                if (nxt.valid) {
                    pft = nxt;
                    pfb = 0;
                } else {
                    pfb = pft.total - 1;
                }
            }
            fsecond = fetch_of(pft, pfb);
            ++pfb;
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto second_half_step = [&](auto base_tag, auto n_tag, int s) __attribute__((always_inline)) {
        constexpr int n = decltype(n_tag)::value;
        using std::integral_constant;
        mfma_one(base_tag, integral_constant<int, 1>{}, integral_constant<int, n / FQ>{}, integral_constant<int, n % FQ>{}, std::false_type{});
        if constexpr (n + 1 < FP * FQ) asm volatile("" : "+a"(acc[n / FQ][n % FQ]), "+v"(fp[1][(n + 1) / FQ]) : : "memory");
        else asm volatile("" : "+a"(acc[n / FQ][n % FQ]) : : "memory");
        if (n < FP + FQ) read_frag_n(smem + ((s + 1) & 1) * STAGE_BYTES, 0, n);
        else if constexpr (MX) read_scale_n(smem + SMEM_STAGES + ((s + 1) & 1) * SC_BYTES, n - (FP + FQ));
        issue_one(fsecond, s & 1, n);
        if constexpr (MX) {
            if (n == 3) issue_one(fsecond, s & 1, 2 * LOADS);
            if (n == 7) issue_one(fsecond, s & 1, 2 * LOADS + 1);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto body = [&](int s, auto base_tag, auto first_tag) __attribute__((always_inline)) {
        using std::integral_constant;
#define MOIN_MX_STEPS(F, ...)                                                                            \
    F(__VA_ARGS__, integral_constant<int, 0>{}, s); F(__VA_ARGS__, integral_constant<int, 1>{}, s);       \
    F(__VA_ARGS__, integral_constant<int, 2>{}, s); F(__VA_ARGS__, integral_constant<int, 3>{}, s);       \
    F(__VA_ARGS__, integral_constant<int, 4>{}, s); F(__VA_ARGS__, integral_constant<int, 5>{}, s);       \
    F(__VA_ARGS__, integral_constant<int, 6>{}, s); F(__VA_ARGS__, integral_constant<int, 7>{}, s);       \
    F(__VA_ARGS__, integral_constant<int, 8>{}, s); F(__VA_ARGS__, integral_constant<int, 9>{}, s);       \
    F(__VA_ARGS__, integral_constant<int, 10>{}, s); F(__VA_ARGS__, integral_constant<int, 11>{}, s);     \
    F(__VA_ARGS__, integral_constant<int, 12>{}, s); F(__VA_ARGS__, integral_constant<int, 13>{}, s);     \
    F(__VA_ARGS__, integral_constant<int, 14>{}, s); F(__VA_ARGS__, integral_constant<int, 15>{}, s);
        MOIN_MX_STEPS(first_half_step, base_tag, first_tag)
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        MOIN_MX_STEPS(second_half_step, base_tag)
#undef MOIN_MX_STEPS
        if constexpr (MX) regroup();
        __builtin_amdgcn_sched_barrier(0);
    };

    // prologue of the stream: two blocks in flight, the first one landed
    issue(cur, 0, 0);
    issue(cur, 1, 1);   // every tile has at least two blocks
    wait_vm_then_barrier<2 * LOADS + (MX ? 2 : 0)>();

    int s = 0;
    for (;;) {
        // scales and leading fragments of the tile's first block (it has landed: the
        // prologue, or the previous tile's last barrier, waited for it).  The previous
        // tile's last block read them too, like every block reads its successor's, but
        // operands held across the epilogue would be spilled there and reloaded here.
        if constexpr (MX) read_scales(smem + SMEM_STAGES + (s & 1) * SC_BYTES);
        read_frags(smem + (s & 1) * STAGE_BYTES, 0);
        if constexpr (MX) regroup();
        const int total = cur.total;
        const int nb = min(nkb0, total);   // a part of a plain tile has fewer blocks than the full range; >= 1
        body(s, std::integral_constant<bool, MX>{}, std::true_type{});
        ++s;
        int b = 1;
        for (; b < nb; ++b, ++s) body(s, std::integral_constant<bool, MX>{}, std::false_type{});
        for (; b < total; ++b, ++s) body(s, std::false_type{}, std::false_type{});

        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // the last MFMAs' results before the epilogue's assembly reads them
        // epilogue through the wave's private 4 KB of LDS beyond the stages (which
        // the next tile's loads are already filling)
        // (the lane id goes in through an opaque copy: the epilogue's per-lane
        // addresses are then recomputed per tile instead of being kept, and
        // spilled, across the main loop)
        int lane_e = lane;
        asm volatile("; lane id, rematerialised" : "+v"(lane_e));
        stream_epilogue_as<FP, FQ, Y_F32>(smem + SMEM_STAGES + SMEM_SCALES + wave * SCR_BYTES, acc, p.y + cur.y_off, p.d_out,
                                          cur.row0, cur.n0, cur.q_rows, cur.p_rows, wp, wq, lane_e);
        if (!nxt.valid) break;
        cur = nxt;
        id += nslot;
        nxt = load_tile<MX>(p, id, band_end);
    }
    // the last blocks' repeated requests must have landed before the LDS is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

hipError_t prepare_mx_kernels()
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&linear_stream4_kernel<true, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, mxs::SMEM_BYTES);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&linear_stream4_kernel<true, true>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, mxs::SMEM_BYTES);
}

bool mx_stream_kernel_fits(int d_in, int r) { return d_in % 128 == 0 && d_in >= 256 && r % 64 == 0; }

// Parts of the contraction range for the plain (decode) base product: enough
// workgroups to keep many loads in flight, at least two blocks per part, at most
// four parts (the decode expand kernel sums up to four partial planes).
void mx_plain_shape(int64_t T, int d_in, int d_out, int *k_splits, int *kb_per_split)
{
    const int nkb = d_in / 128;
    const int64_t tiles = ((T + mxs::BT - 1) / mxs::BT) * ((d_out + mxs::BT - 1) / mxs::BT);
    int want = (int)((128 + tiles - 1) / (tiles > 0 ? tiles : 1));
    if (want > 4) want = 4;
    if (want < 1) want = 1;
    for (;; --want) {
        const int per = (nkb + want - 1) / want;
        const int parts = (nkb + per - 1) / per;
        const int last = nkb - (parts - 1) * per;
        if (want == 1 || (per >= 2 && last >= 2)) {   // every part streams at least two blocks
            *kb_per_split = per;
            *k_splits = parts;
            return;
        }
    }
}

hipError_t launch_linear_mx_stream(const PlanView &pv, const MxLinearArgs &a, int n_cus, hipStream_t stream_)
{
    mxs::Params p;
    p.xq = (const char *)a.xq; p.Wq = (const char *)a.Wq; p.xs = (const char *)a.xs; p.Ws = (const char *)a.Ws;
    p.T = pv.T;
    p.B_stack = (const char *)a.lin.B_stack;
    p.u_hi = (const char *)a.lin.u_hi; p.u_lo = (const char *)a.lin.u_lo;
    p.y = (char *)a.lin.y;
    p.tile_row0 = pv.tile_row0; p.tile_rows = pv.tile_rows; p.tile_expert = pv.tile_expert;
    p.tile_rank = pv.tile_rank;
    p.n_tiles = pv.n_tiles;
    p.d_in = a.lin.d_in; p.d_out = a.lin.d_out; p.r = a.lin.r;
    p.n_tiles_n = (a.lin.d_out + mxs::BT - 1) / mxs::BT;
    p.y_f32 = a.lin.y_f32;
    p.plain = a.plain_splits > 0;
    p.tiles_m = (int)((pv.T + mxs::BT - 1) / mxs::BT);
    p.k_splits = a.plain_splits > 0 ? a.plain_splits : 1;
    p.kb_per_split = a.plain_kb_per_split;
    p.plane_bytes = (int64_t)pv.T * a.lin.d_out * (a.lin.y_f32 ? 4 : 2);
    // one workgroup per compute unit (the LDS footprint allows no more), fewer
    // when the batch has fewer tiles than that; always a multiple of 8
    const int64_t max_work = p.plain ? (int64_t)p.tiles_m * p.n_tiles_n * p.k_splits
                                     : (int64_t)pv.max_tiles * p.n_tiles_n;
    int64_t grid = n_cus > 0 ? n_cus : 256;
    if (grid > max_work) grid = max_work;
    grid = (grid + 7) / 8 * 8;
    // (one instantiation per output type: with both epilogues in one kernel the
    // compiler moved accumulators through scratch memory at every tile's end)
    if (a.lin.y_f32)
        hipLaunchKernelGGL((linear_stream4_kernel<true, true>), dim3((unsigned)grid), dim3(mxs::NT), mxs::SMEM_BYTES,
                           stream_, p);
    else
        hipLaunchKernelGGL((linear_stream4_kernel<true, false>), dim3((unsigned)grid), dim3(mxs::NT), mxs::SMEM_BYTES,
                           stream_, p);
    return hipGetLastError();
}

}  // namespace moin
