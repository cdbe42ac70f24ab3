// Shared building blocks of the bf16 MFMA kernels (gfx950 / CDNA4 only).
//
// Both operands of every contraction here are row-major with the contraction
// index contiguous ("x[T,d_in] . W[d_out,d_in]^T", "centroids . queries^T"), so
// a lane can fetch the 8 consecutive bf16 that v_mfma_f32_32x32x16_bf16 wants
// with one 16-byte load.  A workgroup tile is BM x BN x BK; waves form a
// WM x WN grid and each owns a (BM/WM) x (BN/WN) patch made of 32x32 MFMA
// accumulators.  Two ways of staging operands in LDS:
//   GemmCore : global -> registers -> LDS, rows padded by 16 B, two stages.
//              Handles any contraction length (the tail block is zero-filled).
//   DmaCore  : global -> LDS directly (global_load_lds_dwordx4), NS stages in
//              flight, unpadded rows with an XOR swizzle of the 16-byte chunks.
//              Needs the contraction length to be a multiple of BK.
// One barrier per BK block in both.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moin {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t f32_bits(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float bits_f32(uint32_t u) { return __builtin_bit_cast(float, u); }

// fp32 -> bf16, round to nearest even; NaN stays a (quiet) NaN.  The plain
// conversion compiles to gfx950's v_cvt_pk_bf16_f32 (two values per instruction).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.f) & 0xFFFFu; }
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return bits_f32(h << 16); }

// Activation between the adapter's two linear layers ("Future Works", better
// adapters): applied to W_a x in fp32, before the scale.  Codes as in moin.h.
__device__ __forceinline__ float adapter_act(float v, int act)
{
    switch (act) {
    case 1: return fmaxf(v, 0.f);                                  // ReLU
    case 2: return v / (1.f + expf(-v));                           // SiLU
    case 3: return 0.5f * v * (1.f + erff(v * 0.70710678118654752f));   // GELU
    default: return v;
    }
}

// Values read from global memory with a workgroup-uniform address are uniform,
// but the compiler cannot know; telling it keeps control flow and addressing
// that depend on them on the scalar unit.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Workgroups are handed to the 8 XCDs round-robin by linear id.  Remap so that
// each XCD works through one contiguous band of logical tile ids (its L2 then
// sees the same operand slabs from neighbouring tiles).  `total` logical ids;
// returns -1 for the padding ids of a grid rounded up to a multiple of 8.
__device__ __forceinline__ int xcd_band_id(int bid, int total)
{
    const int per = (total + 7) >> 3;
    const int xcd = bid & 7;
    const int slot = bid >> 3;
    // bands: the first (total % 8 or 8) XCDs own `per` ids ... keep it simple:
    // band x covers [x*per, min((x+1)*per, total)).
    const int id = xcd * per + slot;
    return (slot < per && id < total) ? id : -1;
}

// Row of the 32x32 accumulator that element e of a lane belongs to; the column
// is lane % 32.
__device__ __forceinline__ int mfma32_acc_row(int e, int lane)
{
    return 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
}

// Hands a wave's accumulator patch to `emit(row, col, v[8])`, 8 consecutive
// columns of one row at a time (row/col relative to the workgroup tile), by
// transposing 32-row bands through the wave's private LDS scratch, so that
// global stores can be 16 bytes per lane and row-contiguous.  All waves must
// have passed a barrier after their last read of the staging buffers.
template <class C, typename Emit>
__device__ __forceinline__ void tile_epilogue(char *smem, const typename C::Acc &acc, Emit emit)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave / C::WN, wn = wave % C::WN;
    float *scr = reinterpret_cast<float *>(smem + wave * C::SCR_BYTES);
    constexpr int LPR = C::WTN / 8;   // lanes per row when reading back
    constexpr int RPASS = 64 / LPR;   // rows per read pass
#pragma unroll
    for (int i = 0; i < C::FM; ++i) {
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                scr[mfma32_acc_row(e, lane) * C::SCR_PITCH + j * 32 + (lane & 31)] = acc.v[i][j][e];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int p = 0; p < 32 / RPASS; ++p) {
            const int rr = p * RPASS + lane / LPR;
            const int cc = (lane % LPR) * 8;
            const f32x4_t lo = *reinterpret_cast<const f32x4_t *>(scr + rr * C::SCR_PITCH + cc);
            const f32x4_t hi = *reinterpret_cast<const f32x4_t *>(scr + rr * C::SCR_PITCH + cc + 4);
            float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            emit(wm * C::WTM + i * 32 + rr, wn * C::WTN + cc, v);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct GemmCore {
    static constexpr bool IS_DMA = false;
    static constexpr int PF = 1;                     // blocks in flight per thread (see pipelined_blocks_deep)
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr int NT = 64 * WM * WN;          // threads per workgroup
    static constexpr int KCH = BK / 8;               // 16-byte chunks per tile row
    static constexpr int ROWB = BK * 2 + 16;         // padded LDS row pitch (bytes)
    static constexpr int RPP = NT / KCH;             // rows covered by one load pass
    static constexpr int A_CH = BM / RPP;            // chunks per thread, A operand
    static constexpr int B_CH = BN / RPP;
    static constexpr int A_BYTES = BM * ROWB;
    static constexpr int B_BYTES = BN * ROWB;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int FM = WTM / 32, FN = WTN / 32;
    static constexpr int KSTEPS = BK / 16;
    // epilogue scratch: one 32-row band of the wave's patch, fp32, padded
    static constexpr int SCR_PITCH = WTN + 4;        // floats
    static constexpr int SCR_BYTES = 32 * SCR_PITCH * 4;
    static constexpr int SMEM_BYTES =
        (2 * STAGE_BYTES > WM * WN * SCR_BYTES) ? 2 * STAGE_BYTES : WM * WN * SCR_BYTES;

    static_assert(NT % KCH == 0 && BM % RPP == 0 && BN % RPP == 0, "load mapping");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && BK % 16 == 0, "mfma tiling");
    static_assert(WTN % 8 == 0 && 64 % (WTN / 8) == 0, "epilogue mapping");

    struct Stage {
        uint4 a[A_CH];
        uint4 b[B_CH];
        uint32_t kmask;  // all-ones, or zero when this thread's chunk lies past the row end
    };
    struct Acc {
        f32x16_t v[FM][FN];
    };

    __device__ static __forceinline__ void zero(Acc &acc)
    {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc.v[i][j][e] = 0.f;
    }

    // A thread's share of one operand: NCH 16-byte chunks per BK block, one in
    // each of NCH rows RPP apart.  Rows past the valid count re-read the last
    // valid row: they only feed output rows or columns that the epilogue
    // masks, so their values never matter and the load needs no branch.
    template <int NCH>
    struct View {
        const char *base;      // uniform: (first tile row, k = 0)
        uint32_t rowoff[NCH];  // byte offset of each of this thread's rows
    };

    // rows >= 1; (rows - 1) * ld_bytes must fit 32 bits.
    template <int NCH>
    __device__ static __forceinline__ View<NCH> make_view(const char *base, uint32_t ld_bytes,
                                                          int rows)
    {
        View<NCH> v;
        v.base = base;
        const int row0 = threadIdx.x / KCH;
#pragma unroll
        for (int i = 0; i < NCH; ++i)
            v.rowoff[i] = (uint32_t)min(row0 + i * RPP, rows - 1) * ld_bytes;
        return v;
    }

    // Loads BK block starting at byte `kbyte` of rows that are `klim` bytes long.
    // A chunk at or past klim is fetched from k = 0 instead (in bounds) and
    // zeroed when it is written to LDS.
    __device__ static __forceinline__ void load_stage(Stage &g, const View<A_CH> &va,
                                                      const View<B_CH> &vb, uint32_t kbyte,
                                                      uint32_t klim)
    {
        const uint32_t kc = (uint32_t)(threadIdx.x % KCH) * 16u + kbyte;
        const bool kvalid = kc < klim;
        const uint32_t koff = kvalid ? kc : 0u;
        g.kmask = kvalid ? 0xFFFFFFFFu : 0u;
#pragma unroll
        for (int i = 0; i < A_CH; ++i)
            g.a[i] = *reinterpret_cast<const uint4 *>(va.base + (va.rowoff[i] + koff));
#pragma unroll
        for (int i = 0; i < B_CH; ++i)
            g.b[i] = *reinterpret_cast<const uint4 *>(vb.base + (vb.rowoff[i] + koff));
    }

    template <int NCH>
    __device__ static __forceinline__ void store_operand(char *smem, const uint4 (&src)[NCH],
                                                         uint32_t m)
    {
        const int tid = threadIdx.x;
        const int row0 = tid / KCH;
        const int kc = tid % KCH;
#pragma unroll
        for (int i = 0; i < NCH; ++i)
            *reinterpret_cast<uint4 *>(smem + (row0 + i * RPP) * ROWB + kc * 16) =
                make_uint4(src[i].x & m, src[i].y & m, src[i].z & m, src[i].w & m);
    }

    __device__ static __forceinline__ void store_stage(char *stage, const Stage &g)
    {
        store_operand<A_CH>(stage, g.a, g.kmask);
        store_operand<B_CH>(stage + A_BYTES, g.b, g.kmask);
    }

    // acc += A_tile . B_tile^T for one staged BK block.
    __device__ static __forceinline__ void compute_stage(const char *stage, Acc &acc)
    {
        const int lane = threadIdx.x & 63;
        const int wave = threadIdx.x >> 6;
        const int wm = wave / WN, wn = wave % WN;
        const char *pa = stage + (wm * WTM + (lane & 31)) * ROWB + (lane >> 5) * 16;
        const char *pb = stage + A_BYTES + (wn * WTN + (lane & 31)) * ROWB + (lane >> 5) * 16;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            bf16x8_t a[FM], b[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                a[i] = __builtin_bit_cast(
                    bf16x8_t, *reinterpret_cast<const uint4 *>(pa + i * 32 * ROWB + ks * 32));
#pragma unroll
            for (int j = 0; j < FN; ++j)
                b[j] = __builtin_bit_cast(
                    bf16x8_t, *reinterpret_cast<const uint4 *>(pb + j * 32 * ROWB + ks * 32));
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc.v[i][j] =
                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc.v[i][j], 0, 0, 0);
        }
    }

    template <typename Emit>
    __device__ static __forceinline__ void epilogue(char *smem, const Acc &acc, Emit emit)
    {
        tile_epilogue<GemmCore>(smem, acc, emit);
    }
};

// Main loop of the register-staged core over `total` BK blocks; `issue(it, g)`
// loads block `it` into the staging registers.
template <class C, class Issue>
__device__ __forceinline__ void pipelined_blocks(char *smem, int total, Issue issue,
                                                 typename C::Acc &acc)
{
    typename C::Stage g;
    issue(0, g);
    C::store_stage(smem, g);
    __syncthreads();
    for (int it = 0; it < total; ++it) {
        char *cur = smem + (it & 1) * C::STAGE_BYTES;
        char *nxt = smem + ((it + 1) & 1) * C::STAGE_BYTES;
        const bool more = it + 1 < total;
        if (more) issue(it + 1, g);
        C::compute_stage(cur, acc);
        if (more) C::store_stage(nxt, g);
        __syncthreads();
    }
}

// The same loop with the loads of PF blocks in flight per thread, for operands
// that stream from HBM: a load to registers may stay outstanding for several
// blocks, and the registers of block `it` go to LDS just before they are needed.
// `on_block(it, g)` sees block `it` in registers (after its copy to LDS, before
// the registers are reused).
template <class C, int PF, class Issue, class OnBlock>
__device__ __forceinline__ void pipelined_blocks_deep(char *smem, int total, Issue issue,
                                                      typename C::Acc &acc, OnBlock on_block)
{
    typename C::Stage g[PF];
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (u < total) issue(u, g[u]);
    for (int it0 = 0; it0 < total; it0 += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int it = it0 + u;
            if (it < total) {
                // stage it & 1 was last read for block it - 2: every wave has left that
                // block's MFMAs behind when it met the others at the barrier of block it - 1
                char *st = smem + (it & 1) * C::STAGE_BYTES;
                C::store_stage(st, g[u]);
                on_block(it, g[u]);
                if (it + PF < total) issue(it + PF, g[u]);
                __syncthreads();
                C::compute_stage(st, acc);
            }
        }
    }
    __syncthreads();
}

#define MOIN_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define MOIN_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

// Waits until at most N of this wave's vector-memory operations are still in
// flight (they retire in order), then meets the other waves at the barrier.
// The "memory" clobber keeps the compiler from moving LDS accesses across it.
template <int N>
__device__ __forceinline__ void wait_vm_then_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

template <int BM_, int BN_, int BK_, int WM_, int WN_, int NS_>
struct DmaCore {
    static constexpr bool IS_DMA = true;
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, NS = NS_;
    static constexpr int NW = WM * WN, NT = 64 * NW;
    static constexpr int KCH = BK / 8;                 // 16-byte chunks per tile row
    static constexpr int ROWB = BK * 2;                // LDS row pitch: no padding
    static constexpr int RPI = 64 / KCH;               // tile rows one wave instruction fills
    static constexpr int A_I = BM / RPI / NW;          // load instructions per wave per block
    static constexpr int B_I = BN / RPI / NW;
    static constexpr int LPB = A_I + B_I;
    static constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int FM = WTM / 32, FN = WTN / 32;
    static constexpr int KSTEPS = BK / 16;
    static constexpr int SCR_PITCH = WTN + 4;
    static constexpr int SCR_BYTES = 32 * SCR_PITCH * 4;
    static constexpr int SMEM_BYTES =
        (NS * STAGE_BYTES > NW * SCR_BYTES) ? NS * STAGE_BYTES : NW * SCR_BYTES;

    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "load mapping");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && BK % 16 == 0 && NS >= 2, "tiling");
    static_assert(ROWB <= 256 && 256 % ROWB == 0, "swizzle");
    static_assert((NS - 2) * LPB < 64, "vmcnt field");

    struct Acc {
        f32x16_t v[FM][FN];
    };

    __device__ static __forceinline__ void zero(Acc &acc)
    {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc.v[i][j][e] = 0.f;
    }

    // A wave instruction writes 64 consecutive 16-byte slots of LDS, so LDS slot
    // p of an operand tile is (row p / KCH, physical chunk p % KCH).  The lane
    // that fills it fetches logical chunk (p % KCH) ^ swz(row) from global
    // memory; readers apply the same XOR.  With swz(row) = (row / rows per 256
    // bytes) % KCH the ds_read_b128 of 32 consecutive rows at one logical chunk
    // is conflict-free.
    __device__ static __forceinline__ int swz(int row) { return (row / (256 / ROWB)) & (KCH - 1); }

    // For each of its wave's NI load instructions: the tile row this lane
    // fetches and the byte offset of its (swizzled) 16-byte chunk inside a BK
    // block.  Independent of the row pitch, so one table serves every operand
    // that shares the tile's row range (x and u; W and B_e).
    template <int NI>
    struct Lanes {
        uint32_t row[NI];
        uint32_t c16[NI];
    };

    // Rows past `rows` re-read the last valid row (their results are masked by
    // the epilogue).  rows >= 1.
    template <int NI>
    __device__ static __forceinline__ Lanes<NI> make_lanes(int rows)
    {
        Lanes<NI> o;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int row = (wave * NI + j) * RPI + lane / KCH;
            o.row[j] = (uint32_t)min(row, rows - 1);
            o.c16[j] = (uint32_t)(((lane % KCH) ^ swz(row)) * 16);
        }
        return o;
    }

    // Starts the loads of one BK block (byte offset kbyte inside the rows) of
    // both operands into `stage`.  a / b: uniform pointers to (first tile row,
    // k = 0); lda / ldb: row pitches in bytes; (rows - 1) * pitch + pitch must
    // fit 32 bits.
    __device__ static __forceinline__ void issue(char *stage, const char *a, uint32_t lda,
                                                 const Lanes<A_I> &la, const char *b, uint32_t ldb,
                                                 const Lanes<B_I> &lb, uint32_t kbyte)
    {
        const int wave = threadIdx.x >> 6;
#pragma unroll
        for (int j = 0; j < A_I; ++j)
            __builtin_amdgcn_global_load_lds(
                MOIN_GPTR(a + (la.row[j] * lda + la.c16[j] + kbyte)),
                MOIN_LPTR(stage + (wave * A_I + j) * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < B_I; ++j)
            __builtin_amdgcn_global_load_lds(
                MOIN_GPTR(b + (lb.row[j] * ldb + lb.c16[j] + kbyte)),
                MOIN_LPTR(stage + A_BYTES + (wave * B_I + j) * 1024), 16, 0, 0);
    }

    __device__ static __forceinline__ void compute_stage(const char *stage, Acc &acc)
    {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const int wm = wave / WN, wn = wave % WN;
        const int r = lane & 31, h = lane >> 5;
        // patch bases are multiples of 32 rows, so the swizzle depends on r only
        const int f = swz(r);
        // ask the scheduler for its MFMA / ds_read interleaving strategy (measured
        // +7 % on the 256x256x64 loop over the default order)
        __builtin_amdgcn_iglp_opt(1);
        const char *pa = stage + (wm * WTM + r) * ROWB;
        const char *pb = stage + A_BYTES + (wn * WTN + r) * ROWB;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            bf16x8_t a[FM], b[FN];
            const int o = (((ks * 2 + h) ^ f) & (KCH - 1)) * 16;
#pragma unroll
            for (int i = 0; i < FM; ++i)
                a[i] = __builtin_bit_cast(
                    bf16x8_t, *reinterpret_cast<const uint4 *>(pa + i * 32 * ROWB + o));
#pragma unroll
            for (int j = 0; j < FN; ++j)
                b[j] = __builtin_bit_cast(
                    bf16x8_t, *reinterpret_cast<const uint4 *>(pb + j * 32 * ROWB + o));
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc.v[i][j] =
                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc.v[i][j], 0, 0, 0);
        }
    }

    template <typename Emit>
    __device__ static __forceinline__ void epilogue(char *smem, const Acc &acc, Emit emit)
    {
        tile_epilogue<DmaCore>(smem, acc, emit);
    }
};

// Main loop of the direct-to-LDS core.  `issue(it, stage)` starts the loads of
// block `it` into `stage`; NS - 1 blocks are kept in flight.  `after(it)` runs
// after block `it` has been accumulated (router: fold a finished centroid tile).
// Ends with a barrier, so the staging buffers may be reused at once.
template <class C, class Issue, class After>
__device__ __forceinline__ void dma_pipelined_blocks(char *smem, int total, Issue issue,
                                                     typename C::Acc &acc, After after)
{
#pragma unroll
    for (int s = 0; s < C::NS - 1; ++s)
        if (s < total) issue(s, smem + s * C::STAGE_BYTES);
    int st = 0;   // stage that holds block `it`
    for (int it = 0; it < total; ++it) {
        // everything but the newest NS - 2 blocks has landed => block `it` is in LDS;
        // past the barrier every wave is done with block it - 1, whose stage is reused
        if (it + C::NS - 2 < total) wait_vm_then_barrier<(C::NS - 2) * C::LPB>();
        else wait_vm_then_barrier<0>();
        const int nb = it + C::NS - 1;
        const int ns = (st == 0) ? C::NS - 1 : st - 1;
        if (nb < total) issue(nb, smem + ns * C::STAGE_BYTES);
        C::compute_stage(smem + st * C::STAGE_BYTES, acc);
        after(it);
        st = (st + 1 == C::NS) ? 0 : st + 1;
    }
    __syncthreads();
}

}  // namespace moin
