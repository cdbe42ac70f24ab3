// Shared building blocks of the bf16 MFMA kernels (gfx950 / CDNA4 only).
//
// Both operands of every contraction here are row-major with the contraction
// index contiguous ("x[T,d_in] . W[d_out,d_in]^T", "centroids . queries^T"), so
// a lane can fetch the 8 consecutive bf16 that v_mfma_f32_32x32x16_bf16 wants
// with one 16-byte load.  A workgroup tile is BM x BN x BK; waves form a
// WM x WN grid and each owns a (BM/WM) x (BN/WN) patch made of 32x32 MFMA
// accumulators.  Global -> registers -> LDS staging, two LDS stages, one
// barrier per BK block.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moin {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t f32_bits(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float bits_f32(uint32_t u) { return __builtin_bit_cast(float, u); }

// fp32 -> bf16, round to nearest even; NaN stays a (quiet) NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = f32_bits(f);
    uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return (f != f) ? 0x7FC0u : rounded;
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return bits_f32(h << 16); }
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

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

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct GemmCore {
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

    // Row of the 32x32 accumulator that element e of a lane belongs to; the
    // column is lane % 32.
    __device__ static __forceinline__ int acc_row(int e, int lane)
    {
        return 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
    }

    // Hands the wave's patch to `emit(row, col, v[8])`, 8 consecutive columns
    // of one row at a time (row/col relative to the workgroup tile), by
    // transposing 32-row bands through the wave's private LDS scratch.  All
    // waves must have passed a barrier after their last compute_stage.
    template <typename Emit>
    __device__ static __forceinline__ void epilogue(char *smem, const Acc &acc, Emit emit)
    {
        const int lane = threadIdx.x & 63;
        const int wave = threadIdx.x >> 6;
        const int wm = wave / WN, wn = wave % WN;
        float *scr = reinterpret_cast<float *>(smem + wave * SCR_BYTES);
        constexpr int LPR = WTN / 8;      // lanes per row when reading back
        constexpr int RPASS = 64 / LPR;   // rows per read pass
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    scr[acc_row(e, lane) * SCR_PITCH + j * 32 + (lane & 31)] = acc.v[i][j][e];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int p = 0; p < 32 / RPASS; ++p) {
                const int rr = p * RPASS + lane / LPR;
                const int cc = (lane % LPR) * 8;
                const f32x4_t lo = *reinterpret_cast<const f32x4_t *>(scr + rr * SCR_PITCH + cc);
                const f32x4_t hi = *reinterpret_cast<const f32x4_t *>(scr + rr * SCR_PITCH + cc + 4);
                float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                emit(wm * WTM + i * 32 + rr, wn * WTN + cc, v);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
};

}  // namespace moin
