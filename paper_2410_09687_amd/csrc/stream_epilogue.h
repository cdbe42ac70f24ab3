// Epilogue shared by the streaming prefill kernels (256 x 256 output tiles; each
// wave holds FP x FQ accumulators of 32 outputs x 32 tokens).
#pragma once
#include "gemm_core.h"

namespace moin {

// Writes one wave's accumulators to y.  A lane holds, per accumulator, token
// (lane % 32) and outputs 8 * g + 4 * (lane / 32) + 0..3 for g = 0..3.  The wave
// regroups one 32-token block at a time through its private 4 KB of LDS (`scr`)
// so that eight lanes store one full 128-byte line of a token's row.
// row0 / n0: first token / output of the tile; q_rows / p_rows: valid tokens /
// outputs; wp / wq: the wave's position along outputs / tokens.
// Orders this wave's LDS accesses before and after it.  A wave's LDS instructions
// execute in the order they were issued, so lanes see each other's earlier writes
// without any wait; only the compiler has to be kept from moving accesses across.
// (A wavefront-scope fence would do as well, but it is compiled to a wait on every
// outstanding memory operation, the tile's own global stores included.)
// The scheduling fence also keeps the next block's accumulator reads from being
// hoisted above this point: all at once they do not fit the register file.
__device__ __forceinline__ void lds_order()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}

// Y_F32: y is fp32 (else bf16, rounded to nearest even).
template <int FP, int FQ, bool Y_F32>
__device__ __forceinline__ void stream_epilogue_as(char *scr, const f32x16_t (&acc)[FP][FQ], char *y, int d_out,
                                                   int row0, int n0, int q_rows, int p_rows, int wp, int wq,
                                                   int lane)
{
    const int r = lane & 31, h = lane >> 5;
    const int m2 = lane >> 3, c2 = lane & 7;   // read-back: token m2 + 8 * pass, 16-byte chunk c2
    if constexpr (Y_F32) {
        const int64_t ldy = (int64_t)d_out * 4;
#pragma unroll
        for (int j = 0; j < FQ; ++j) {
#pragma unroll
            for (int i = 0; i < FP; ++i) {
                // 32 tokens x 32 outputs fp32: 128-byte rows, 16-byte chunks swizzled by token
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x16_t &a = acc[i][j];
                    *reinterpret_cast<f32x4_t *>(scr + r * 128 + (((2 * g + h) ^ (r & 7)) * 16)) =
                        f32x4_t{a[4 * g], a[4 * g + 1], a[4 * g + 2], a[4 * g + 3]};
                }
                lds_order();
#pragma unroll
                for (int ps = 0; ps < 4; ++ps) {
                    const int mt = ps * 8 + m2;
                    const f32x4_t v = *reinterpret_cast<const f32x4_t *>(scr + mt * 128 + ((c2 ^ (mt & 7)) * 16));
                    const int m = wq * (FQ * 32) + j * 32 + mt;
                    const int n = wp * (FP * 32) + i * 32 + c2 * 4;
                    if (m < q_rows && n < p_rows)   // d_out % 8 == 0: a chunk is all in or all out
                        *reinterpret_cast<f32x4_t *>(y + (int64_t)(row0 + m) * ldy + (int64_t)(n0 + n) * 4) = v;
                }
                lds_order();
            }
        }
    } else {
        const int64_t ldy = (int64_t)d_out * 2;
        // 32 tokens x 64 outputs bf16: 128-byte rows of sixteen 8-byte slots;
        // the slot index is XORed with an even number, so slot pairs stay adjacent
        const int fw = ((r >> 1) & 7) << 1;
        static_assert(FP % 2 == 0, "outputs are regrouped 64 at a time");
#pragma unroll
        for (int j = 0; j < FQ; ++j) {
#pragma unroll
            for (int ip = 0; ip < FP / 2; ++ip) {
#pragma unroll
                for (int ii = 0; ii < 2; ++ii) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        // (the accumulators live in AccVGPRs; each value is read in place by an instruction
                        // of its own: left to itself the compiler copies whole accumulators out ahead of time,
                        // and the main loop's registers pay for it)
                        float a4[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a4[e]) : "a"(acc[ip * 2 + ii][j][4 * g + e]));
                        const int slot = ii * 8 + 2 * g + h;
                        *reinterpret_cast<uint2 *>(scr + r * 128 + ((slot ^ fw) * 8)) =
                            make_uint2(pack_bf16x2(a4[0], a4[1]), pack_bf16x2(a4[2], a4[3]));
                    }
                }
                lds_order();
#pragma unroll
                for (int ps = 0; ps < 4; ++ps) {
                    const int mt = ps * 8 + m2;
                    const int fr = ((mt >> 1) & 7) << 1;
                    const uint4 v = *reinterpret_cast<const uint4 *>(scr + mt * 128 + (((2 * c2) ^ fr) * 8));
                    const int m = wq * (FQ * 32) + j * 32 + mt;
                    const int n = wp * (FP * 32) + ip * 64 + c2 * 8;
                    if (m < q_rows && n < p_rows)
                        *reinterpret_cast<uint4 *>(y + (int64_t)(row0 + m) * ldy + (int64_t)(n0 + n) * 2) = v;
                }
                lds_order();
            }
        }
    }
}

// The same with the output type chosen at run time.
template <int FP, int FQ>
__device__ __forceinline__ void stream_epilogue(char *scr, const f32x16_t (&acc)[FP][FQ], char *y, int y_f32,
                                                int d_out, int row0, int n0, int q_rows, int p_rows,
                                                int wp, int wq, int lane)
{
    if (y_f32) stream_epilogue_as<FP, FQ, true>(scr, acc, y, d_out, row0, n0, q_rows, p_rows, wp, wq, lane);
    else stream_epilogue_as<FP, FQ, false>(scr, acc, y, d_out, row0, n0, q_rows, p_rows, wp, wq, lane);
}

}  // namespace moin
