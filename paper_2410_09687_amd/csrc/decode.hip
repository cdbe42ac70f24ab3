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
// Idle MFMA columns cost nothing here: the kernels are HBM-bound.
//
//   shrink : ug[pos, :]   = scale * A_e x_tok     (bf16 high part + remainder)
//   expand : ylora[tok,:] = B_e ug[pos]           (fp32, added by the base GEMM)
#include "gemm_core.h"
#include "kernels.h"

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

// grid (max_groups, ceil(r / 16)), 256 threads: the 4 waves split the d_in range.
__global__ __launch_bounds__(256) void decode_shrink_kernel(
    const char *x, const char *A_stack, char *ug_hi, char *ug_lo, const int *tok_sorted,
    const int *grp_expert, const int *grp_start, const int *n_groups, int d_in, int r, float scale)
{
    __shared__ float red[4][64][4];
    const int g = blockIdx.x;
    if (g >= uniform(*n_groups)) return;
    const int e = uniform(grp_expert[g]);
    if (e < 0) return;
    const int gs = uniform(grp_start[g]), ge = uniform(grp_start[g + 1]);
    if (ge <= gs) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j0 = blockIdx.y * 16;
    const int jrow = j0 + (lane & 15);
    const bool jvalid = jrow < r;
    const int kq = (lane >> 4) * 8;               // element offset of this lane's k-group
    const int64_t ld = (int64_t)d_in * 2;
    const char *arow = A_stack + ((int64_t)e * r + (jvalid ? jrow : 0)) * ld;
    const int nks = (d_in + 31) / 32;

    for (int t0 = gs; t0 < ge; t0 += 16) {
        const int pos = t0 + (lane & 15);
        const bool tvalid = pos < ge;
        const char *xrow = x + (int64_t)(tvalid ? tok_sorted[pos] : 0) * ld;
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
        // UNR independent load pairs in flight per lane before the MFMAs that
        // consume them; steps past the row end are zero-masked by ldg_frag
        constexpr int UNR = 8;
        for (int ks0 = wave; ks0 < nks; ks0 += 4 * UNR) {
            bf16x8_t a[UNR], b[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int k = (ks0 + 4 * u) * 32 + kq;
                a[u] = ldg_frag(arow, k, d_in);
                b[u] = ldg_frag(xrow, k, d_in);
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], b[u], acc, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) red[wave][lane][i] = acc[i];
        __syncthreads();
        if (wave == 0) {
            // lane holds u[token = lane % 16][j0 + 4 * (lane / 16) + i]
            uint32_t h[4], l[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float f =
                    (red[0][lane][i] + red[1][lane][i] + red[2][lane][i] + red[3][lane][i]) * scale;
                h[i] = f32_to_bf16_bits(f);
                l[i] = f32_to_bf16_bits(f - bf16_bits_to_f32(h[i]));
            }
            const int jj = j0 + 4 * (lane >> 4);
            if (tvalid && jj < r) {   // r % 8 == 0, so a group of 4 is all in or all out
                const int64_t off = ((int64_t)pos * r + jj) * 2;
                *reinterpret_cast<uint2 *>(ug_hi + off) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                *reinterpret_cast<uint2 *>(ug_lo + off) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
            }
        }
        __syncthreads();
    }
}

// grid (max_groups, ceil(d_out / 256)), 256 threads: each wave owns 64 rows of
// B_e (a contiguous 64 * r * 2 byte slab).
template <int KS_HOLD>
__global__ __launch_bounds__(256) void decode_expand_kernel(
    const char *B_stack, const char *ug_hi, const char *ug_lo, float *ylora, const int *tok_sorted,
    const int *grp_expert, const int *grp_start, const int *n_groups, int d_out, int r)
{
    const int g = blockIdx.x;
    if (g >= uniform(*n_groups)) return;
    const int e = uniform(grp_expert[g]);
    if (e < 0) return;
    const int gs = uniform(grp_start[g]), ge = uniform(grp_start[g + 1]);
    if (ge <= gs) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int o_base = blockIdx.y * 256 + wave * 64;
    if (o_base >= d_out) return;
    const int kq = (lane >> 4) * 8;
    const int64_t ldb = (int64_t)r * 2;
    const int nks = (r + 31) / 32;
    const char *bexp = B_stack + (int64_t)e * d_out * ldb;

    for (int t0 = gs; t0 < ge; t0 += 16) {
        const int pos = t0 + (lane & 15);
        const bool tvalid = pos < ge;
        const int tok = tvalid ? tok_sorted[pos] : 0;
        const char *uh = ug_hi + (int64_t)(tvalid ? pos : gs) * ldb;
        const char *ul = ug_lo + (int64_t)(tvalid ? pos : gs) * ldb;
        bf16x8_t fh[KS_HOLD > 0 ? KS_HOLD : 1], fl[KS_HOLD > 0 ? KS_HOLD : 1];
        if (KS_HOLD > 0) {
#pragma unroll
            for (int ks = 0; ks < KS_HOLD; ++ks) {
                const int k = ks * 32 + kq;
                fh[ks] = ldg_frag(uh, k, r);
                fl[ks] = ldg_frag(ul, k, r);
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int orow = o_base + c * 16 + (lane & 15);
            const bool ovalid = orow < d_out;
            const char *brow = bexp + (int64_t)(ovalid ? orow : 0) * ldb;
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
            if (KS_HOLD > 0) {
#pragma unroll
                for (int ks = 0; ks < KS_HOLD; ++ks) {
                    const int k = ks * 32 + kq;
                    const bf16x8_t a = ldg_frag(brow, k, r);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, fh[ks], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, fl[ks], acc, 0, 0, 0);
                }
            } else {
                for (int ks = 0; ks < nks; ++ks) {
                    const int k = ks * 32 + kq;
                    const bf16x8_t a = ldg_frag(brow, k, r);
                    const bf16x8_t bh = ldg_frag(uh, k, r);
                    const bf16x8_t bl = ldg_frag(ul, k, r);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl, acc, 0, 0, 0);
                }
            }
            // lane holds ylora[token = lane % 16][o_base + c*16 + 4*(lane/16) + i]
            const int oo = o_base + c * 16 + 4 * (lane >> 4);
            if (tvalid && oo < d_out)   // d_out % 4 == 0
                *reinterpret_cast<f32x4_t *>(ylora + (int64_t)tok * d_out + oo) = acc;
        }
    }
}

hipError_t launch_decode_shrink(const PlanView &pv, const DecodeArgs &d, hipStream_t stream)
{
    const LinearArgs &a = d.lin;
    if (a.r <= 0 || pv.max_groups <= 0) return hipSuccess;
    dim3 grid((unsigned)pv.max_groups, (unsigned)((a.r + 15) / 16));
    hipLaunchKernelGGL(decode_shrink_kernel, grid, dim3(256), 0, stream, (const char *)a.x,
                       (const char *)a.A_stack, (char *)d.ug_hi, (char *)d.ug_lo, pv.tok_sorted,
                       pv.grp_expert, pv.grp_start, pv.n_groups, a.d_in, a.r, a.scale);
    return hipGetLastError();
}

hipError_t launch_decode_expand(const PlanView &pv, const DecodeArgs &d, hipStream_t stream)
{
    const LinearArgs &a = d.lin;
    if (a.r <= 0 || pv.max_groups <= 0) return hipSuccess;
    dim3 grid((unsigned)pv.max_groups, (unsigned)((a.d_out + 255) / 256));
    const int nks = (a.r + 31) / 32;
#define MOIN_EXPAND(KS)                                                                         \
    hipLaunchKernelGGL(decode_expand_kernel<KS>, grid, dim3(256), 0, stream,                    \
                       (const char *)a.B_stack, (const char *)d.ug_hi, (const char *)d.ug_lo,   \
                       d.ylora, pv.tok_sorted, pv.grp_expert, pv.grp_start, pv.n_groups,        \
                       a.d_out, a.r)
    if (nks <= 1) MOIN_EXPAND(1);
    else if (nks <= 2) MOIN_EXPAND(2);
    else if (nks <= 4) MOIN_EXPAND(4);
    else MOIN_EXPAND(0);
#undef MOIN_EXPAND
    return hipGetLastError();
}

}  // namespace moin
