// Merged adapters ("Future Works", creating new experts on the fly: a server that merges
// existing adapters for a query that needs several): the weighted sum
// sum_m w_m W_b[e_m] W_a[e_m] written as one adapter of rank n r by concatenation,
//     A_out[m r + j, :] = A[e_m][j, :],   B_out[:, m r + j] = bf16(w_m * B[e_m][:, j]),
// the product taken in fp32 and rounded to nearest even.  Ids and weights are read on
// the device (they come from moin_route_topk and the caller's own weighting), an id
// of -1 gives a block of zeros, and so does everything from n r up to r_out.  Plain
// copies: one thread per 8 values.
#include "gemm_core.h"
#include "kernels.h"

namespace moin {

__global__ __launch_bounds__(256) void merge_a_kernel(const uint4 *__restrict__ A_stack, int E, int r, int d_in8,
                                                      const int *__restrict__ ids, int n, int r_out,
                                                      uint4 *__restrict__ A_out, int *err_word)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (int64_t)r_out * d_in8) return;
    const int row = (int)(t / d_in8), c8 = (int)(t - (int64_t)row * d_in8);
    const int m = row / r, j = row - m * r;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (m < n) {
        const int e = ids[m];
        if (e >= E || e < -1) {
            if (c8 == 0 && j == 0) atomicOr(err_word, ERR_BAD_EXPERT);
        } else if (e >= 0) {
            v = A_stack[((int64_t)e * r + j) * d_in8 + c8];
        }
    }
    A_out[t] = v;
}

// B_out [d_out, r_out]: thread = (output row o, 8 consecutive columns); r % 8 == 0, so the
// eight columns lie in one block m
__global__ __launch_bounds__(256) void merge_b_kernel(const uint4 *__restrict__ B_stack, int E, int r8, int d_out,
                                                      const int *__restrict__ ids, const float *__restrict__ weights,
                                                      int n, int r_out8, uint4 *__restrict__ B_out)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (int64_t)d_out * r_out8) return;
    const int o = (int)(t / r_out8), c8 = (int)(t - (int64_t)o * r_out8);
    const int m = c8 / r8, j8 = c8 - m * r8;
    uint4 out = make_uint4(0, 0, 0, 0);
    if (m < n) {
        const int e = ids[m];
        if (e >= 0 && e < E) {
            const float w = weights[m];
            const uint4 v = B_stack[((int64_t)e * d_out + o) * r8 + j8];
            const uint32_t in[4] = {v.x, v.y, v.z, v.w};
            uint32_t q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                q[i] = pack_bf16x2(bits_f32(in[i] << 16) * w, bits_f32(in[i] & 0xFFFF0000u) * w);
            out = make_uint4(q[0], q[1], q[2], q[3]);
        }
    }
    B_out[t] = out;
}

hipError_t launch_merge_adapters(const void *A_stack, const void *B_stack, int E, int r, int d_in, int d_out,
                                 const int *ids, const float *weights, int n, int r_out, void *A_out, void *B_out,
                                 int *err_word, hipStream_t stream)
{
    const int64_t na = (int64_t)r_out * (d_in / 8), nb = (int64_t)d_out * (r_out / 8);
    if (na > 0)
        hipLaunchKernelGGL(merge_a_kernel, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, stream,
                           reinterpret_cast<const uint4 *>(A_stack), E, r, d_in / 8, ids, n, r_out,
                           reinterpret_cast<uint4 *>(A_out), err_word);
    if (nb > 0)
        hipLaunchKernelGGL(merge_b_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, stream,
                           reinterpret_cast<const uint4 *>(B_stack), E, r / 8, d_out, ids, weights, n, r_out / 8,
                           reinterpret_cast<uint4 *>(B_out));
    return hipGetLastError();
}

}  // namespace moin
