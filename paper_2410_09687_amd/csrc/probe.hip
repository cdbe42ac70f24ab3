// On-box ceilings that the roofline fractions of the real kernels are read
// against, beside the datasheet peaks: a loop of nothing but bf16 MFMAs on
// operands the caller supplies (matrix-core throughput depends on the data: the
// chip runs into its power limit on random values long before it does on
// constants), and a plain streaming read.  Measurement aids, not steps of the
// method.
#include "gemm_core.h"
#include <algorithm>

#include "kernels.h"

namespace moin {

constexpr int PROBE_BLOCK = 512;      // 8 waves
constexpr int PROBE_WG_PER_CU = 2;
constexpr int PROBE_OPS = 4;          // A and B operand registers per lane (16 bytes each)

// Per iteration and wave: 32 independent v_mfma_f32_16x16x32_bf16 (the instruction of the prefill
// and router kernels; on N(0,1) operands the chip sustains some 13 % more flops with it than with
// v_mfma_f32_32x32x16_bf16 before it throttles, and the same on constants), no memory access.
// out[tid] = sum of the lane's accumulators.
__global__ __launch_bounds__(PROBE_BLOCK) void probe_mfma_kernel(const uint4 *__restrict__ in, uint32_t n16,
                                                                 int iters, float *__restrict__ out)
{
    const uint32_t tid = blockIdx.x * PROBE_BLOCK + threadIdx.x;
    bf16x8_t a[PROBE_OPS], b[PROBE_OPS];
#pragma unroll
    for (int j = 0; j < PROBE_OPS; ++j) {
        a[j] = __builtin_bit_cast(bf16x8_t, in[(tid * (2u * PROBE_OPS) + j) % n16]);
        b[j] = __builtin_bit_cast(bf16x8_t, in[(tid * (2u * PROBE_OPS) + PROBE_OPS + j) % n16]);
    }
    f32x4_t acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 32; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3], b[(i >> 2) & 3], acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) s += acc[i][e];
    out[tid] = s;
}

// The same for the block-scaled FP8 instruction of the quantised-base kernel: per
// iteration and wave eight independent v_mfma_scale_f32_32x32x64_f8f6f4 on operand
// registers filled from `in` (FP8 E4M3 codes), every block scale 2^0 (byte 127).
typedef int probe_i32x8_t __attribute__((ext_vector_type(8)));
__global__ __launch_bounds__(PROBE_BLOCK) void probe_mfma_mx_kernel(const uint4 *__restrict__ in, uint32_t n16,
                                                                    int iters, float *__restrict__ out)
{
    const uint32_t tid = blockIdx.x * PROBE_BLOCK + threadIdx.x;
    probe_i32x8_t a[2], b[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint4 a0 = in[(tid * 8u + 4 * j) % n16], a1 = in[(tid * 8u + 4 * j + 1) % n16];
        const uint4 b0 = in[(tid * 8u + 4 * j + 2) % n16], b1 = in[(tid * 8u + 4 * j + 3) % n16];
        a[j] = probe_i32x8_t{(int)a0.x, (int)a0.y, (int)a0.z, (int)a0.w, (int)a1.x, (int)a1.y, (int)a1.z, (int)a1.w};
        b[j] = probe_i32x8_t{(int)b0.x, (int)b0.y, (int)b0.z, (int)b0.w, (int)b1.x, (int)b1.y, (int)b1.z, (int)b1.w};
    }
    f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    const int sc = 0x7F7F7F7F;   // scale bytes: 2^(127 - 127) for both 32-step blocks
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i & 1], b[(i >> 1) & 1], acc[i], 0, 0, 0, sc, 0, sc);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    out[tid] = s;
}

// Every 16-byte word of src once: workgroups take 32 KB chunks in turn, a wave instruction
// reads 1 KB of consecutive bytes, eight loads per thread in flight, non-temporal (each byte
// is used once) -- the shape that read fastest in a sweep over strides, chunk sizes, depths
// and workgroup counts on this part (a grid-strided read of the same buffer is ~20 % slower,
// plain loads ~12 %).  out[tid] = sum (mod 2^32) of the 32-bit words the thread read.
typedef uint32_t probe_u32x4_t __attribute__((ext_vector_type(4)));
// Only the first `readers` workgroups read (two per compute unit: more of them read slower); the others
// just report zero, so that every element of out is written.
__global__ __launch_bounds__(256) void probe_read_kernel(const probe_u32x4_t *__restrict__ src, int64_t n16,
                                                         uint32_t *__restrict__ out, int readers)
{
    constexpr int64_t CHUNK = 2048;   // 16-byte words per chunk
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t s = 0;
    const int64_t full = n16 / CHUNK;
    if ((int)blockIdx.x >= readers) {
        out[tid] = 0;
        return;
    }
    for (int64_t c = blockIdx.x; c < full; c += readers) {
        const probe_u32x4_t *p = src + c * CHUNK + threadIdx.x;
        probe_u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u].x + v[u].y + v[u].z + v[u].w;
    }
    // what does not fill a chunk
    for (int64_t i = full * CHUNK + tid; i < n16; i += (int64_t)readers * 256) {
        const probe_u32x4_t v = src[i];
        s += v.x + v.y + v.z + v.w;
    }
    out[tid] = s;
}

int64_t probe_out_len() { return (int64_t)compute_units() * PROBE_WG_PER_CU * PROBE_BLOCK; }

hipError_t launch_probe_mfma(const void *operands, int64_t n_bytes, int iters, float *out, double *flops,
                             hipStream_t stream)
{
    const int grid = compute_units() * PROBE_WG_PER_CU;
    if (flops) *flops = (double)grid * (PROBE_BLOCK / 64) * (double)iters * 32.0 * (2.0 * 16 * 16 * 32);
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(grid), dim3(PROBE_BLOCK), 0, stream,
                       reinterpret_cast<const uint4 *>(operands), (uint32_t)(n_bytes / 16), iters, out);
    return hipGetLastError();
}

hipError_t launch_probe_mfma_mx(const void *codes, int64_t n_bytes, int iters, float *out, double *flops,
                                hipStream_t stream)
{
    const int grid = compute_units() * PROBE_WG_PER_CU;
    if (flops) *flops = (double)grid * (PROBE_BLOCK / 64) * (double)iters * 8.0 * (2.0 * 32 * 32 * 64);
    hipLaunchKernelGGL(probe_mfma_mx_kernel, dim3(grid), dim3(PROBE_BLOCK), 0, stream,
                       reinterpret_cast<const uint4 *>(codes), (uint32_t)(n_bytes / 16), iters, out);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void *src, int64_t n_bytes, uint32_t *out, hipStream_t stream)
{
    const int grid = (int)(probe_out_len() / 256);
    const int readers = std::min(grid, compute_units() * 2);
    hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, stream,
                       reinterpret_cast<const probe_u32x4_t *>(src), n_bytes / 16, out, readers);
    return hipGetLastError();
}

}  // namespace moin
