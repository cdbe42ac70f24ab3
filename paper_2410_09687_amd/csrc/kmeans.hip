// Centre update of K-means (Section 3.1: the topics are the cells of a plain
// K-means clustering of the document embeddings and its cluster centres are
// the topic embeddings; Section 4 "Implementation details": k = 5000, clusters
// that stay extremely small are dropped).  The assignment step is the router.
//
// The update is a segmented mean over 1.6 GB of embeddings (1 048 576 x 768
// bf16) and is bound by HBM: every embedding row is read exactly once.
//   1. km_chunk_hist   per chunk of points, how many go to each centre
//   2. km_col_scan     per centre, prefix over the chunks (+ its total count)
//   3. km_segments     prefix over the centres; cuts each cluster's point list
//                      into pieces of at most KM_PIECE points (a heavy cluster
//                      must not hang on one workgroup)
//   4. km_scatter      stable counting sort: perm[] lists point indices grouped
//                      by centre, ascending inside a group, so sums run in a
//                      fixed order and results repeat bit for bit
//   5. km_segsum       one workgroup per piece streams its rows (16 bytes per
//                      lane, whole rows contiguous) into fp32 column sums and
//                      the piece's share of the objective
//   6. km_finalize     pieces -> mean (fp64 across pieces), empty clusters keep
//                      their old centre; the objective is summed in a fixed
//                      order in fp64
// No floating-point atomics anywhere.
#include "gemm_core.h"
#include "kernels.h"

namespace moin {

namespace {

__device__ __forceinline__ uint64_t lanemask_lt()
{
    const int lane = threadIdx.x & 63;
    return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

}  // namespace

// table[c][k] = number of points of chunk c assigned to centre k.  Ids outside
// [0, K) are left out (here and in the scatter) and raise the sticky fault.
__global__ __launch_bounds__(256) void km_chunk_hist(KmeansArgs a)
{
    extern __shared__ int km_bins[];
    const int K = a.K;
    for (int k = threadIdx.x; k < K; k += 256) km_bins[k] = 0;
    __syncthreads();
    const int64_t i0 = (int64_t)blockIdx.x * a.chunk;
    const int64_t i1 = min(a.N, i0 + a.chunk);
    bool bad = false;
    for (int64_t i = i0 + threadIdx.x; i < i1; i += 256) {
        const int id = a.ids[i];
        if ((unsigned)id < (unsigned)K) atomicAdd(&km_bins[id], 1);
        else bad = true;
    }
    if (bad) atomicOr(a.err_word, ERR_BAD_ID);
    __syncthreads();
    int *row = a.table + (int64_t)blockIdx.x * K;
    for (int k = threadIdx.x; k < K; k += 256) row[k] = km_bins[k];
}

// Exclusive prefix of table[.][k] along the chunks, for 64 centres per
// workgroup (lane = centre, each of the 16 waves takes a run of chunks);
// counts[k] = column total.
constexpr int KM_SCAN_WAVES = 16;
__global__ __launch_bounds__(64 * KM_SCAN_WAVES) void km_col_scan(KmeansArgs a)
{
    __shared__ int part[KM_SCAN_WAVES][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + lane;
    const bool valid = k < a.K;
    const int q = (a.n_chunks + KM_SCAN_WAVES - 1) / KM_SCAN_WAVES;
    const int c0 = min(wave * q, a.n_chunks), c1 = min(c0 + q, a.n_chunks);
    int *col = a.table + (valid ? k : 0);
    const int64_t K = a.K;
    int sum = 0;
    if (valid) {
        int c = c0;
        for (; c + 8 <= c1; c += 8) {   // eight independent loads in flight
            int v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = col[(c + u) * K];
#pragma unroll
            for (int u = 0; u < 8; ++u) sum += v[u];
        }
        for (; c < c1; ++c) sum += col[c * K];
    }
    part[wave][lane] = sum;
    __syncthreads();
    int run = 0, total = 0;
#pragma unroll
    for (int w = 0; w < KM_SCAN_WAVES; ++w) {
        if (w < wave) run += part[w][lane];
        total += part[w][lane];
    }
    if (valid) {
        int c = c0;
        for (; c + 8 <= c1; c += 8) {
            int v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = col[(c + u) * K];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                col[(c + u) * K] = run;
                run += v[u];
            }
        }
        for (; c < c1; ++c) {
            const int v = col[c * K];
            col[c * K] = run;
            run += v;
        }
        if (wave == 0) a.counts[k] = total;
    }
}

// seg_start[k] = first position of centre k's points in perm[]; pieces[] =
// {centre, first, one-past-last, 0} for every run of at most KM_PIECE points of
// one centre, pieces of a centre adjacent and in order; piece_start[k] = index
// of centre k's first piece.  One workgroup.
__global__ __launch_bounds__(1024) void km_segments(KmeansArgs a)
{
    __shared__ int s_cnt[1024], s_pcs[1024];
    const int tid = threadIdx.x;
    const int per = (a.K + 1023) / 1024;
    const int lo = min(tid * per, a.K), hi = min(lo + per, a.K);
    int cnt = 0, pcs = 0;
    for (int k = lo; k < hi; ++k) {
        const int c = a.counts[k];
        cnt += c;
        pcs += (c + KM_PIECE - 1) / KM_PIECE;
    }
    s_cnt[tid] = cnt;
    s_pcs[tid] = pcs;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        const int vc = (tid >= off) ? s_cnt[tid - off] : 0;
        const int vp = (tid >= off) ? s_pcs[tid - off] : 0;
        __syncthreads();
        s_cnt[tid] += vc;
        s_pcs[tid] += vp;
        __syncthreads();
    }
    int run_c = s_cnt[tid] - cnt, run_p = s_pcs[tid] - pcs;
    for (int k = lo; k < hi; ++k) {
        const int c = a.counts[k];
        a.seg_start[k] = run_c;
        a.piece_start[k] = run_p;
        for (int f = 0; f < c; f += KM_PIECE) a.pieces[run_p++] = make_int4(k, run_c + f, run_c + min(f + KM_PIECE, c), 0);
        run_c += c;
    }
    if (tid == 1023) {
        a.seg_start[a.K] = s_cnt[1023];
        a.piece_start[a.K] = s_pcs[1023];
        *a.n_pieces = s_pcs[1023];
    }
}

// One workgroup per chunk walks the chunk's points in order, 64 at a time.
// Lanes holding the same centre find each other with one ballot per id bit; the
// lowest of them reserves the group's positions in the chunk's private cursor
// table (in LDS), and each lane takes the slot of its rank inside the group.
// The matching (most of the instructions) runs on KM_SCATTER_WAVES batches at
// once, one per wave; the cursor updates then take turns in batch order, so
// ranks and cursors follow the point order and the sort is stable.
constexpr int KM_SCATTER_WAVES = 8;
__global__ __launch_bounds__(64 * KM_SCATTER_WAVES) void km_scatter(KmeansArgs a)
{
    extern __shared__ int km_pos[];
    constexpr int NT = 64 * KM_SCATTER_WAVES;
    static_assert(KM_MAX_K <= (1 << 15), "id bits matched per batch");
    const int K = a.K;
    const int *row = a.table + (int64_t)blockIdx.x * K;
    for (int k0 = threadIdx.x; k0 < K; k0 += NT * 4) {   // four independent loads per thread in flight
        int v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = k0 + u * NT;
            v[u] = (k < K) ? a.seg_start[k] + row[k] : 0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (k0 + u * NT < K) km_pos[k0 + u * NT] = v[u];
    }
    const int wave = uniform(threadIdx.x >> 6);
    const uint64_t lt = lanemask_lt();
    const int64_t i0 = (int64_t)blockIdx.x * a.chunk;
    const int64_t i1 = min(a.N, i0 + a.chunk);
    int64_t i = i0 + threadIdx.x;
    int nxt = (i < i1) ? a.ids[i] : -1;
    __syncthreads();
    for (int64_t b = i0; b < i1; b += NT) {   // uniform trip count for the whole workgroup
        i = b + threadIdx.x;
        const int id = nxt;
        nxt = (i + NT < i1) ? a.ids[i + NT] : -1;
        const bool ok = (unsigned)id < (unsigned)K;
        uint64_t m = __ballot(ok);
        // bits above log2(K) are zero in every valid id and cost nothing but their turn; a
        // fixed trip count lets all ballots issue before the first select
#pragma unroll
        for (int bit = 0; bit < 15; ++bit) {
            const bool one = (id >> bit) & 1;
            const uint64_t bal = __ballot(one);
            m &= one ? bal : ~bal;
        }
        const int rank = __popcll(m & lt);
        const int cnt = __popcll(m);
        const int leader = ok ? (__ffsll((unsigned long long)m) - 1) : 0;
        int base = 0;
#pragma unroll 1
        for (int turn = 0; turn < KM_SCATTER_WAVES; ++turn) {
            if (wave == turn && ok && rank == 0) {
                base = km_pos[id];
                km_pos[id] = base + cnt;
            }
            __syncthreads();
        }
        base = __shfl(base, leader);
        if (ok) a.perm[base + rank] = (int)i;
    }
}

// VPC values per 16-byte chunk: 8 (bf16) or 4 (fp32).
template <int VPC>
__device__ __forceinline__ void km_unpack(const uint4 &v, float (&f)[VPC])
{
    if constexpr (VPC == 8) {
        f[0] = bits_f32(v.x << 16); f[1] = bits_f32(v.x & 0xFFFF0000u);
        f[2] = bits_f32(v.y << 16); f[3] = bits_f32(v.y & 0xFFFF0000u);
        f[4] = bits_f32(v.z << 16); f[5] = bits_f32(v.z & 0xFFFF0000u);
        f[6] = bits_f32(v.w << 16); f[7] = bits_f32(v.w & 0xFFFF0000u);
    } else {
        f[0] = bits_f32(v.x); f[1] = bits_f32(v.y); f[2] = bits_f32(v.z); f[3] = bits_f32(v.w);
    }
}

// One piece (at most KM_PIECE points of one centre) and one block of up to 256
// 16-byte column chunks per workgroup.  With cw chunks in the block, 256 / cw
// rows are in flight per pass ("phases"); every thread owns one chunk of one
// phase and keeps fp32 column sums.  The squared distance to the old centre is
// summed per row in fp32 (VPC terms) and across rows in fp64.
template <int VPC>
__global__ __launch_bounds__(256) void km_segsum(KmeansArgs a)
{
    __shared__ float red[256 * VPC];
    __shared__ double dred[4];
    const int piece = blockIdx.x;
    if (piece >= uniform(*a.n_pieces)) return;
    const int4 rec = a.pieces[piece];
    const int k = uniform(rec.x), first = uniform(rec.y), last = uniform(rec.z);
    const int cpr = a.D / VPC;
    const int cb0 = blockIdx.y * 256;
    const int cw = min(256, cpr - cb0);
    const int rpp = 256 / cw;
    const int tid = threadIdx.x;
    const int phase = tid / cw, ch = cb0 + (tid - phase * cw);
    const bool active = phase < rpp;
    const int64_t row_bytes = (int64_t)a.D * (16 / VPC);
    const char *emb = static_cast<const char *>(a.emb) + (int64_t)ch * 16;

    float old[VPC], acc[VPC];
#pragma unroll
    for (int j = 0; j < VPC; ++j) acc[j] = 0.f;
    double dacc = 0.0;
    if (active) {
        km_unpack<VPC>(*reinterpret_cast<const uint4 *>(static_cast<const char *>(a.cent) + k * row_bytes + (int64_t)ch * 16), old);
        constexpr int UNR = 4;
        for (int row = first + phase; row < last; row += rpp * UNR) {
            int idx[UNR];
            uint4 v[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) idx[u] = (row + u * rpp < last) ? a.perm[row + u * rpp] : -1;
#pragma unroll
            for (int u = 0; u < UNR; ++u)
                if (idx[u] >= 0) v[u] = *reinterpret_cast<const uint4 *>(emb + idx[u] * row_bytes);
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                if (idx[u] < 0) continue;
                float f[VPC];
                km_unpack<VPC>(v[u], f);
                float d2 = 0.f;
#pragma unroll
                for (int j = 0; j < VPC; ++j) {
                    acc[j] += f[j];
                    const float d = f[j] - old[j];
                    d2 = fmaf(d, d, d2);
                }
                dacc += (double)d2;
            }
        }
    }
    // column sums: phases added in phase order by the phase-0 thread of each chunk
#pragma unroll
    for (int j = 0; j < VPC; ++j) red[j * 256 + tid] = acc[j];
    // objective: fixed butterfly inside the wave, then waves in order
    for (int off = 32; off > 0; off >>= 1) dacc += __shfl_xor(dacc, off);
    if ((tid & 63) == 0) dred[tid >> 6] = dacc;
    __syncthreads();
    if (phase == 0) {
        float *out = a.partial + (int64_t)piece * a.D + (int64_t)ch * VPC;
#pragma unroll
        for (int j = 0; j < VPC; ++j) {
            float s = acc[j];
            for (int p = 1; p < rpp; ++p) s += red[j * 256 + tid + p * cw];
            out[j] = s;
        }
    }
    if (tid == 0) a.inertia_part[(int64_t)piece * gridDim.y + blockIdx.y] = (dred[0] + dred[1]) + (dred[2] + dred[3]);
}

// new centre = (sum over the centre's pieces, fp64, in piece order) / count;
// a centre without points keeps its old value.  One thread per 4 columns.
// Workgroup 0 also adds up the objective.
__global__ __launch_bounds__(256) void km_finalize(KmeansArgs a)
{
    if (a.inertia && blockIdx.x == 0) {
        __shared__ double s[256];
        const int64_t n = (int64_t)(*a.n_pieces) * a.ncb;
        double t = 0.0;
        for (int64_t i = threadIdx.x; i < n; i += 256) t += a.inertia_part[i];
        s[threadIdx.x] = t;
        __syncthreads();
        for (int off = 128; off > 0; off >>= 1) {
            if ((int)threadIdx.x < off) s[threadIdx.x] += s[threadIdx.x + off];
            __syncthreads();
        }
        if (threadIdx.x == 0) *a.inertia = s[0];
    }
    if (!a.out) return;
    const int d4 = a.D >> 2;
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= (int64_t)a.K * d4) return;
    const int k = (int)(g / d4), j4 = (int)(g - (int64_t)k * d4);
    const int cnt = a.seg_start[k + 1] - a.seg_start[k];
    float v[4];
    if (cnt > 0) {
        double s[4] = {0.0, 0.0, 0.0, 0.0};
        for (int p = a.piece_start[k]; p < a.piece_start[k + 1]; ++p) {
            const f32x4_t q = *reinterpret_cast<const f32x4_t *>(a.partial + (int64_t)p * a.D + j4 * 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) s[j] += (double)q[j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (float)(s[j] / (double)cnt);
    } else if (a.is_bf16) {
        const uint2 o = *reinterpret_cast<const uint2 *>(static_cast<const char *>(a.cent) + ((int64_t)k * a.D + j4 * 4) * 2);
        v[0] = bits_f32(o.x << 16); v[1] = bits_f32(o.x & 0xFFFF0000u);
        v[2] = bits_f32(o.y << 16); v[3] = bits_f32(o.y & 0xFFFF0000u);
    } else {
        const f32x4_t o = *reinterpret_cast<const f32x4_t *>(static_cast<const char *>(a.cent) + ((int64_t)k * a.D + j4 * 4) * 4);
        v[0] = o[0]; v[1] = o[1]; v[2] = o[2]; v[3] = o[3];
    }
    if (a.out_bf16)
        *reinterpret_cast<uint2 *>(static_cast<char *>(a.out) + ((int64_t)k * a.D + j4 * 4) * 2) =
            make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
    else
        *reinterpret_cast<f32x4_t *>(static_cast<char *>(a.out) + ((int64_t)k * a.D + j4 * 4) * 4) = f32x4_t{v[0], v[1], v[2], v[3]};
}

// slot[k] = rank of centre k among the centres with counts[k] >= min_count
// (ascending k), or -1 for a dropped one; *n_retained = how many stay.
__global__ __launch_bounds__(1024) void km_retain(const int *counts, int K, int min_count, int *slot,
                                                  int *n_retained)
{
    __shared__ int s[1024];
    const int tid = threadIdx.x;
    const int per = (K + 1023) / 1024;
    const int lo = min(tid * per, K), hi = min(lo + per, K);
    int n = 0;
    for (int k = lo; k < hi; ++k) n += counts[k] >= min_count;
    s[tid] = n;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        const int v = (tid >= off) ? s[tid - off] : 0;
        __syncthreads();
        s[tid] += v;
        __syncthreads();
    }
    int run = s[tid] - n;
    for (int k = lo; k < hi; ++k) slot[k] = (counts[k] >= min_count) ? run++ : -1;
    if (tid == 1023 && n_retained) *n_retained = s[1023];
}

hipError_t prepare_kmeans_kernels()
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&km_chunk_hist),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, KM_MAX_K * 4);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&km_scatter),
                               hipFuncAttributeMaxDynamicSharedMemorySize, KM_MAX_K * 4);
}

void kmeans_shape(int64_t N, int K, int D, int is_bf16, int *chunk, int *n_chunks, int *max_pieces, int *ncb)
{
    int64_t c = 4096;
    if ((N + c - 1) / c > 1024) c = ((N + 1023) / 1024 + 63) / 64 * 64;
    *chunk = (int)c;
    *n_chunks = (int)((N + c - 1) / c);
    const int64_t nonempty = N < K ? N : K;
    *max_pieces = (int)(nonempty + N / KM_PIECE);
    const int cpr = D / (is_bf16 ? 8 : 4);
    *ncb = (cpr + 255) / 256;
}

// Steps 1-4: perm[] and the piece list.
hipError_t launch_kmeans_sort(const KmeansArgs &a, hipStream_t stream)
{
    const size_t lds = (size_t)a.K * 4;
    if (a.N > 0) hipLaunchKernelGGL(km_chunk_hist, dim3(a.n_chunks), dim3(256), lds, stream, a);
    hipLaunchKernelGGL(km_col_scan, dim3((a.K + 63) / 64), dim3(64 * KM_SCAN_WAVES), 0, stream, a);
    hipLaunchKernelGGL(km_segments, dim3(1), dim3(1024), 0, stream, a);
    if (a.N > 0) hipLaunchKernelGGL(km_scatter, dim3(a.n_chunks), dim3(64 * KM_SCATTER_WAVES), lds, stream, a);
    return hipGetLastError();
}

// Step 5: the pass over the embeddings.
hipError_t launch_kmeans_segsum(const KmeansArgs &a, hipStream_t stream)
{
    if (a.N <= 0 || a.max_pieces <= 0) return hipSuccess;
    const dim3 grid((unsigned)a.max_pieces, (unsigned)a.ncb);
    if (a.is_bf16) hipLaunchKernelGGL(km_segsum<8>, grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(km_segsum<4>, grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

// Step 6.
hipError_t launch_kmeans_finalize(const KmeansArgs &a, hipStream_t stream)
{
    const int64_t threads = a.out ? (int64_t)a.K * (a.D / 4) : 1;
    hipLaunchKernelGGL(km_finalize, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_kmeans_retain(const int *counts, int K, int min_count, int *slot, int *n_retained,
                                hipStream_t stream)
{
    hipLaunchKernelGGL(km_retain, dim3(1), dim3(1024), 0, stream, counts, K, min_count, slot, n_retained);
    return hipGetLastError();
}

}  // namespace moin
