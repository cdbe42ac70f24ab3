// C-ABI front end of libmoin: argument validation, workspace and plan
// management, kernel sequencing and optional per-kernel event timing.  All
// arithmetic of the method lives in the kernels; nothing here touches tensor
// data on the host.
#include "../../include/moin.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <new>
#include <vector>

#include "kernels.h"

namespace moin {
hipError_t prepare_linear_kernels();
hipError_t prepare_route_kernels();
hipError_t prepare_decode_kernels();
hipError_t prepare_kmeans_kernels();
hipError_t prepare_mx_kernels();
hipError_t prepare_kernels()
{
    hipError_t e = prepare_linear_kernels();
    if (e != hipSuccess) return e;
    if ((e = prepare_decode_kernels()) != hipSuccess) return e;
    if ((e = prepare_kmeans_kernels()) != hipSuccess) return e;
    if ((e = prepare_mx_kernels()) != hipSuccess) return e;
    return prepare_route_kernels();
}
}  // namespace moin

using namespace moin;

struct moin_plan {
    PlanView pv;
    void *buf;
    size_t bytes;
    int device;
    int built;
    // set once a call that uses the plan was recorded into a HIP graph: the graph holds
    // buf's address, so a later regrowth keeps the old block (until moin_plan_destroy)
    mutable int pinned;
    std::vector<void *> retired;
};

struct TimedSpan {
    hipEvent_t start, stop;
    int kernel;
};

struct moin_ctx {
    int device;
    int *err_word;
    void *ws;
    size_t ws_bytes;
    int ws_pinned;                  // a captured graph may hold ws's address (see moin_plan::pinned)
    std::vector<void *> ws_retired;
    // small routing batches: centroid norms, packed minima and the arrival counter in a block of their
    // own, which the kernel leaves clean for the next call; `route_key` says whose norms it holds
    void *route_buf;
    size_t route_bytes;
    int route_pinned;
    std::vector<void *> route_retired;
    struct {
        const void *cent, *slot;
        int K, D, dt, retained, valid;
    } route_key;
    moin_plan *own_plan;
    int act;   // activation between the adapter's two layers (MOIN_ACT_*)
    int timing;
    std::vector<TimedSpan> spans;
    std::vector<hipEvent_t> free_events;
    double ms_sum[MOIN_K_COUNT];
    int64_t launches[MOIN_K_COUNT];
};

// Device memory for moin_route_static, the entry point that may not allocate: one
// array per GPU the library is loaded on, held until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; the address the
// kernels get is looked up once per device (moin_create, with that device
// current) and kept in g_scratch_ptr.
constexpr int ROUTE_SELF_CLEAN_MAX_K = 65536;   // one workgroup zeroes the histogram in these calls
constexpr size_t SCRATCH_BYTES = 1u << 20;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void *g_scratch_ptr[MAX_DEVICES];

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }

struct DeviceGuard {
    int prev;
    bool ok;
    explicit DeviceGuard(int dev) : prev(-1), ok(false)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == dev) || (hipSetDevice(dev) == hipSuccess);
    }
    ~DeviceGuard()
    {
        int cur = -1;
        if (ok && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};

bool capturing(hipStream_t st)
{
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return cs == hipStreamCaptureStatusActive;
}

// Makes the context's workspace at least `bytes` large for a call on `st`.  While
// `st` is being captured nothing is (re)allocated: a call that needs more than the
// workspace holds fails with MOIN_ECAPTURE and records nothing.  A workspace that a
// captured call has used is never freed before moin_destroy -- a graph replays with
// the addresses it recorded -- so growing it later keeps the old block aside.
int ensure_ws(moin_ctx *ctx, size_t bytes, hipStream_t st, bool exact = false)
{
    const bool cap = capturing(st);
    if (bytes > ctx->ws_bytes) {
        if (cap) return MOIN_ECAPTURE;
        const size_t want = exact ? align_up(bytes, 256) : align_up(bytes + bytes / 4, 1 << 20);
        void *p = nullptr;
        if (hipMalloc(&p, want) != hipSuccess) {
            (void)hipGetLastError();
            return MOIN_ENOMEM;
        }
        if (ctx->ws) {
            if (ctx->ws_pinned) {
                ctx->ws_retired.push_back(ctx->ws);
            } else if (hipFree(ctx->ws) != hipSuccess) {   // waits for work that may still read the old block
                (void)hipFree(p);
                return MOIN_EHIP;
            }
        }
        ctx->ws = p;
        ctx->ws_bytes = want;
        ctx->ws_pinned = 0;
    }
    if (cap && bytes > 0) ctx->ws_pinned = 1;
    return MOIN_OK;
}

hipEvent_t take_event(moin_ctx *ctx)
{
    if (!ctx->free_events.empty()) {
        hipEvent_t e = ctx->free_events.back();
        ctx->free_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Runs `launch` (which enqueues exactly one kernel id's work) and, when timing
// is on, brackets it with events on the same stream.
template <typename F>
hipError_t timed(moin_ctx *ctx, int kernel, hipStream_t stream, F launch)
{
    if (!ctx->timing) return launch();
    TimedSpan s;
    s.kernel = kernel;
    s.start = take_event(ctx);
    s.stop = take_event(ctx);
    if (!s.start || !s.stop) return hipErrorOutOfMemory;
    hipError_t e = hipEventRecord(s.start, stream);
    if (e != hipSuccess) return e;
    e = launch();
    if (e != hipSuccess) return e;
    e = hipEventRecord(s.stop, stream);
    if (e != hipSuccess) return e;
    ctx->spans.push_back(s);
    return hipSuccess;
}

int drain_spans(moin_ctx *ctx)
{
    int rc = MOIN_OK;
    for (const TimedSpan &s : ctx->spans) {
        float ms = 0.f;
        if (hipEventSynchronize(s.stop) != hipSuccess ||
            hipEventElapsedTime(&ms, s.start, s.stop) != hipSuccess) {
            rc = MOIN_EHIP;
        } else {
            ctx->ms_sum[s.kernel] += ms;
            ctx->launches[s.kernel] += 1;
        }
        ctx->free_events.push_back(s.start);
        ctx->free_events.push_back(s.stop);
    }
    ctx->spans.clear();
    return rc;
}

struct PlanLayout {
    size_t tile_row0, tile_rows, tile_expert, tile_rank, n_tiles, tok_sorted, grp_meta,
        grp_start, grp_tmp, n_groups, keys, tmp, plain, total;
    int max_tiles, max_groups, max_plain, decode;
};

// upper_bound: sizes that hold the plan of ANY batch of at most S sequences and T tokens
// (every array at its larger variant), for moin_plan_reserve.
PlanLayout plan_layout(int32_t S, int64_t T, int32_t E, bool upper_bound = false)
{
    PlanLayout L;
    // one record per distinct expert (and one for "no adapter"), plus what cutting the
    // groups into chunks of GROUP_CHUNK tokens can add
    const int64_t groups = std::min<int64_t>(S, (int64_t)E + 1) + T / GROUP_CHUNK + 1;
    L.decode = upper_bound || ((T <= DECODE_MAX_T || T <= (int64_t)GATHER_MAX_AVG_LEN * S) && groups <= 65535);
    L.max_tiles = (int)(T / TILE_M) + S + 1;
    L.max_groups = L.decode ? (int)std::min<int64_t>(groups, 65535) : 0;
    size_t npow2 = 1;
    while (npow2 < (size_t)S) npow2 <<= 1;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    L.keys = take(npow2 * 8);
    L.tile_row0 = take((size_t)L.max_tiles * 4);
    L.tile_rows = take((size_t)L.max_tiles * 4);
    L.tile_expert = take((size_t)L.max_tiles * 4);
    L.tile_rank = take((size_t)L.max_tiles * 4);
    L.n_tiles = take(4);
    L.tok_sorted = take(L.decode ? (size_t)T * 4 : 4);
    L.grp_meta = take((size_t)(L.max_groups + 1) * 16);
    L.grp_start = take((size_t)(L.max_groups + 2) * 4);
    L.grp_tmp = take((size_t)(L.max_groups + 1) * 8);
    L.n_groups = take(4);
    L.tmp = take((size_t)4 * ((size_t)S + 1) * 4);
    L.max_plain = (L.decode && (T > DECODE_MAX_T || upper_bound)) ? (int)((T + TILE_M - 1) / TILE_M) : 0;
    L.plain = take(((size_t)4 * L.max_plain + 1) * 4);
    L.total = off;
    return L;
}

// The plan's buffer, at least `bytes` large; same rules under stream capture as ensure_ws.
int plan_grow(moin_plan *plan, size_t bytes, hipStream_t st)
{
    const bool cap = capturing(st);
    if (bytes > plan->bytes) {
        if (cap) return MOIN_ECAPTURE;
        void *p = nullptr;
        if (hipMalloc(&p, bytes) != hipSuccess) {
            (void)hipGetLastError();
            return MOIN_ENOMEM;
        }
        if (plan->buf) {
            if (plan->pinned) {
                plan->retired.push_back(plan->buf);
            } else if (hipFree(plan->buf) != hipSuccess) {
                (void)hipFree(p);
                return MOIN_EHIP;
            }
        }
        plan->buf = p;
        plan->bytes = bytes;
        plan->pinned = 0;
    }
    if (cap) plan->pinned = 1;
    return MOIN_OK;
}

// Sizes the plan's buffer for a batch and points the view's arrays into it; nothing is launched.
// Returns 1 when the batch is empty (the plan is then complete as it stands), 0 when the grouping
// has to run, a negative status on a fault.
static int plan_prepare(moin_plan *plan, const int32_t *seq_offsets, const int32_t *expert_ids, int32_t S,
                        int64_t T, int32_t E, hipStream_t stream)
{
    if (S < 0 || T < 0 || E < 0 || T > 0x7fffffffLL - TILE_M) return MOIN_EINVAL;
    plan->built = 0;
    plan->pv.S = S;
    plan->pv.T = T;
    plan->pv.E = E;
    if (S == 0 || T == 0) {
        // nothing to compute; a planned call returns at once
        plan->built = 1;
        return 1;
    }
    if (!seq_offsets || !expert_ids) return MOIN_EINVAL;
    const PlanLayout L = plan_layout(S, T, E);
    const int grc = plan_grow(plan, L.total, stream);
    if (grc != MOIN_OK) return grc;
    char *b = static_cast<char *>(plan->buf);
    PlanView &pv = plan->pv;
    pv.keys = reinterpret_cast<unsigned long long *>(b + L.keys);
    pv.tile_row0 = reinterpret_cast<int *>(b + L.tile_row0);
    pv.tile_rows = reinterpret_cast<int *>(b + L.tile_rows);
    pv.tile_expert = reinterpret_cast<int *>(b + L.tile_expert);
    pv.tile_rank = reinterpret_cast<int *>(b + L.tile_rank);
    pv.n_tiles = reinterpret_cast<int *>(b + L.n_tiles);
    pv.tok_sorted = reinterpret_cast<int *>(b + L.tok_sorted);
    pv.grp_meta = reinterpret_cast<int4 *>(b + L.grp_meta);
    pv.grp_start = reinterpret_cast<int *>(b + L.grp_start);
    pv.grp_tmp = reinterpret_cast<int2 *>(b + L.grp_tmp);
    pv.plain_row0 = reinterpret_cast<int *>(b + L.plain);
    pv.plain_rows = pv.plain_row0 + L.max_plain;
    pv.plain_expert = pv.plain_rows + L.max_plain;
    pv.plain_rank = pv.plain_expert + L.max_plain;
    pv.plain_n = pv.plain_rank + L.max_plain;
    pv.max_plain = L.max_plain;
    pv.n_groups = reinterpret_cast<int *>(b + L.n_groups);
    pv.tmp = reinterpret_cast<int *>(b + L.tmp);
    pv.max_tiles = L.max_tiles;
    pv.max_groups = L.max_groups;
    pv.decode = L.decode;
    return 0;
}

int plan_build_impl(moin_ctx *ctx, moin_plan *plan, const int32_t *seq_offsets,
                    const int32_t *expert_ids, int32_t S, int64_t T, int32_t E,
                    const int32_t *rank_of_expert, hipStream_t stream)
{
    const int prc = plan_prepare(plan, seq_offsets, expert_ids, S, T, E, stream);
    if (prc != 0) return prc < 0 ? prc : MOIN_OK;
    const PlanView &pv = plan->pv;
    const hipError_t e = timed(ctx, MOIN_K_PLAN, stream, [&] {
        return launch_plan(pv, seq_offsets, expert_ids, rank_of_expert, ctx->err_word, stream);
    });
    if (e != hipSuccess) return MOIN_EHIP;
    plan->built = 1;
    return MOIN_OK;
}

// Host-checkable faults of a linear call; nothing is launched when this fails.
int validate_linear(const void *x, const void *W, const void *A_stack, const void *B_stack,
                    int32_t E, int32_t d_in, int32_t d_out, int32_t r, float scale, const void *y,
                    moin_dtype y_dt)
{
    if (!x || !W || !y) return MOIN_EINVAL;
    if (d_in <= 0 || d_out <= 0 || r < 0 || E < 0) return MOIN_EINVAL;
    if (d_in % 8 || d_out % 8 || r % 8) return MOIN_EINVAL;
    if (d_in > (1 << 22) || d_out > (1 << 24) || r > (1 << 16)) return MOIN_EINVAL;
    if (y_dt != MOIN_BF16 && y_dt != MOIN_F32) return MOIN_EINVAL;
    if (misaligned(x, 16) || misaligned(W, 16) || misaligned(y, 16)) return MOIN_EINVAL;
    if (E > 0 && r > 0 &&
        (!A_stack || !B_stack || misaligned(A_stack, 16) || misaligned(B_stack, 16)))
        return MOIN_EINVAL;
    if (!(scale == scale)) return MOIN_EINVAL;
    return MOIN_OK;
}

int linear_planned_impl(moin_ctx *ctx, const moin_plan *plan, const void *x, const void *W,
                        const void *A_stack, const void *B_stack, int32_t d_in, int32_t d_out,
                        int32_t r, float scale, void *y, moin_dtype y_dt, hipStream_t stream)
{
    if (!plan->built) return MOIN_EINVAL;
    const PlanView &pv = plan->pv;
    if (pv.S == 0 || pv.T == 0) return MOIN_OK;
    const int vrc = validate_linear(x, W, A_stack, B_stack, pv.E, d_in, d_out, r, scale, y, y_dt);
    if (vrc != MOIN_OK) return vrc;
    if (capturing(stream)) plan->pinned = 1;
    const bool adapters = pv.E > 0 && r > 0;

    LinearArgs a;
    a.x = x; a.W = W; a.A_stack = A_stack; a.B_stack = B_stack;
    a.y = y; a.y_f32 = (y_dt == MOIN_F32);
    a.d_in = d_in; a.d_out = d_out; a.r = adapters ? r : 0; a.scale = scale; a.act = ctx->act;
    a.u_hi = a.u_lo = nullptr;

    const size_t u_bytes = align_up((size_t)pv.T * (size_t)a.r * 2, 256);
    if (!pv.decode) {
        if (a.r > 0) {
            const int rc = ensure_ws(ctx, 2 * u_bytes, stream);
            if (rc != MOIN_OK) return rc;
            a.u_hi = ctx->ws;
            a.u_lo = static_cast<char *>(ctx->ws) + u_bytes;
            if (timed(ctx, MOIN_K_SHRINK, stream, [&] { return launch_prefill_shrink(pv, a, stream); }) !=
                hipSuccess)
                return MOIN_EHIP;
        }
        if (timed(ctx, MOIN_K_LINEAR, stream, [&] { return launch_prefill_linear(pv, a, stream); }) !=
            hipSuccess)
            return MOIN_EHIP;
        return MOIN_OK;
    }

    // Beyond the small-batch size the base product runs on plain row tiles in the
    // prefill kernel (full 256-row tiles, no adapter), where its shapes allow.
    LinearArgs ab = a;
    ab.r = 0;
    const bool big = pv.max_plain > 0 && stream_kernel_fits(ab);
    PlanView pp = pv;
    pp.tile_row0 = pv.plain_row0; pp.tile_rows = pv.plain_rows; pp.tile_expert = pv.plain_expert;
    pp.tile_rank = pv.plain_rank; pp.n_tiles = pv.plain_n; pp.max_tiles = pv.max_plain;
    if (a.r == 0) {
        // no adapters anywhere in the call: the base GEMM writes y itself
        if (big) {
            if (timed(ctx, MOIN_K_LINEAR, stream, [&] { return launch_prefill_linear(pp, ab, stream); }) != hipSuccess)
                return MOIN_EHIP;
        } else if (timed(ctx, MOIN_K_DECODE_BASE, stream, [&] { return launch_decode_base_only(pv, a, stream); }) !=
                   hipSuccess)
            return MOIN_EHIP;
        return MOIN_OK;
    }
    DecodeArgs d;
    d.lin = a;
    d.k_splits = big ? 1 : decode_base_splits(pv.T, d_in, d_out);
    const size_t yb_bytes = align_up((size_t)d.k_splits * (size_t)pv.T * (size_t)d_out * 4, 256);
    const int rc = ensure_ws(ctx, 2 * u_bytes + yb_bytes, stream);
    if (rc != MOIN_OK) return rc;
    char *w = static_cast<char *>(ctx->ws);
    d.ug_hi = w;
    d.ug_lo = w + u_bytes;
    d.ybase = reinterpret_cast<float *>(w + 2 * u_bytes);
    d.ybase_by_pos = big ? 0 : 1;   // the small-batch base product gathers its rows in the plan's order
    if (big) {
        ab.y = d.ybase;
        ab.y_f32 = 1;
        if (timed(ctx, MOIN_K_LINEAR, stream, [&] { return launch_prefill_linear(pp, ab, stream); }) != hipSuccess)
            return MOIN_EHIP;
        if (timed(ctx, MOIN_K_DECODE_SHRINK, stream, [&] { return launch_decode_shrink(pv, d, stream); }) !=
            hipSuccess)
            return MOIN_EHIP;
    } else if (decode_base_shrink_fits(pv, d)) {
        if (timed(ctx, MOIN_K_DECODE_SHRINK, stream, [&] { return launch_decode_base_shrink(pv, d, stream); }) !=
            hipSuccess)
            return MOIN_EHIP;
    } else {
        if (timed(ctx, MOIN_K_DECODE_BASE, stream, [&] { return launch_decode_base(pv, d, stream); }) !=
            hipSuccess)
            return MOIN_EHIP;
        if (timed(ctx, MOIN_K_DECODE_SHRINK, stream, [&] { return launch_decode_shrink(pv, d, stream); }) !=
            hipSuccess)
            return MOIN_EHIP;
    }
    if (timed(ctx, MOIN_K_DECODE_EXPAND, stream, [&] { return launch_decode_expand(pv, d, stream); }) !=
        hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

// Quantised-base variant of the prefill sequence: shrink on the bf16 x, x
// through the quantiser, then the block-scaled main kernel.
// xq / xs: the activations already quantised (blocked scale layout), or both null:
// then they are quantised here, into the workspace.
int linear_mx_planned_impl(moin_ctx *ctx, const moin_plan *plan, const void *x, void *xq,
                           void *xs, bool x_given, const void *Wq, const void *Ws, const void *A_stack,
                           const void *B_stack, int32_t d_in, int32_t d_out, int32_t r, float scale,
                           void *y, moin_dtype y_dt, hipStream_t stream)
{
    if (!plan->built) return MOIN_EINVAL;
    const PlanView &pv = plan->pv;
    if (pv.S == 0 || pv.T == 0) return MOIN_OK;
    if (capturing(stream)) plan->pinned = 1;
    const bool adapters = pv.E > 0 && r > 0;
    MxLinearArgs m;
    LinearArgs &a = m.lin;
    a.x = x; a.W = nullptr; a.A_stack = A_stack; a.B_stack = B_stack;
    a.y = y; a.y_f32 = (y_dt == MOIN_F32);
    a.d_in = d_in; a.d_out = d_out; a.r = adapters ? r : 0; a.scale = scale; a.act = ctx->act;
    a.u_hi = a.u_lo = nullptr;
    const size_t u_bytes = align_up((size_t)pv.T * (size_t)a.r * 2, 256);
    const bool ws_q = xq == nullptr;      // codes and scales live in the workspace
    const bool own_q = !x_given;          // this call quantises x
    const size_t xq_bytes = ws_q ? align_up((size_t)pv.T * (size_t)d_in, 256) : 0;
    const size_t xs_bytes = ws_q ? align_up((size_t)pv.T * (size_t)(d_in / 32), 256) : 0;
    m.plain_splits = 0;
    m.plain_kb_per_split = 0;
    // decode-sized batches with adapters: the base product for all tokens at once as
    // fp32 partial planes, then the decode path's own shrink and expand kernels
    const bool decode = pv.decode && a.r > 0;
    size_t yb_bytes = 0;
    if (decode) {
        mx_plain_shape(pv.T, d_in, d_out, &m.plain_splits, &m.plain_kb_per_split);
        yb_bytes = align_up((size_t)m.plain_splits * (size_t)pv.T * (size_t)d_out * 4, 256);
    } else if (pv.decode) {
        m.plain_splits = 1;            // no adapters anywhere: the plain product writes y itself
        m.plain_kb_per_split = d_in / 128;
    }
    const int rc = ensure_ws(ctx, 2 * u_bytes + xq_bytes + xs_bytes + yb_bytes, stream);
    if (rc != MOIN_OK) return rc;
    char *w = static_cast<char *>(ctx->ws);
    a.u_hi = w;
    a.u_lo = w + u_bytes;
    m.xq = ws_q ? w + 2 * u_bytes : xq;
    m.xs = ws_q ? w + 2 * u_bytes + xq_bytes : xs;
    m.Wq = Wq;
    m.Ws = Ws;
    // prefill with adapters: the shrink's pass over x writes the codes and scales as well
    const bool fused_q = own_q && !pv.decode && a.r > 0;
    if (own_q && !fused_q && timed(ctx, MOIN_K_MX_QUANT, stream, [&] {
            return launch_mx_quantize(x, pv.T, d_in, const_cast<void *>(m.xq), const_cast<void *>(m.xs), 1, stream);
        }) != hipSuccess)
        return MOIN_EHIP;
    if (decode) {
        DecodeArgs d;
        d.lin = a;
        d.ug_hi = a.u_hi;
        d.ug_lo = a.u_lo;
        d.ybase = reinterpret_cast<float *>(w + 2 * u_bytes + xq_bytes + xs_bytes);
        d.k_splits = m.plain_splits;
        m.lin.y = d.ybase;
        m.lin.y_f32 = 1;
        if (timed(ctx, MOIN_K_MX_LINEAR, stream, [&] {
                return launch_linear_mx_stream(pv, m, compute_units(), stream);
            }) != hipSuccess)
            return MOIN_EHIP;
        if (timed(ctx, MOIN_K_DECODE_SHRINK, stream, [&] { return launch_decode_shrink(pv, d, stream); }) !=
            hipSuccess)
            return MOIN_EHIP;
        if (timed(ctx, MOIN_K_DECODE_EXPAND, stream, [&] { return launch_decode_expand(pv, d, stream); }) !=
            hipSuccess)
            return MOIN_EHIP;
        return MOIN_OK;
    }
    if (a.r > 0 && !pv.decode && timed(ctx, MOIN_K_SHRINK, stream, [&] {
            return fused_q ? launch_prefill_shrink_quant(pv, a, const_cast<void *>(m.xq),
                                                         const_cast<void *>(m.xs), stream)
                           : launch_prefill_shrink(pv, a, stream);
        }) != hipSuccess)
        return MOIN_EHIP;
    if (timed(ctx, MOIN_K_MX_LINEAR, stream, [&] {
            return launch_linear_mx_stream(pv, m, compute_units(), stream);
        }) != hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

}  // namespace

extern "C" {

int moin_create(moin_ctx **out, int device)
{
    if (!out || device < 0) return MOIN_EINVAL;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess) {
        (void)hipGetLastError();
        return MOIN_EHIP;
    }
    if (device >= n) return MOIN_EINVAL;
    DeviceGuard guard(device);
    if (!guard.ok) return MOIN_EHIP;
    moin_ctx *ctx = new (std::nothrow) moin_ctx();
    if (!ctx) return MOIN_ENOMEM;
    ctx->device = device;
    ctx->err_word = nullptr;
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
    ctx->ws_pinned = 0;
    ctx->route_buf = nullptr;
    ctx->route_bytes = 0;
    ctx->route_pinned = 0;
    ctx->route_key.valid = 0;
    ctx->own_plan = nullptr;
    ctx->act = MOIN_ACT_NONE;
    ctx->timing = 0;
    for (int i = 0; i < MOIN_K_COUNT; ++i) {
        ctx->ms_sum[i] = 0.0;
        ctx->launches[i] = 0;
    }
    if (prepare_kernels() != hipSuccess) {
        delete ctx;
        return MOIN_EHIP;
    }
    if (device < MAX_DEVICES && !g_scratch_ptr[device]) {
        // this device's copy of the static scratch array (the guard above made it current)
        void *sp = nullptr;
        if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || !sp) {
            (void)hipGetLastError();
            delete ctx;
            return MOIN_EHIP;
        }
        g_scratch_ptr[device] = sp;
    }
    if (hipMalloc(reinterpret_cast<void **>(&ctx->err_word), 256) != hipSuccess) {
        (void)hipGetLastError();
        delete ctx;
        return MOIN_ENOMEM;
    }
    if (hipMemset(ctx->err_word, 0, 256) != hipSuccess) {
        (void)hipFree(ctx->err_word);
        delete ctx;
        return MOIN_EHIP;
    }
    *out = ctx;
    return MOIN_OK;
}

void moin_destroy(moin_ctx *ctx)
{
    if (!ctx) return;
    DeviceGuard guard(ctx->device);
    (void)drain_spans(ctx);
    for (hipEvent_t e : ctx->free_events) (void)hipEventDestroy(e);
    if (ctx->own_plan) moin_plan_destroy(ctx->own_plan);
    if (ctx->ws) (void)hipFree(ctx->ws);
    for (void *p : ctx->ws_retired) (void)hipFree(p);
    if (ctx->route_buf) (void)hipFree(ctx->route_buf);
    for (void *p : ctx->route_retired) (void)hipFree(p);
    if (ctx->err_word) (void)hipFree(ctx->err_word);
    delete ctx;
}

const char *moin_strerror(int code)
{
    switch (code) {
    case MOIN_OK: return "success";
    case MOIN_EINVAL: return "invalid argument (null pointer, bad size, unsupported shape or alignment)";
    case MOIN_ENOMEM: return "workspace allocation failed";
    case MOIN_EHIP: return "HIP runtime call failed";
    case MOIN_EDATA: return "device-side data fault (expert id or rank out of range, bad offsets or ids)";
    case MOIN_ETOOBIG: return "size beyond the fixed limit of an entry point that does not allocate";
    case MOIN_ECAPTURE: return "the call would have to reallocate its workspace while the stream is being captured";
    default: return "unknown moin status";
    }
}

int moin_check(moin_ctx *ctx, void *stream)
{
    if (!ctx) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int word = 0;
    if (hipMemcpyAsync(&word, ctx->err_word, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess)
        return MOIN_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return MOIN_EHIP;
    if (word != 0) {
        if (hipMemsetAsync(ctx->err_word, 0, sizeof(int), st) != hipSuccess) return MOIN_EHIP;
        if (hipStreamSynchronize(st) != hipSuccess) return MOIN_EHIP;
        return MOIN_EDATA;
    }
    return MOIN_OK;
}

// Host-checkable faults of a routing call.
static int validate_route(moin_ctx *ctx, const void *emb, const void *centroids, int64_t N, int32_t K,
                          int32_t D, moin_dtype dt, const int32_t *slot_of_centroid, uint32_t flags)
{
    if (!ctx || N < 0 || K <= 0 || D <= 0) return MOIN_EINVAL;
    if (dt != MOIN_BF16 && dt != MOIN_F32) return MOIN_EINVAL;
    if (flags & ~(MOIN_ROUTE_RETAINED_ONLY | MOIN_ROUTE_SAME_CENTROIDS)) return MOIN_EINVAL;
    if ((flags & MOIN_ROUTE_RETAINED_ONLY) && !slot_of_centroid) return MOIN_EINVAL;
    if (!centroids) return MOIN_EINVAL;
    if (N > 0 && !emb) return MOIN_EINVAL;
    if (dt == MOIN_BF16 ? (D % 8 != 0) : (D % 4 != 0)) return MOIN_EINVAL;
    if (D > (1 << 20) || K > (1 << 28)) return MOIN_EINVAL;
    if (misaligned(centroids, 16) || (emb && misaligned(emb, 16))) return MOIN_EINVAL;
    return MOIN_OK;
}

// A grouping that rides in the routing launch (request-sized batches only).
struct RoutePlanFuse {
    const PlanView *pv;
    const int32_t *seq_offsets, *rank_of_expert;
};

// Where a routing call keeps its intermediate results inside a block of device memory.
struct RouteScratch {
    size_t cnorm, cinit, best, arrivals, cid, total;
    int group;
};

static RouteScratch route_scratch(int64_t N, int32_t K, int32_t D, moin_dtype dt, bool need_cid)
{
    RouteScratch L;
    const size_t Kpad = align_up((size_t)K, 256);
    const size_t cn_bytes = align_up(Kpad * 4, 256);
    L.group = route_stream_group(N, K, D, dt == MOIN_BF16);
    const size_t n_best = L.group > 1 ? (size_t)N : (size_t)ROUTE_SMALL_MAX_N;
    L.cnorm = 0;
    L.cinit = cn_bytes;
    L.best = 2 * cn_bytes;
    L.arrivals = L.best + align_up(n_best * 8, 256);
    L.cid = L.arrivals + 256;
    L.total = L.cid + (need_cid ? align_up((size_t)N * 4, 256) : 0);
    return L;
}

// The launches of a routing call; `w` holds L.total bytes.  With `record` off the
// launches are not bracketed by timing events (the caller must not allocate).
static int route_launches(moin_ctx *ctx, const void *emb, const void *centroids, int64_t N, int32_t K,
                          int32_t D, moin_dtype dt, const int32_t *slot_of_centroid, uint32_t flags,
                          int32_t *expert_ids, int32_t *centroid_ids, int32_t *counts, char *w,
                          const RouteScratch &L, bool need_cid, bool record, hipStream_t st, int self_clean = 0,
                          const RoutePlanFuse *fuse = nullptr)
{
    RouteArgs a;
    a.emb = emb; a.cent = centroids; a.N = N; a.K = K; a.D = D;
    a.is_bf16 = (dt == MOIN_BF16);
    a.slot = slot_of_centroid;
    a.retained_only = (flags & MOIN_ROUTE_RETAINED_ONLY) ? 1 : 0;
    a.group = L.group;
    a.cnorm = reinterpret_cast<float *>(w + L.cnorm);
    a.cinit = reinterpret_cast<float *>(w + L.cinit);
    a.best = reinterpret_cast<unsigned long long *>(w + L.best);
    a.arrivals = reinterpret_cast<int *>(w + L.arrivals);
    a.cid = centroid_ids ? centroid_ids : (need_cid ? reinterpret_cast<int *>(w + L.cid) : nullptr);
    a.expert_ids = expert_ids;
    a.counts = counts;
    a.self_clean = self_clean ? 1 : 0;   // 1: norms kernel + self-cleaning kernel, 2: the norms in w are current
    if (fuse) {
        a.plan = fuse->pv;
        a.seq_offsets = fuse->seq_offsets;
        a.rank_of_expert = fuse->rank_of_expert;
        a.err_word = ctx->err_word;
    }

    auto run = [&](int kernel, auto launch) {
        return record ? timed(ctx, kernel, st, launch) : launch();
    };
    const bool routed = N > 0 && (a.cid || a.expert_ids);
    if (routed) {
        if (self_clean != 2 &&
            run(MOIN_K_ROUTE_AUX, [&] { return launch_centroid_norms(a, st); }) != hipSuccess)
            return MOIN_EHIP;
        if (run(MOIN_K_ROUTE, [&] { return launch_route(a, st); }) != hipSuccess) return MOIN_EHIP;
    }
    if (counts && !(routed && route_tallies_counts(a))) {
        // the norms kernel, when it ran, has already zeroed counts
        if (run(MOIN_K_ROUTE_AUX, [&] {
                return launch_histogram(a.cid, N, K, counts, routed ? 0 : 1, ctx->err_word, st);
            }) != hipSuccess)
            return MOIN_EHIP;
    }
    return MOIN_OK;
}

int moin_reserve_workspace(moin_ctx *ctx, int64_t bytes, void *stream)
{
    if (!ctx || bytes < 0) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    return ensure_ws(ctx, (size_t)bytes, static_cast<hipStream_t>(stream), true);
}

int64_t moin_workspace_bytes(const moin_ctx *ctx) { return ctx ? (int64_t)ctx->ws_bytes : 0; }

int moin_plan_reserve(moin_ctx *ctx, moin_plan *plan, int32_t S, int64_t T, int32_t E, void *stream)
{
    if (!ctx || !plan || plan->device != ctx->device) return MOIN_EINVAL;
    if (S < 0 || T < 0 || E < 0 || T > 0x7fffffffLL - TILE_M) return MOIN_EINVAL;
    if (S == 0 || T == 0) return MOIN_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    // a plan holds either kind of batch of up to this size: the larger of the two layouts
    const size_t need = plan_layout(S, T, E, true).total;
    return plan_grow(plan, need, static_cast<hipStream_t>(stream));
}

// True when route_impl would take the single self-cleaning launch for this call.
static bool route_one_launch(int64_t N, int32_t K, int32_t D, moin_dtype dt, const int32_t *expert_ids,
                             const int32_t *centroid_ids)
{
    return N > 0 && (expert_ids || centroid_ids) && K <= ROUTE_SELF_CLEAN_MAX_K &&
           route_small_batch(N, K, D, dt == MOIN_BF16);
}

// moin_route after validation, with the device current.  `fuse` (only with route_one_launch() true):
// the launch goes on to group the batch by the ids it has just written.
static int route_impl(moin_ctx *ctx, const void *emb, const void *centroids, int64_t N, int32_t K,
                      int32_t D, moin_dtype dt, const int32_t *slot_of_centroid, uint32_t flags,
                      int32_t *expert_ids, int32_t *centroid_ids, int32_t *counts, hipStream_t st,
                      const RoutePlanFuse *fuse)
{
    const bool need_cid = counts && !centroid_ids && N > 0;
    RouteScratch L = route_scratch(N, K, D, dt, need_cid);
    if (route_one_launch(N, K, D, dt, expert_ids, centroid_ids)) {
        // (minima and counter first, at offsets that do not move with K: they must stay clean)
        const size_t cn_bytes = L.cinit - L.cnorm;
        L.best = 0;
        L.arrivals = (size_t)ROUTE_SMALL_MAX_N * 8;
        L.cnorm = L.arrivals + 256;
        L.cinit = L.cnorm + cn_bytes;
        L.cid = L.cinit + cn_bytes;
        L.total = L.cid + (need_cid ? align_up((size_t)N * 4, 256) : 0);
        // Request-sized batches: one launch.  Norms, packed minima and the arrival counter live in a
        // block of the context's own (the shared workspace is overwritten by the linear calls in
        // between); the kernel's finishing workgroup leaves minima and counter clean and zeroes the
        // histogram itself, and the norms are computed again only if the caller does not vouch for the
        // table (or it is not the table they were computed from).
        const bool cap = capturing(st);
        if (L.total > ctx->route_bytes) {
            if (cap) return MOIN_ECAPTURE;
            void *p = nullptr;
            const size_t want = align_up(L.total, 4096);
            if (hipMalloc(&p, want) != hipSuccess) {
                (void)hipGetLastError();
                return MOIN_ENOMEM;
            }
            if (ctx->route_buf) {
                if (ctx->route_pinned) ctx->route_retired.push_back(ctx->route_buf);
                else if (hipFree(ctx->route_buf) != hipSuccess) {
                    (void)hipFree(p);
                    return MOIN_EHIP;
                }
            }
            ctx->route_buf = p;
            ctx->route_bytes = want;
            ctx->route_pinned = 0;
            ctx->route_key.valid = 0;
            // minima at "nothing won yet", counter at zero (the kernels keep them so from here on)
            char *b = static_cast<char *>(p);
            if (hipMemsetAsync(b + L.best, 0xFF, L.arrivals - L.best, st) != hipSuccess ||
                hipMemsetAsync(b + L.arrivals, 0, 256, st) != hipSuccess)
                return MOIN_EHIP;
        }
        if (cap) ctx->route_pinned = 1;
        const int retained = (flags & MOIN_ROUTE_RETAINED_ONLY) ? 1 : 0;
        const bool same = ctx->route_key.valid && ctx->route_key.cent == centroids &&
                          ctx->route_key.slot == (retained ? slot_of_centroid : nullptr) && ctx->route_key.K == K &&
                          ctx->route_key.D == D && ctx->route_key.dt == (int)dt && ctx->route_key.retained == retained;
        const bool reuse = (flags & MOIN_ROUTE_SAME_CENTROIDS) && same;
        ctx->route_key.cent = centroids;
        ctx->route_key.slot = retained ? slot_of_centroid : nullptr;
        ctx->route_key.K = K; ctx->route_key.D = D; ctx->route_key.dt = (int)dt;
        ctx->route_key.retained = retained; ctx->route_key.valid = 1;
        return route_launches(ctx, emb, centroids, N, K, D, dt, slot_of_centroid, flags, expert_ids,
                              centroid_ids, counts, static_cast<char *>(ctx->route_buf), L, need_cid, true, st,
                              reuse ? 2 : 1, fuse);
    }
    if (fuse) return MOIN_EINVAL;   // (the caller asks for it only where it applies)
    const int rc = ensure_ws(ctx, L.total, st);
    if (rc != MOIN_OK) return rc;
    return route_launches(ctx, emb, centroids, N, K, D, dt, slot_of_centroid, flags, expert_ids,
                          centroid_ids, counts, static_cast<char *>(ctx->ws), L, need_cid, true, st);
}

int moin_route(moin_ctx *ctx, const void *emb, const void *centroids, int64_t N, int32_t K,
               int32_t D, moin_dtype dt, const int32_t *slot_of_centroid, uint32_t flags,
               int32_t *expert_ids, int32_t *centroid_ids, int32_t *counts, void *stream)
{
    const int vrc = validate_route(ctx, emb, centroids, N, K, D, dt, slot_of_centroid, flags);
    if (vrc != MOIN_OK) return vrc;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    return route_impl(ctx, emb, centroids, N, K, D, dt, slot_of_centroid, flags, expert_ids, centroid_ids,
                      counts, static_cast<hipStream_t>(stream), nullptr);
}

int moin_route_plan(moin_ctx *ctx, moin_plan *plan, const void *emb, const void *centroids, int64_t N,
                    int32_t K, int32_t D, moin_dtype dt, const int32_t *slot_of_centroid, uint32_t flags,
                    const int32_t *seq_offsets, int64_t T, int32_t E, const int32_t *rank_of_expert,
                    int32_t *expert_ids, int32_t *centroid_ids, int32_t *counts, void *stream)
{
    const int vrc = validate_route(ctx, emb, centroids, N, K, D, dt, slot_of_centroid, flags);
    if (vrc != MOIN_OK) return vrc;
    if (!plan || plan->device != ctx->device || (N > 0 && !expert_ids) || N > 0x7fffffffLL) return MOIN_EINVAL;
    // ids are adapter slots when a map is given, centroid indices otherwise: E must cover them
    if (!slot_of_centroid && E < K) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t S = (int32_t)N;
    if (S <= ROUTE_PLAN_FUSED_MAX_S && T > 0 && route_one_launch(N, K, D, dt, expert_ids, centroid_ids)) {
        const int prc = plan_prepare(plan, seq_offsets, expert_ids, S, T, E, st);
        if (prc < 0) return prc;
        const RoutePlanFuse fuse{&plan->pv, seq_offsets, rank_of_expert};
        const int rc = route_impl(ctx, emb, centroids, N, K, D, dt, slot_of_centroid, flags, expert_ids,
                                  centroid_ids, counts, st, &fuse);
        if (rc == MOIN_OK) plan->built = 1;
        return rc;
    }
    const int rc = route_impl(ctx, emb, centroids, N, K, D, dt, slot_of_centroid, flags, expert_ids,
                              centroid_ids, counts, st, nullptr);
    if (rc != MOIN_OK) return rc;
    return plan_build_impl(ctx, plan, seq_offsets, expert_ids, S, T, E, rank_of_expert, st);
}

int moin_route_static(moin_ctx *ctx, const void *emb, const void *centroids, int64_t N, int32_t K,
                      int32_t D, moin_dtype dt, const int32_t *slot_of_centroid, uint32_t flags,
                      int32_t *expert_ids, int32_t *centroid_ids, int32_t *counts, void *stream)
{
    const int vrc = validate_route(ctx, emb, centroids, N, K, D, dt, slot_of_centroid, flags);
    if (vrc != MOIN_OK) return vrc;
    if (N > MOIN_ROUTE_STATIC_MAX_N || K > MOIN_ROUTE_STATIC_MAX_K) return MOIN_ETOOBIG;
    if (ctx->device < 0 || ctx->device >= MAX_DEVICES || !g_scratch_ptr[ctx->device]) return MOIN_EHIP;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool need_cid = counts && !centroid_ids && N > 0;
    const RouteScratch L = route_scratch(N, K, D, dt, need_cid);
    if (L.total > SCRATCH_BYTES) return MOIN_ETOOBIG;   // cannot happen within the two limits above
    return route_launches(ctx, emb, centroids, N, K, D, dt, slot_of_centroid, flags, expert_ids,
                          centroid_ids, counts, static_cast<char *>(g_scratch_ptr[ctx->device]), L, need_cid,
                          false, st);
}

int moin_histogram(moin_ctx *ctx, const int32_t *ids, int64_t N, int32_t K, int32_t *counts,
                   void *stream)
{
    if (!ctx || N < 0 || K <= 0 || !counts) return MOIN_EINVAL;
    if (N > 0 && !ids) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (timed(ctx, MOIN_K_ROUTE_AUX, st, [&] {
            return launch_histogram(ids, N, K, counts, 1, ctx->err_word, st);
        }) != hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

int moin_plan_create(moin_ctx *ctx, moin_plan **out)
{
    if (!ctx || !out) return MOIN_EINVAL;
    moin_plan *p = new (std::nothrow) moin_plan();
    if (!p) return MOIN_ENOMEM;
    p->buf = nullptr;
    p->bytes = 0;
    p->device = ctx->device;
    p->built = 0;
    p->pinned = 0;
    *out = p;
    return MOIN_OK;
}

void moin_plan_destroy(moin_plan *plan)
{
    if (!plan) return;
    DeviceGuard guard(plan->device);
    if (plan->buf) (void)hipFree(plan->buf);
    for (void *p : plan->retired) (void)hipFree(p);
    delete plan;
}

int moin_plan_build_ranked(moin_ctx *ctx, moin_plan *plan, const int32_t *seq_offsets,
                           const int32_t *expert_ids, int32_t S, int64_t T, int32_t E,
                           const int32_t *rank_of_expert, void *stream)
{
    if (!ctx || !plan || plan->device != ctx->device) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    return plan_build_impl(ctx, plan, seq_offsets, expert_ids, S, T, E, rank_of_expert,
                           static_cast<hipStream_t>(stream));
}

int moin_plan_build(moin_ctx *ctx, moin_plan *plan, const int32_t *seq_offsets,
                    const int32_t *expert_ids, int32_t S, int64_t T, int32_t E, void *stream)
{
    return moin_plan_build_ranked(ctx, plan, seq_offsets, expert_ids, S, T, E, nullptr, stream);
}

int moin_lora_linear_planned(moin_ctx *ctx, const moin_plan *plan, const void *x, const void *W,
                             const void *A_stack, const void *B_stack, int32_t d_in, int32_t d_out,
                             int32_t r, float scale, void *y, moin_dtype y_dt, void *stream)
{
    if (!ctx || !plan || plan->device != ctx->device) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    return linear_planned_impl(ctx, plan, x, W, A_stack, B_stack, d_in, d_out, r, scale, y, y_dt,
                               static_cast<hipStream_t>(stream));
}

int moin_lora_linear_planned_shared(moin_ctx *ctx, const moin_plan *plan, const void *x, int32_t n,
                                    const void *const *W, const void *const *A_stack,
                                    const void *const *B_stack, int32_t d_in, const int32_t *d_out, int32_t r,
                                    float scale, void *const *y, moin_dtype y_dt, void *stream)
{
    if (!ctx || !plan || plan->device != ctx->device) return MOIN_EINVAL;
    if (n < 1 || n > MAX_SHARED_X || !W || !d_out || !y) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    if (!plan->built) return MOIN_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const PlanView &pv = plan->pv;
    if (pv.S == 0 || pv.T == 0) return MOIN_OK;
    if (capturing(st)) plan->pinned = 1;
    const bool adapters = pv.E > 0 && r > 0;
    if (adapters && (!A_stack || !B_stack)) return MOIN_EINVAL;
    for (int i = 0; i < n; ++i) {
        const int vrc = validate_linear(x, W[i], adapters ? A_stack[i] : nullptr, adapters ? B_stack[i] : nullptr,
                                        pv.E, d_in, d_out[i], r, scale, y[i], y_dt);
        if (vrc != MOIN_OK) return vrc;
    }
    if (pv.decode && adapters && n > 1 && pv.max_plain == 0) {
        // Decode-sized batch: the projections' base tiles and shrink slabs in one launch, their expand
        // blocks in another, where they agree in everything those launches share.
        DecodeArgs d[MAX_SHARED_X];
        size_t off[MAX_SHARED_X], total = 0;
        const size_t u_bytes = align_up((size_t)pv.T * (size_t)r * 2, 256);
        for (int i = 0; i < n; ++i) {
            LinearArgs &a = d[i].lin;
            a.x = x; a.W = W[i]; a.A_stack = A_stack[i]; a.B_stack = B_stack[i];
            a.y = y[i]; a.y_f32 = (y_dt == MOIN_F32);
            a.d_in = d_in; a.d_out = d_out[i]; a.r = r; a.scale = scale; a.act = ctx->act;
            a.u_hi = a.u_lo = nullptr;
            d[i].k_splits = decode_base_splits(pv.T, d_in, d_out[i]);
            d[i].ybase_by_pos = 1;
            off[i] = total;
            total += 2 * u_bytes + align_up((size_t)d[i].k_splits * (size_t)pv.T * (size_t)d_out[i] * 4, 256);
        }
        if (decode_shared_fits(pv, d, n)) {
            const int rc = ensure_ws(ctx, total, st);
            if (rc != MOIN_OK) return rc;
            for (int i = 0; i < n; ++i) {
                char *w = static_cast<char *>(ctx->ws) + off[i];
                d[i].ug_hi = w;
                d[i].ug_lo = w + u_bytes;
                d[i].ybase = reinterpret_cast<float *>(w + 2 * u_bytes);
            }
            if (timed(ctx, MOIN_K_DECODE_SHRINK, st, [&] { return launch_decode_base_shrink_shared(pv, d, n, st); }) !=
                hipSuccess)
                return MOIN_EHIP;
            if (timed(ctx, MOIN_K_DECODE_EXPAND, st, [&] { return launch_decode_expand_shared(pv, d, n, st); }) !=
                hipSuccess)
                return MOIN_EHIP;
            return MOIN_OK;
        }
    }
    if (pv.decode || !adapters || n == 1) {
        // nothing to share on these paths: the projections one after the other
        for (int i = 0; i < n; ++i) {
            const int rc = linear_planned_impl(ctx, plan, x, W[i], adapters ? A_stack[i] : nullptr,
                                               adapters ? B_stack[i] : nullptr, d_in, d_out[i], r, scale, y[i],
                                               y_dt, st);
            if (rc != MOIN_OK) return rc;
        }
        return MOIN_OK;
    }
    const size_t u_bytes = align_up((size_t)pv.T * (size_t)r * 2, 256);
    const int rc = ensure_ws(ctx, (size_t)n * 2 * u_bytes, st);
    if (rc != MOIN_OK) return rc;
    void *u_hi[MAX_SHARED_X], *u_lo[MAX_SHARED_X];
    for (int i = 0; i < n; ++i) {
        u_hi[i] = static_cast<char *>(ctx->ws) + (size_t)i * 2 * u_bytes;
        u_lo[i] = static_cast<char *>(u_hi[i]) + u_bytes;
    }
    LinearArgs a;
    a.x = x; a.W = nullptr; a.A_stack = nullptr; a.B_stack = nullptr;
    a.u_hi = a.u_lo = nullptr;
    a.y = nullptr; a.y_f32 = (y_dt == MOIN_F32);
    a.d_in = d_in; a.d_out = 0; a.r = r; a.scale = scale; a.act = ctx->act;
    if (timed(ctx, MOIN_K_SHRINK, st, [&] {
            return launch_prefill_shrink_shared(pv, a, n, A_stack, u_hi, u_lo, st);
        }) != hipSuccess)
        return MOIN_EHIP;
    LinearArgs all[MAX_SHARED_X];
    bool stream_all = true;
    for (int i = 0; i < n; ++i) {
        all[i] = a;
        all[i].W = W[i]; all[i].A_stack = A_stack[i]; all[i].B_stack = B_stack[i];
        all[i].u_hi = u_hi[i]; all[i].u_lo = u_lo[i];
        all[i].y = y[i]; all[i].d_out = d_out[i];
        stream_all = stream_all && stream_kernel_fits(all[i]);
    }
    if (stream_all) {
        // one launch: the projections' column tiles side by side in the streaming kernel, so a narrow
        // projection (k, v) shares the wide one's x panels in L2 instead of streaming x on its own
        if (timed(ctx, MOIN_K_LINEAR, st, [&] { return launch_prefill_linear_shared(pv, all, n, st); }) != hipSuccess)
            return MOIN_EHIP;
        return MOIN_OK;
    }
    for (int i = 0; i < n; ++i)
        if (timed(ctx, MOIN_K_LINEAR, st, [&] { return launch_prefill_linear(pv, all[i], st); }) != hipSuccess)
            return MOIN_EHIP;
    return MOIN_OK;
}

int moin_lora_linear_ranked(moin_ctx *ctx, const void *x, const int32_t *seq_offsets,
                            const int32_t *expert_ids, int32_t S, int64_t T, const void *W,
                            const void *A_stack, const void *B_stack, int32_t E, int32_t d_in,
                            int32_t d_out, int32_t r, const int32_t *rank_of_expert, float scale,
                            void *y, moin_dtype y_dt, void *stream)
{
    if (!ctx) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    if (!ctx->own_plan) {
        const int rc = moin_plan_create(ctx, &ctx->own_plan);
        if (rc != MOIN_OK) return rc;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (S < 0 || T < 0 || E < 0) return MOIN_EINVAL;
    if (S > 0 && T > 0) {
        const int vrc = validate_linear(x, W, A_stack, B_stack, E, d_in, d_out, r, scale, y, y_dt);
        if (vrc != MOIN_OK) return vrc;
    }
    int rc = plan_build_impl(ctx, ctx->own_plan, seq_offsets, expert_ids, S, T, E, rank_of_expert, st);
    if (rc != MOIN_OK) return rc;
    return linear_planned_impl(ctx, ctx->own_plan, x, W, A_stack, B_stack, d_in, d_out, r, scale, y,
                               y_dt, st);
}

int moin_lora_linear(moin_ctx *ctx, const void *x, const int32_t *seq_offsets,
                     const int32_t *expert_ids, int32_t S, int64_t T, const void *W,
                     const void *A_stack, const void *B_stack, int32_t E, int32_t d_in,
                     int32_t d_out, int32_t r, float scale, void *y, moin_dtype y_dt, void *stream)
{
    return moin_lora_linear_ranked(ctx, x, seq_offsets, expert_ids, S, T, W, A_stack, B_stack, E, d_in,
                                   d_out, r, nullptr, scale, y, y_dt, stream);
}

int moin_mx_quantize(moin_ctx *ctx, const void *src, int64_t rows, int64_t cols, void *codes,
                     void *scales, int32_t scale_layout, void *stream)
{
    if (!ctx || rows < 0 || cols <= 0 || cols % 32) return MOIN_EINVAL;
    if (scale_layout != MOIN_MX_ROW_MAJOR && scale_layout != MOIN_MX_BLOCKED) return MOIN_EINVAL;
    if (scale_layout == MOIN_MX_BLOCKED && cols % 128) return MOIN_EINVAL;
    if (rows == 0) return MOIN_OK;
    if (!src || !codes || !scales || misaligned(src, 16) || misaligned(codes, 16) || misaligned(scales, 4))
        return MOIN_EINVAL;
    if (rows > (int64_t)1 << 40 || cols > (int64_t)1 << 30 || rows * cols > (int64_t)1 << 46)
        return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (timed(ctx, MOIN_K_MX_QUANT, st, [&] { return launch_mx_quantize(src, rows, cols, codes, scales, scale_layout == MOIN_MX_BLOCKED, st); }) !=
        hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

int moin_lora_linear_mx(moin_ctx *ctx, const void *x, const int32_t *seq_offsets,
                        const int32_t *expert_ids, int32_t S, int64_t T, const void *Wq,
                        const void *Ws, const void *A_stack, const void *B_stack, int32_t E,
                        int32_t d_in, int32_t d_out, int32_t r, const int32_t *rank_of_expert,
                        float scale, void *y, moin_dtype y_dt, void *stream)
{
    if (!ctx) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    if (!ctx->own_plan) {
        const int rc = moin_plan_create(ctx, &ctx->own_plan);
        if (rc != MOIN_OK) return rc;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (S < 0 || T < 0 || E < 0) return MOIN_EINVAL;
    if (S > 0 && T > 0) {
        const int vrc = validate_linear(x, Wq, A_stack, B_stack, E, d_in, d_out, r, scale, y, y_dt);
        if (vrc != MOIN_OK) return vrc;
        if (!Ws || misaligned(Ws, 16)) return MOIN_EINVAL;
        if (!mx_stream_kernel_fits(d_in, (E > 0 && r > 0) ? r : 0)) return MOIN_EINVAL;
    }
    int rc = plan_build_impl(ctx, ctx->own_plan, seq_offsets, expert_ids, S, T, E, rank_of_expert, st);
    if (rc != MOIN_OK) return rc;
    return linear_mx_planned_impl(ctx, ctx->own_plan, x, nullptr, nullptr, false, Wq, Ws, A_stack, B_stack, d_in,
                                  d_out, r, scale, y, y_dt, st);
}

int moin_lora_linear_mx_planned(moin_ctx *ctx, const moin_plan *plan, const void *x, void *xq, void *xs,
                                int32_t x_codes, const void *Wq, const void *Ws, const void *A_stack,
                                const void *B_stack, int32_t d_in, int32_t d_out, int32_t r,
                                float scale, void *y, moin_dtype y_dt, void *stream)
{
    if (!ctx || !plan || plan->device != ctx->device) return MOIN_EINVAL;
    if (x_codes != MOIN_MX_X_INTERNAL && x_codes != MOIN_MX_X_EMIT && x_codes != MOIN_MX_X_GIVEN)
        return MOIN_EINVAL;
    if ((xq == nullptr) != (xs == nullptr) || (xq == nullptr) != (x_codes == MOIN_MX_X_INTERNAL))
        return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    if (plan->built && plan->pv.S > 0 && plan->pv.T > 0) {
        const int vrc = validate_linear(x, Wq, A_stack, B_stack, plan->pv.E, d_in, d_out, r, scale, y, y_dt);
        if (vrc != MOIN_OK) return vrc;
        if (!Ws || misaligned(Ws, 16)) return MOIN_EINVAL;
        if (xq && (misaligned(xq, 16) || misaligned(xs, 16))) return MOIN_EINVAL;
        if (!mx_stream_kernel_fits(d_in, (plan->pv.E > 0 && r > 0) ? r : 0)) return MOIN_EINVAL;
    }
    return linear_mx_planned_impl(ctx, plan, x, xq, xs, x_codes == MOIN_MX_X_GIVEN, Wq, Ws, A_stack, B_stack, d_in, d_out, r, scale, y,
                                  y_dt, static_cast<hipStream_t>(stream));
}

int moin_kmeans_update(moin_ctx *ctx, const void *emb, const int32_t *ids, int64_t N,
                       const void *centroids, int32_t K, int32_t D, moin_dtype dt,
                       void *new_centroids, moin_dtype out_dt, int32_t *counts, double *inertia,
                       void *stream)
{
    if (!ctx || N < 0 || K <= 0 || D <= 0 || !centroids) return MOIN_EINVAL;
    if (dt != MOIN_BF16 && dt != MOIN_F32) return MOIN_EINVAL;
    if (out_dt != MOIN_BF16 && out_dt != MOIN_F32) return MOIN_EINVAL;
    if (N > 0 && (!emb || !ids)) return MOIN_EINVAL;
    if (dt == MOIN_BF16 ? (D % 8 != 0) : (D % 4 != 0)) return MOIN_EINVAL;
    if (K > KM_MAX_K || D > (1 << 20) || N > 0x7fffffffLL - 4096) return MOIN_EINVAL;
    if (misaligned(centroids, 16) || (emb && misaligned(emb, 16)) ||
        (new_centroids && misaligned(new_centroids, 16)))
        return MOIN_EINVAL;
    if (new_centroids == centroids && out_dt != dt) return MOIN_EINVAL;
    if (!new_centroids && !counts && !inertia) return MOIN_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);

    KmeansArgs a;
    a.emb = emb; a.ids = ids; a.N = N; a.cent = centroids; a.K = K; a.D = D;
    a.is_bf16 = (dt == MOIN_BF16);
    a.out = new_centroids; a.out_bf16 = (out_dt == MOIN_BF16);
    a.inertia = inertia;
    a.err_word = ctx->err_word;
    kmeans_shape(N, K, D, a.is_bf16, &a.chunk, &a.n_chunks, &a.max_pieces, &a.ncb);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    const size_t o_table = take((size_t)a.n_chunks * K * 4);
    const size_t o_counts = take((size_t)K * 4);
    const size_t o_seg = take((size_t)(K + 1) * 4);
    const size_t o_pst = take((size_t)(K + 1) * 4);
    const size_t o_pieces = take((size_t)(a.max_pieces + 1) * 16);
    const size_t o_np = take(4);
    const size_t o_perm = take((size_t)(N + 1) * 4);
    const size_t o_part = take((size_t)(a.max_pieces + 1) * D * 4);
    const size_t o_ipart = take((size_t)(a.max_pieces + 1) * a.ncb * 8);
    const int rc = ensure_ws(ctx, off, st);
    if (rc != MOIN_OK) return rc;
    char *w = static_cast<char *>(ctx->ws);
    a.table = reinterpret_cast<int *>(w + o_table);
    a.counts = counts ? counts : reinterpret_cast<int *>(w + o_counts);
    a.seg_start = reinterpret_cast<int *>(w + o_seg);
    a.piece_start = reinterpret_cast<int *>(w + o_pst);
    a.pieces = reinterpret_cast<int4 *>(w + o_pieces);
    a.n_pieces = reinterpret_cast<int *>(w + o_np);
    a.perm = reinterpret_cast<int *>(w + o_perm);
    a.partial = reinterpret_cast<float *>(w + o_part);
    a.inertia_part = reinterpret_cast<double *>(w + o_ipart);

    if (timed(ctx, MOIN_K_KMEANS_SORT, st, [&] { return launch_kmeans_sort(a, st); }) != hipSuccess)
        return MOIN_EHIP;
    if (!new_centroids && !inertia) return MOIN_OK;   // counts only
    if (timed(ctx, MOIN_K_KMEANS_SUM, st, [&] { return launch_kmeans_segsum(a, st); }) != hipSuccess)
        return MOIN_EHIP;
    if (timed(ctx, MOIN_K_KMEANS_FINAL, st, [&] { return launch_kmeans_finalize(a, st); }) != hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

int moin_retain_clusters(moin_ctx *ctx, const int32_t *counts, int32_t K, int32_t min_count,
                         int32_t *slot_of_centroid, int32_t *n_retained, void *stream)
{
    if (!ctx || K <= 0 || !counts || !slot_of_centroid) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (timed(ctx, MOIN_K_KMEANS_FINAL, st, [&] {
            return launch_kmeans_retain(counts, K, min_count, slot_of_centroid, n_retained, st);
        }) != hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

int moin_kmeans_fit(moin_ctx *ctx, const void *emb, int64_t N, void *centroids, int32_t K, int32_t D,
                    moin_dtype dt, int32_t iters, int32_t *ids, int32_t *counts, double *inertia,
                    void *stream)
{
    if (!ctx || iters < 0 || N < 0 || !centroids) return MOIN_EINVAL;
    if (N > 0 && (!emb || !ids)) return MOIN_EINVAL;
    if (K <= 0 || K > KM_MAX_K) return MOIN_EINVAL;
    for (int32_t it = 0; it <= iters; ++it) {
        // assignment against the current centres
        int rc = moin_route(ctx, emb, centroids, N, K, D, dt, nullptr, 0, nullptr, ids, nullptr, stream);
        if (rc != MOIN_OK) return rc;
        // objective of this assignment; all but the last round also move the centres (in place)
        const bool last = it == iters;
        rc = moin_kmeans_update(ctx, emb, ids, N, centroids, K, D, dt, last ? nullptr : centroids, dt,
                                last ? counts : nullptr, inertia ? inertia + it : nullptr, stream);
        if (rc != MOIN_OK) return rc;
    }
    return MOIN_OK;
}

int moin_timing_enable(moin_ctx *ctx, int on)
{
    if (!ctx) return MOIN_EINVAL;
    ctx->timing = on ? 1 : 0;
    return MOIN_OK;
}

int moin_timing_reset(moin_ctx *ctx)
{
    if (!ctx) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    const int rc = drain_spans(ctx);
    for (int i = 0; i < MOIN_K_COUNT; ++i) {
        ctx->ms_sum[i] = 0.0;
        ctx->launches[i] = 0;
    }
    return rc;
}

int moin_timing_read(moin_ctx *ctx, int kernel_id, double *ms_sum, int64_t *launches)
{
    if (!ctx || kernel_id < 0 || kernel_id >= MOIN_K_COUNT) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    const int rc = drain_spans(ctx);
    if (ms_sum) *ms_sum = ctx->ms_sum[kernel_id];
    if (launches) *launches = ctx->launches[kernel_id];
    return rc;
}

int moin_route_topk(moin_ctx *ctx, const void *emb, const void *centroids, int64_t N, int32_t K, int32_t D,
                    moin_dtype dt, const int32_t *slot_of_centroid, uint32_t flags, int32_t k,
                    int32_t *expert_ids, int32_t *centroid_ids, float *dist2, void *stream)
{
    if (!ctx || N < 0 || K <= 0 || D <= 0 || k < 1 || k > 8) return MOIN_EINVAL;
    if (dt != MOIN_BF16 && dt != MOIN_F32) return MOIN_EINVAL;
    if (flags & ~MOIN_ROUTE_RETAINED_ONLY) return MOIN_EINVAL;
    if ((flags & MOIN_ROUTE_RETAINED_ONLY) && !slot_of_centroid) return MOIN_EINVAL;
    if (!centroids || (N > 0 && !emb)) return MOIN_EINVAL;
    if (dt == MOIN_BF16 ? (D % 8 != 0) : (D % 4 != 0)) return MOIN_EINVAL;
    if (D > (1 << 20) || K > (1 << 28) || N > (int64_t)0x7fffffff / 8) return MOIN_EINVAL;
    if (misaligned(centroids, 16) || (emb && misaligned(emb, 16))) return MOIN_EINVAL;
    if (N == 0 || (!expert_ids && !centroid_ids && !dist2)) return MOIN_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    RouteArgs a{};
    a.emb = emb; a.cent = centroids; a.N = N; a.K = K; a.D = D;
    a.is_bf16 = (dt == MOIN_BF16);
    a.slot = slot_of_centroid;
    a.retained_only = (flags & MOIN_ROUTE_RETAINED_ONLY) ? 1 : 0;
    a.cid = centroid_ids;
    a.expert_ids = expert_ids;
    if (timed(ctx, MOIN_K_ROUTE, st, [&] { return launch_route_topk(a, k, dist2, st); }) != hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

int moin_merge_adapters(moin_ctx *ctx, const void *A_stack, const void *B_stack, int32_t E, int32_t r,
                        int32_t d_in, int32_t d_out, const int32_t *ids, const float *weights, int32_t n,
                        int32_t r_out, void *A_out, void *B_out, void *stream)
{
    if (!ctx || !A_stack || !B_stack || !A_out || !B_out) return MOIN_EINVAL;
    if (E <= 0 || r <= 0 || d_in <= 0 || d_out <= 0 || n < 0 || r_out <= 0) return MOIN_EINVAL;
    if (r % 8 || d_in % 8 || r_out % 8 || (int64_t)n * r > r_out) return MOIN_EINVAL;
    if (n > 0 && (!ids || !weights)) return MOIN_EINVAL;
    if (misaligned(A_stack, 16) || misaligned(B_stack, 16) || misaligned(A_out, 16) || misaligned(B_out, 16))
        return MOIN_EINVAL;
    if ((int64_t)r_out * d_in > 0x7fffffffLL * 8 || (int64_t)d_out * r_out > 0x7fffffffLL * 8) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (launch_merge_adapters(A_stack, B_stack, E, r, d_in, d_out, ids, weights, n, r_out, A_out, B_out,
                              ctx->err_word, st) != hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

int moin_set_adapter_activation(moin_ctx *ctx, int32_t activation)
{
    if (!ctx || activation < MOIN_ACT_NONE || activation > MOIN_ACT_GELU) return MOIN_EINVAL;
    ctx->act = activation;
    return MOIN_OK;
}

int64_t moin_probe_out_len(moin_ctx *ctx)
{
    if (!ctx) return 0;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return 0;
    return probe_out_len();
}

int moin_probe_mfma_bf16(moin_ctx *ctx, const void *operands, int64_t n_bytes, int32_t iters, float *out,
                         double *flops, void *stream)
{
    if (!ctx || !operands || !out || n_bytes < 16 || n_bytes % 16 || iters < 0 || misaligned(operands, 16))
        return MOIN_EINVAL;
    if (n_bytes / 16 > 0x7fffffffLL) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (timed(ctx, MOIN_K_PROBE_MFMA, st, [&] {
            return launch_probe_mfma(operands, n_bytes, iters, out, flops, st);
        }) != hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

int moin_probe_mfma_mxfp8(moin_ctx *ctx, const void *codes, int64_t n_bytes, int32_t iters, float *out,
                          double *flops, void *stream)
{
    if (!ctx || !codes || !out || n_bytes < 16 || n_bytes % 16 || iters < 0 || misaligned(codes, 16))
        return MOIN_EINVAL;
    if (n_bytes / 16 > 0x7fffffffLL) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (timed(ctx, MOIN_K_PROBE_MFMA, st, [&] {
            return launch_probe_mfma_mx(codes, n_bytes, iters, out, flops, st);
        }) != hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

int moin_probe_read(moin_ctx *ctx, const void *src, int64_t n_bytes, uint32_t *out, void *stream)
{
    if (!ctx || !src || !out || n_bytes < 0 || n_bytes % 16 || misaligned(src, 16)) return MOIN_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return MOIN_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (timed(ctx, MOIN_K_PROBE_READ, st, [&] { return launch_probe_read(src, n_bytes, out, st); }) != hipSuccess)
        return MOIN_EHIP;
    return MOIN_OK;
}

}  // extern "C"
