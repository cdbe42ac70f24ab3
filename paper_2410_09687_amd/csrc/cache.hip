// Adapter residency cache (Section 2, "efficiently serving" paragraph: the
// adapters of thousands of topics live in CPU memory, the most frequently
// routed ones are cached in GPU memory).  Host-side bookkeeping plus the
// host-to-device copies of the adapters a batch needs and does not find
// resident; the kernels then run on the slot stacks with slot ids in place of
// expert ids.  Nothing here reads device memory.
//
// Policy (the paper names only the goal; this is the reading taken):
//   * every sequence of an admitted batch adds one to its expert's use count;
//   * an expert the batch needs is always made resident -- a slot is working
//     memory first and cache second;
//   * a free slot is taken lowest index first; otherwise the victim is the
//     resident expert NOT needed by this batch with the smallest use count,
//     then the least recently used, then the lowest slot index;
//   * if every slot holds an expert of this batch, the remaining experts of the
//     batch get slot -1: their sequences run on the base model alone.
// Overlap mode (moin_cache_set_overlap): the copies go on a stream of the cache's
// own, so the adapters of batch k+1 cross PCIe while batch k computes.  What
// batch k reads must then not be overwritten: the experts of the batch admitted
// just before are protected like the batch's own, and the copy stream first waits
// for the compute work that was enqueued before THAT admission (everything that
// may still read any other slot).  The compute stream waits for the copies.
#include "../../include/moin.h"

#include <hip/hip_runtime.h>

#include <new>
#include <vector>

struct CacheStack {
    const char *a_host, *b_host;
    char *a_slots, *b_slots;
    size_t a_bytes, b_bytes;
};

struct moin_cache {
    int32_t E, n_slots;
    std::vector<int32_t> slot_of;      // [E] slot or -1
    std::vector<int32_t> expert_in;    // [n_slots] expert or -1
    std::vector<int64_t> uses;         // [E]
    std::vector<int64_t> last_used;    // [E] batch number of the last use
    std::vector<int64_t> seen_in;      // [E] batch number in which the expert was last seen (scratch)
    std::vector<int32_t> batch_count;  // [E] scratch
    std::vector<int32_t> order;        // distinct experts of the batch, first appearance first
    std::vector<CacheStack> stacks;
    // overlap mode
    int overlap;
    hipStream_t copy_stream;
    hipEvent_t compute_mark[2];   // compute stream at the last two admissions (newest: index tick % 2)
    hipEvent_t copies_done;
    int marks;                    // admissions that recorded a mark so far
    int64_t tick;
    int64_t stats[MOIN_CACHE_STAT_COUNT];
};

extern "C" {

int moin_cache_create(moin_cache **out, int32_t E, int32_t n_slots)
{
    if (!out || E <= 0 || n_slots <= 0) return MOIN_EINVAL;
    *out = nullptr;
    moin_cache *c = new (std::nothrow) moin_cache();
    if (!c) return MOIN_ENOMEM;
    try {
        c->E = E;
        c->n_slots = n_slots;
        c->slot_of.assign(E, -1);
        c->expert_in.assign(n_slots, -1);
        c->uses.assign(E, 0);
        c->last_used.assign(E, 0);
        c->seen_in.assign(E, 0);
        c->batch_count.assign(E, 0);
        c->order.reserve(1024);
    } catch (...) {
        delete c;
        return MOIN_ENOMEM;
    }
    c->tick = 0;
    c->overlap = 0;
    c->copy_stream = nullptr;
    c->compute_mark[0] = c->compute_mark[1] = c->copies_done = nullptr;
    c->marks = 0;
    for (int i = 0; i < MOIN_CACHE_STAT_COUNT; ++i) c->stats[i] = 0;
    *out = c;
    return MOIN_OK;
}

void moin_cache_destroy(moin_cache *cache)
{
    if (!cache) return;
    if (cache->copy_stream) {
        (void)hipStreamSynchronize(cache->copy_stream);
        (void)hipStreamDestroy(cache->copy_stream);
    }
    for (hipEvent_t e : {cache->compute_mark[0], cache->compute_mark[1], cache->copies_done})
        if (e) (void)hipEventDestroy(e);
    delete cache;
}

int moin_cache_set_overlap(moin_cache *cache, int on)
{
    if (!cache) return MOIN_EINVAL;
    for (int32_t s = 0; s < cache->n_slots; ++s)
        if (cache->expert_in[s] >= 0) return MOIN_EINVAL;   // a property of the whole request stream
    cache->overlap = on ? 1 : 0;
    return MOIN_OK;
}

int moin_cache_add_stack(moin_cache *cache, const void *A_host, const void *B_host, void *A_slots,
                         void *B_slots, int64_t a_bytes_per_expert, int64_t b_bytes_per_expert)
{
    if (!cache || !A_host || !B_host || !A_slots || !B_slots) return MOIN_EINVAL;
    if (a_bytes_per_expert <= 0 || b_bytes_per_expert <= 0) return MOIN_EINVAL;
    for (int32_t s = 0; s < cache->n_slots; ++s)
        if (cache->expert_in[s] >= 0) return MOIN_EINVAL;   // stacks are registered before the first batch
    CacheStack st;
    st.a_host = static_cast<const char *>(A_host);
    st.b_host = static_cast<const char *>(B_host);
    st.a_slots = static_cast<char *>(A_slots);
    st.b_slots = static_cast<char *>(B_slots);
    st.a_bytes = (size_t)a_bytes_per_expert;
    st.b_bytes = (size_t)b_bytes_per_expert;
    try {
        cache->stacks.push_back(st);
    } catch (...) {
        return MOIN_ENOMEM;
    }
    return MOIN_OK;
}

int moin_cache_admit(moin_cache *cache, const int32_t *expert_ids, int32_t S, int32_t *slot_ids,
                     void *stream)
{
    if (!cache || S < 0) return MOIN_EINVAL;
    if (S == 0) return MOIN_OK;
    if (!expert_ids || !slot_ids) return MOIN_EINVAL;
    moin_cache &c = *cache;
    for (int32_t i = 0; i < S; ++i)
        if (expert_ids[i] < -1 || expert_ids[i] >= c.E) return MOIN_EINVAL;   // nothing has changed yet
    const int64_t now = ++c.tick;
    c.stats[MOIN_CACHE_BATCHES] += 1;

    // 1. distinct experts of the batch in order of first appearance, use counts
    c.order.clear();
    for (int32_t i = 0; i < S; ++i) {
        const int32_t e = expert_ids[i];
        if (e < 0) continue;
        if (c.seen_in[e] != now) {
            c.seen_in[e] = now;
            c.batch_count[e] = 0;
            try {
                c.order.push_back(e);
            } catch (...) {
                return MOIN_ENOMEM;
            }
        }
        c.batch_count[e] += 1;
    }
    for (int32_t e : c.order) {
        c.uses[e] += c.batch_count[e];
        c.last_used[e] = now;
    }

    // 2. residency
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool side = c.overlap && !c.stacks.empty();
    hipStream_t cp = st;   // the stream the copies go on
    if (side) {
        if (!c.copy_stream) {
            if (hipStreamCreateWithFlags(&c.copy_stream, hipStreamNonBlocking) != hipSuccess ||
                hipEventCreateWithFlags(&c.compute_mark[0], hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&c.compute_mark[1], hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&c.copies_done, hipEventDisableTiming) != hipSuccess) {
                (void)hipGetLastError();
                return MOIN_EHIP;
            }
        }
        cp = c.copy_stream;
        // Slots this admission may overwrite are read by nothing newer than the compute work that was
        // enqueued before the PREVIOUS admission (the previous batch's experts are protected below):
        // the copies wait for that mark, not for the batch that is computing now.
        if (c.marks > 0 && hipStreamWaitEvent(cp, c.compute_mark[(c.marks - 1) & 1], 0) != hipSuccess) return MOIN_EHIP;
        if (hipEventRecord(c.compute_mark[c.marks & 1], st) != hipSuccess) return MOIN_EHIP;
        c.marks += 1;
    }
    int32_t next_free = 0;
    for (int32_t e : c.order) {
        if (c.slot_of[e] >= 0) {
            c.stats[MOIN_CACHE_SEQ_HITS] += c.batch_count[e];
            continue;
        }
        c.stats[MOIN_CACHE_SEQ_MISSES] += c.batch_count[e];
        int32_t slot = -1;
        while (next_free < c.n_slots && c.expert_in[next_free] >= 0) ++next_free;
        if (next_free < c.n_slots) {
            slot = next_free;
        } else {
            for (int32_t s = 0; s < c.n_slots; ++s) {
                const int32_t v = c.expert_in[s];
                if (v < 0) {   // left free by a failed copy
                    slot = s;
                    break;
                }
                if (c.seen_in[v] == now) continue;   // needed by this batch
                if (c.overlap && c.seen_in[v] == now - 1) continue;   // may still be read by the batch before
                if (slot < 0) {
                    slot = s;
                    continue;
                }
                const int32_t w = c.expert_in[slot];
                if (c.uses[v] < c.uses[w] || (c.uses[v] == c.uses[w] && c.last_used[v] < c.last_used[w])) slot = s;
            }
            if (slot < 0) {
                c.stats[MOIN_CACHE_OVERFLOWS] += 1;
                continue;   // no slot to give: base model only
            }
            // the victim leaves the tables before its slot is touched
            if (c.expert_in[slot] >= 0) {
                c.slot_of[c.expert_in[slot]] = -1;
                c.expert_in[slot] = -1;
                c.stats[MOIN_CACHE_EVICTIONS] += 1;
            }
        }
        // copies first, tables after: a slot is never named as holding an expert whose bytes were not
        // all enqueued (after a failed copy the slot stays free, its contents undefined)
        int64_t bytes = 0;
        for (const CacheStack &k : c.stacks) {
            if (hipMemcpyAsync(k.a_slots + (size_t)slot * k.a_bytes, k.a_host + (size_t)e * k.a_bytes, k.a_bytes,
                               hipMemcpyHostToDevice, cp) != hipSuccess ||
                hipMemcpyAsync(k.b_slots + (size_t)slot * k.b_bytes, k.b_host + (size_t)e * k.b_bytes, k.b_bytes,
                               hipMemcpyHostToDevice, cp) != hipSuccess) {
                (void)hipGetLastError();
                if (side) {   // what was enqueued so far still has to land before the compute stream goes on
                    if (hipEventRecord(c.copies_done, cp) == hipSuccess) (void)hipStreamWaitEvent(st, c.copies_done, 0);
                }
                return MOIN_EHIP;
            }
            bytes += (int64_t)(k.a_bytes + k.b_bytes);
        }
        c.expert_in[slot] = e;
        c.slot_of[e] = slot;
        c.stats[MOIN_CACHE_LOADS] += 1;
        c.stats[MOIN_CACHE_BYTES] += bytes;
    }
    if (side) {
        // the batch's kernels, enqueued on `stream` after this call, wait for its adapters
        if (hipEventRecord(c.copies_done, cp) != hipSuccess || hipStreamWaitEvent(st, c.copies_done, 0) != hipSuccess)
            return MOIN_EHIP;
    }

    // 3. slot per sequence
    for (int32_t i = 0; i < S; ++i) slot_ids[i] = expert_ids[i] < 0 ? -1 : c.slot_of[expert_ids[i]];
    return MOIN_OK;
}

int moin_cache_table(const moin_cache *cache, int32_t *slot_of_expert, int32_t *expert_in_slot)
{
    if (!cache) return MOIN_EINVAL;
    if (slot_of_expert)
        for (int32_t e = 0; e < cache->E; ++e) slot_of_expert[e] = cache->slot_of[e];
    if (expert_in_slot)
        for (int32_t s = 0; s < cache->n_slots; ++s) expert_in_slot[s] = cache->expert_in[s];
    return MOIN_OK;
}

int moin_cache_stats(const moin_cache *cache, int64_t *stats)
{
    if (!cache || !stats) return MOIN_EINVAL;
    for (int i = 0; i < MOIN_CACHE_STAT_COUNT; ++i) stats[i] = cache->stats[i];
    return MOIN_OK;
}

}  // extern "C"
