// Host-only exercise of the adapter residency cache's bookkeeping (no stack registered: no GPU call is
// made), meant to be built with AddressSanitizer / UBSan on the host side and run on the CPU.  Random
// request streams in both modes, error paths, table and statistics reads; exits non-zero on a wrong
// invariant (the sanitizers abort on a memory error by themselves).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/moin.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd()
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}

#define REQUIRE(c)                                                        \
    do {                                                                  \
        if (!(c)) {                                                       \
            std::fprintf(stderr, "%s:%d: %s failed\n", __FILE__, __LINE__, #c); \
            return 1;                                                     \
        }                                                                 \
    } while (0)

static int run(int E, int n_slots, int overlap, int batches)
{
    moin_cache *c = nullptr;
    REQUIRE(moin_cache_create(&c, E, n_slots) == MOIN_OK);
    REQUIRE(moin_cache_set_overlap(c, overlap) == MOIN_OK);
    std::vector<int32_t> slot_of(E), expert_in(n_slots);
    std::vector<int32_t> prev_ids, prev_slots;
    int64_t seqs = 0, counted = 0;
    for (int b = 0; b < batches; ++b) {
        const int S = (int)(rnd() % 40);
        counted += S > 0;   // an empty batch is a no-op: not an admission
        std::vector<int32_t> ids(S), slots(S, -7);
        for (int i = 0; i < S; ++i) {
            // skewed: a square pushes most draws towards the low ids; about one in sixteen is "no adapter"
            const uint32_t u = rnd() % (uint32_t)E;
            ids[i] = (rnd() % 16 == 0) ? -1 : (int32_t)((uint64_t)u * u / (uint32_t)E);
        }
        REQUIRE(moin_cache_admit(c, ids.data(), S, slots.data(), nullptr) == MOIN_OK);
        REQUIRE(moin_cache_table(c, slot_of.data(), expert_in.data()) == MOIN_OK);
        for (int i = 0; i < S; ++i) {
            REQUIRE(slots[i] >= -1 && slots[i] < n_slots);
            if (ids[i] < 0) REQUIRE(slots[i] == -1);
            else REQUIRE(slots[i] == slot_of[ids[i]]);
            if (slots[i] >= 0) REQUIRE(expert_in[slots[i]] == ids[i]);
            seqs += ids[i] >= 0;
        }
        if (overlap)   // nothing the previous batch uses may have moved
            for (size_t i = 0; i < prev_ids.size(); ++i)
                if (prev_ids[i] >= 0 && prev_slots[i] >= 0) REQUIRE(slot_of[prev_ids[i]] == prev_slots[i]);
        if (S > 0) {
            prev_ids = ids;
            prev_slots = slots;
        }
    }
    int64_t st[MOIN_CACHE_STAT_COUNT];
    REQUIRE(moin_cache_stats(c, st) == MOIN_OK);
    REQUIRE(st[MOIN_CACHE_BATCHES] == counted);
    REQUIRE(st[MOIN_CACHE_SEQ_HITS] + st[MOIN_CACHE_SEQ_MISSES] == seqs);
    int resident = 0;
    for (int e = 0; e < E; ++e) resident += slot_of[e] >= 0;
    REQUIRE(st[MOIN_CACHE_LOADS] - st[MOIN_CACHE_EVICTIONS] == resident);
    // error paths leave everything as it was
    const int32_t bad[2] = {0, E};
    int32_t out[2];
    REQUIRE(moin_cache_admit(c, bad, 2, out, nullptr) == MOIN_EINVAL);
    REQUIRE(moin_cache_admit(c, nullptr, 3, out, nullptr) == MOIN_EINVAL);
    REQUIRE(moin_cache_admit(c, bad, 0, out, nullptr) == MOIN_OK);
    REQUIRE(moin_cache_set_overlap(c, !overlap) == (resident ? MOIN_EINVAL : MOIN_OK));
    int64_t st2[MOIN_CACHE_STAT_COUNT];
    REQUIRE(moin_cache_stats(c, st2) == MOIN_OK);
    for (int i = 0; i < MOIN_CACHE_STAT_COUNT; ++i) REQUIRE(st[i] == st2[i]);
    moin_cache_destroy(c);
    return 0;
}

int main()
{
    moin_cache *none = nullptr;
    if (moin_cache_create(&none, 0, 4) != MOIN_EINVAL || moin_cache_create(nullptr, 4, 4) != MOIN_EINVAL) return 1;
    moin_cache_destroy(nullptr);
    for (int overlap = 0; overlap < 2; ++overlap) {
        if (run(200, 17, overlap, 400)) return 1;
        if (run(5000, 512, overlap, 60)) return 1;
        if (run(7, 1, overlap, 200)) return 1;
        if (run(30, 64, overlap, 100)) return 1;
    }
    std::puts("cache host checks passed");
    return 0;
}
