"""The residency cache's bookkeeping in libmoin (host code: no GPU is touched
while no stack is registered) against the oracle's, batch by batch."""
import numpy as np
import pytest

import oracle
from paper_2410_09687_amd import moin


def _compare(E, n_slots, batches, overlap=False):
    c = moin.Cache(E, n_slots, overlap=overlap)
    ref = oracle.AdapterCache(E, n_slots, protect_previous=overlap)
    for ids in batches:
        got = c.admit(np.asarray(ids, np.int32)).numpy()
        want, _ = ref.admit(ids)
        assert np.array_equal(got, want)
        so, ei = c.tables()
        rso, rei = ref.tables()
        assert np.array_equal(so.numpy(), rso) and np.array_equal(ei.numpy(), rei)
    st = c.stats()
    assert [st["batches"], st["seq_hits"], st["seq_misses"], st["loads"], st["evictions"], st["overflows"]] == \
        [ref.batches, ref.hits, ref.misses, ref.loads, ref.evictions, ref.overflows]
    assert st["bytes"] == 0
    c.close()
    return st


def test_hand_trace_and_random_streams_match_the_oracle():
    _compare(6, 3, [[4, 4, 1], [2, 4], [5, 2], [0, 3, 5, -1], [0, 1, 2, 3]])
    rng = np.random.default_rng(3)
    for E, n_slots, n_batches, size in ((200, 17, 300, 40), (5000, 512, 60, 256), (10, 1, 50, 4), (50, 64, 40, 30)):
        batches = [(rng.zipf(1.2, size=rng.integers(1, size + 1)) % (E + 1) - 1) for _ in range(n_batches)]
        _compare(E, n_slots, batches)


def test_zipf_stream_hit_rate_rises_with_the_slot_count():
    # Table 3 of the paper: a workload touches a small share of the adapters; a cache an
    # order of magnitude smaller than the expert count then serves most sequences
    from paper_2410_09687_amd import workloads as wl
    rates = []
    for n_slots in (64, 256, 1024):
        batches = [wl.draw_expert_ids(256, 5000, "zipf", 1.1, 1000 + k, perm_seed=77) for k in range(40)]
        st = _compare(5000, n_slots, batches)
        rates.append(st["seq_hits"] / (st["seq_hits"] + st["seq_misses"]))
    assert rates[0] < rates[1] < rates[2] and rates[2] > 0.6


def test_errors_leave_the_cache_unchanged():
    c = moin.Cache(8, 2)
    c.admit(np.array([1, 2], np.int32))
    before = c.tables()[0].clone()
    with pytest.raises(moin.MoinError):
        c.admit(np.array([1, 8], np.int32))
    with pytest.raises(moin.MoinError):
        c.admit(np.array([-2], np.int32))
    assert np.array_equal(c.tables()[0].numpy(), before.numpy()) and c.stats()["batches"] == 1
    assert c.admit(np.zeros(0, np.int32)).numel() == 0
    with pytest.raises(moin.MoinError):
        moin.Cache(0, 4)
    c.close()


def test_overlap_mode_protects_the_previous_batch_like_the_oracle():
    # admitting batch k+1 while batch k computes: nothing batch k reads may be evicted
    rng = np.random.default_rng(5)
    for E, n_slots, n_batches, size in ((200, 17, 300, 12), (5000, 512, 60, 256), (10, 2, 50, 3), (40, 9, 80, 6)):
        batches = [(rng.zipf(1.2, size=rng.integers(1, size + 1)) % (E + 1) - 1) for _ in range(n_batches)]
        st = _compare(E, n_slots, batches, overlap=True)
    # the hand case: two slots, batch [0, 1] then [2]: in overlap mode 2 finds both slots protected
    c = moin.Cache(4, 2, overlap=True)
    assert c.admit(np.array([0, 1], np.int32)).tolist() == [0, 1]
    assert c.admit(np.array([2], np.int32)).tolist() == [-1]
    assert c.admit(np.array([2], np.int32)).tolist() == [0]      # batch [0, 1] is two admissions back now
    assert c.stats()["overflows"] == 1
    with pytest.raises(moin.MoinError):
        moin.load().moin_cache_set_overlap  # (exists)
        moin._ck(moin.load().moin_cache_set_overlap(c._h, 0), "moin_cache_set_overlap")   # too late: slots in use
    c.close()
