"""Pins of the oracle's adapter residency bookkeeping (Section 2: the most
frequently routed adapters are cached on the GPU): a hand-worked trace,
invariants of any valid cache, and limits that reduce to something obvious."""
import os

import numpy as np
import pytest

import oracle
from tests.helpers import read_golden

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "cache_hand_example.txt")


def test_hand_worked_trace():
    g = read_golden(GOLDEN)
    c = oracle.AdapterCache(6, 3)
    for b in range(1, 6):
        ids = [int(v) for v in g[f"batch{b}_ids"]]
        slots, _ = c.admit(ids)
        assert slots.tolist() == [int(v) for v in g[f"batch{b}_slots"]], b
        assert c.tables()[1].tolist() == [int(v) for v in g[f"batch{b}_state"]], b
    assert [c.hits, c.misses, c.loads, c.evictions, c.overflows] == [int(v) for v in g["totals"]]


def test_hand_worked_trace_with_the_previous_batch_protected():
    g = read_golden(GOLDEN)
    c = oracle.AdapterCache(6, 3, protect_previous=True)
    for b in range(1, 6):
        ids = [int(v) for v in g[f"batch{b}_ids"]]
        slots, _ = c.admit(ids)
        assert slots.tolist() == [int(v) for v in g[f"overlap_batch{b}_slots"]], b
        assert c.tables()[1].tolist() == [int(v) for v in g[f"overlap_batch{b}_state"]], b
    assert [c.hits, c.misses, c.loads, c.evictions, c.overflows] == [int(v) for v in g["overlap_totals"]]
    # nothing a batch uses is evicted by the admission after it, whatever the stream
    rng = np.random.default_rng(4)
    c = oracle.AdapterCache(60, 7, protect_previous=True)
    prev = {}
    for _ in range(400):
        ids = rng.zipf(1.3, size=rng.integers(1, 6)) % 61 - 1
        slots, _ = c.admit(ids)
        slot_of = c.tables()[0]
        for e, s in prev.items():
            assert slot_of[e] == s, "an expert of the previous batch lost its slot"
        prev = {int(e): int(s) for e, s in zip(ids, slots) if e >= 0 and s >= 0}


def test_invariants_on_random_batches():
    rng = np.random.default_rng(0)
    E, n_slots = 200, 17
    c = oracle.AdapterCache(E, n_slots)
    total = 0
    for _ in range(300):
        ids = rng.zipf(1.3, size=rng.integers(1, 40)) % (E + 1) - 1      # -1 .. E-1, skewed
        slots, loaded = c.admit(ids)
        total += int((ids >= 0).sum())
        slot_of, expert_in = c.tables()
        # the two tables are inverse to each other, every slot holds at most one expert
        res = np.flatnonzero(slot_of >= 0)
        assert len(res) <= n_slots and len(set(slot_of[res])) == len(res)
        assert all(expert_in[slot_of[e]] == e for e in res)
        # a sequence either gets the slot that now holds its expert or -1
        for e, s in zip(ids, slots):
            assert s == (slot_of[e] if e >= 0 else -1)
        # with at most n_slots distinct experts in a batch nobody is left out
        if len(set(ids[ids >= 0])) <= n_slots:
            assert (slots[ids >= 0] >= 0).all()
        # whatever was loaded in this batch is resident now
        assert all(slot_of[e] == s for e, s in loaded)
    assert c.hits + c.misses == total
    assert c.loads - c.evictions == int((c.tables()[0] >= 0).sum())


def test_limits():
    # as many slots as experts: every expert misses once, nothing is ever evicted
    rng = np.random.default_rng(1)
    c = oracle.AdapterCache(30, 30)
    seen = set()
    for _ in range(50):
        ids = rng.integers(0, 30, size=8)
        c.admit(ids)
        seen.update(ids.tolist())
    assert c.evictions == 0 and c.overflows == 0 and c.loads == len(seen)
    # the same batch twice: the second pass is all hits
    c = oracle.AdapterCache(100, 8)
    ids = [3, 9, 9, 27, 81, 3]
    c.admit(ids)
    h = c.hits
    slots, loaded = c.admit(ids)
    assert loaded == [] and c.hits - h == len(ids) and (slots >= 0).all()
    # one slot: a two-expert batch leaves the second expert out
    c = oracle.AdapterCache(5, 1)
    slots, _ = c.admit([2, 4, 2])
    assert slots.tolist() == [0, -1, 0] and c.overflows == 1
    # frequency decides: a much used expert survives a stream of one-off experts
    c = oracle.AdapterCache(50, 2)
    c.admit([7] * 10)
    for e in range(10, 30):
        c.admit([e])
        assert c.tables()[0][7] >= 0
    with pytest.raises(ValueError):
        c.admit([50])
