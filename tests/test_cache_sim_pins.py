"""Pins of the expert-cache simulator against the paper's statements and textbook LRU."""
from collections import OrderedDict

import numpy as np

from oracle.cache_sim import CacheSim


def test_prefill_each_expert_fetched_once_through_two_slots():
    # Section V-B: with a GPU cache of 2 and 8 experts per layer, the first experts are
    # prefetched during the non-MoE compute, then every expert's weights are fetched exactly
    # once, the two slots alternating between "computing" and "being fetched".
    c = CacheSim(E=8, S=2, blob_bytes=100)
    issued = c.prefetch([0, 1])
    assert issued == [(0, 0), (1, 1)]
    hits, misses, fetched = c.serve(range(8))
    assert hits == [0, 1] and misses == [2, 3, 4, 5, 6, 7]
    assert [e for e, _ in c.copies] == list(range(8))            # each expert once, ascending
    assert [s for _, s in c.copies] == [n % 2 for n in range(8)]  # ring through the slots
    assert c.bytes_h2d == 8 * 100
    assert c.counters()["prefetch_useful"] == 2


def test_speculative_expert_with_no_tokens_is_wasted_not_wrong():
    c = CacheSim(E=8, S=2, blob_bytes=10)
    c.prefetch([0, 1])
    hits, misses, _ = c.serve([1, 4, 6])
    assert hits == [1] and misses == [4, 6]
    assert c.counters()["prefetch_useful"] == 1
    assert c.bytes_h2d == 4 * 10
    # expert 0's slot (never served) is the first victim, then the hit's slot
    assert c.copies[2:] == [(4, 0), (6, 1)]


def test_all_resident_never_copies():
    c = CacheSim(E=8, S=8, blob_bytes=1, initial=list(range(8)))
    for _ in range(5):
        hits, misses, fetched = c.serve([0, 3, 7])
        assert misses == [] and fetched == []
    assert c.prefetch([1, 2, 3]) == []
    assert c.bytes_h2d == 0 and c.hits == 15


def test_decode_cache_of_k_serves_single_request():
    # Section V-A: a GPU cache of k slots is enough for single-request decode
    rng = np.random.default_rng(0)
    c = CacheSim(E=8, S=2, blob_bytes=1)
    for _ in range(100):
        act = rng.choice(8, 2, replace=False)
        hits, misses, fetched = c.serve(act)
        assert sorted(hits + misses) == sorted(act.tolist())
        assert all(c.slot_of(int(e)) >= 0 for e in act)  # both resident after the call
    assert c.hits + c.misses == 200


def test_single_expert_stream_is_textbook_lru():
    rng = np.random.default_rng(1)
    E, S = 10, 4
    c = CacheSim(E, S, 1)
    lru = OrderedDict()
    for e in rng.integers(0, E, 500):
        e = int(e)
        hits, misses, _ = c.serve([e])
        if e in lru:
            lru.move_to_end(e)
            assert hits == [e]
        else:
            assert misses == [e]
            if len(lru) == S:
                lru.popitem(last=False)
            lru[e] = True
        assert sorted(x for x in c.slot_expert if x >= 0) == sorted(lru)


def test_prefetch_protects_its_own_request_and_drops_overflow():
    c = CacheSim(E=8, S=3, blob_bytes=1, initial=[0, 1, 2])
    issued = c.prefetch([5, 1, 6, 7, 5])
    # 1 is resident (kept, stamped); 5 and 6 evict 0 and 2; 7 finds every slot protected
    assert issued == [(5, 0), (6, 2)]
    assert c.slot_expert == [5, 1, 6]
    assert c.counters()["prefetch_dropped"] == 1 and c.counters()["prefetch_issued"] == 2


def test_wrong_prediction_is_refetched():
    # Section V-C: a mismatch between the gate's choice and the cache triggers a re-fetch
    c = CacheSim(E=8, S=3, blob_bytes=7, initial=[0, 1, 2])
    c.prefetch([3, 4, 5])
    hits, misses, fetched = c.serve([6, 7])
    assert hits == [] and misses == [6, 7]
    assert c.slot_of(6) >= 0 and c.slot_of(7) >= 0
    assert c.counters() == dict(hits=0, misses=2, prefetch_issued=3, prefetch_useful=0,
                                prefetch_dropped=0, bytes_h2d=5 * 7)


def test_more_active_than_slots_streams_all():
    c = CacheSim(E=60, S=15, blob_bytes=1, initial=list(range(15)))
    act = [0, 3, 14, 20, 21, 22, 23, 24, 25, 26, 27, 28, 29, 30, 31, 32, 33, 34, 35, 36]
    hits, misses, fetched = c.serve(act)
    assert hits == [0, 3, 14] and len(misses) == 17
    # non-active residents go first (they carry the oldest stamps), hits last
    victims = [s for _, s in fetched]
    assert victims[:12] == [1, 2, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13]
    assert victims[12:15] == [0, 3, 14]
    assert len(set(e for e, _ in fetched)) == 17


# ---------------------------------------------------------------- one cache for all layers (Section V-A)
def test_shared_cache_of_k_is_refilled_layer_after_layer():
    """A cache of k = 2 experts serving 3 layers: right predictions are hits, each expert is fetched once
    per layer visit, and the slot of the expert that was used first is the first one refilled."""
    from oracle.cache_sim import SharedCacheSim
    sim = SharedCacheSim(3, 8, 2, 100)
    sim.prefetch(0, [1, 5])
    assert sim.state(0) == [1, 5] and sim.state(1) == [-1, -1]
    hits, misses = sim.serve(0, [5, 1])
    assert hits == [1, 5] and misses == []
    sim.prefetch(1, [2, 7])                       # evicts layer 0's experts in the order they were used
    assert sim.copies[-2:] == [(1, 2, 0), (1, 7, 1)]
    assert sim.state(0) == [-1, -1] and sim.state(1) == [2, 7]
    hits, misses = sim.serve(1, [2, 3])           # 7 was a wrong guess: 3 is fetched again into the LRU slot
    assert hits == [2] and misses == [3] and sim.state(1) == [2, 3]
    assert sim.counters(1) == dict(hits=1, misses=1, prefetch_issued=2, prefetch_useful=1, prefetch_dropped=0,
                                   bytes_h2d=300)
    assert sim.counters(0)["bytes_h2d"] == 200 and sim.counters(0)["prefetch_useful"] == 2


def test_shared_cache_reduces_to_per_layer_cache_for_one_layer():
    """With a single layer the shared cache is the per-layer cache: same copies, same counters."""
    import random
    from oracle.cache_sim import CacheSim, SharedCacheSim
    rng = random.Random(5)
    a, b = CacheSim(8, 3, 10), SharedCacheSim(1, 8, 3, 10)
    for _ in range(200):
        ids = rng.sample(range(8), rng.randint(1, 4))
        if rng.random() < 0.5:
            a.prefetch(ids); b.prefetch(0, ids)
        else:
            a.serve(ids); b.serve(0, ids)
        assert a.slot_expert == b.state(0)
    assert a.counters() == b.counters(0)
    assert [(e, s) for _, e, s in b.copies] == a.copies


def test_shared_cache_protects_only_the_asking_layer():
    """Full cache, every slot holds the asking layer's own request: nothing to evict, the rest is dropped;
    another layer's entries are fair game."""
    from oracle.cache_sim import SharedCacheSim
    sim = SharedCacheSim(2, 8, 2, 1)
    sim.prefetch(0, [0, 1])
    sim.prefetch(0, [0, 1, 2])
    assert sim.counters(0)["prefetch_dropped"] == 1 and sim.state(0) == [0, 1]
    sim.prefetch(1, [0, 1])                       # same ids, other layer: both slots change owner
    assert sim.state(0) == [-1, -1] and sim.state(1) == [0, 1]
