"""The oracle's side of the four entry points (oracle/entry_points.py) is a composition of pinned pieces;
pinned here against those pieces called directly, against the stored digest of the small configuration,
and against what the paper says about the cache (Sections V-B, V-C)."""
import json
import os

import numpy as np
import pytest

import oracle
from oracle.cache_sim import CacheSim
from oracle.entry_points import RefMoe
from paper_2509_07379_amd import synth as S

HERE = os.path.dirname(os.path.abspath(__file__))


def make(w, slots, layer=0, **kw):
    ref = RefMoe(w.d, w.I, w.E, w.k, max(1, w.L), slots, w.I_shared, **kw)
    blobs = [S.expert_blob(w, layer, e) for e in range(w.E)]
    ref.moe_bind_layer(layer, blobs, S.router_weight(w, layer), S.shared_blob(w, layer), None)
    return ref, blobs


def test_layer_call_is_the_pinned_composition_and_matches_the_stored_digest():
    w = S.WORKLOADS["c1_tiny"]
    ref, blobs = make(w, 2)
    x = S.activations(w)
    r = ref.moe_prefill_layer(0, x, w.T)
    direct = oracle.moe_layer(x, S.router_weight(w, 0), blobs, w.k, shared_blob=S.shared_blob(w, 0), I=w.I,
                              I_shared=w.I_shared)
    for key in ("ids", "counts", "offsets", "perm", "inv_perm", "out"):
        np.testing.assert_array_equal(r[key], direct[key], err_msg=key)
    gold = json.load(open(os.path.join(HERE, "golden", "c1_tiny_oracle.json")))
    assert r["counts"].tolist() == gold["counts"]
    assert int(r["out"].astype(np.int64).sum()) == gold["out_bits_sum"]


def test_prefill_through_two_slots_fetches_every_active_expert_once():
    # Section V-B: with two slots every expert that received tokens crosses the link once per layer
    w = S.WORKLOADS["c1_tiny"]
    ref, _ = make(w, 2)
    r = ref.moe_prefill_layer(0, S.activations(w), w.T)
    active = int((r["counts"] > 0).sum())
    st = ref.moe_get_stats(0)
    assert st["misses"] == active and st["hits"] == 0 and st["bytes_h2d"] == active * 6 * w.d * w.I
    assert r["call_stats"]["misses"] == active and st["layer_calls"] == 1


def test_decode_prefetch_then_verify_and_refetch():
    # Section V-C: a right guess is a hit and a useful prefetch, a wrong one is fetched again; the output
    # is the same bits either way
    w = S.Workload("ep", d=64, I=32, E=8, k=2, T=1, seed=5)
    x = S.activations(w)
    plain, _ = make(w, 3)
    want = plain.moe_decode_layer(0, x, 1)
    chosen = sorted(want["ids"][0].tolist())
    others = [e for e in range(w.E) if e not in chosen]
    good, _ = make(w, 3)
    good.expert_cache_prefetch(0, chosen)
    g = good.moe_decode_layer(0, x, 1)
    assert g["call_stats"]["hits"] == 2 and g["call_stats"]["misses"] == 0 and g["call_stats"]["prefetch_useful"] == 2
    bad, _ = make(w, 3)
    bad.expert_cache_prefetch(0, others[:2])
    b = bad.moe_decode_layer(0, x, 1)
    assert b["call_stats"]["hits"] == 0 and b["call_stats"]["misses"] == 2 and b["call_stats"]["prefetch_useful"] == 0
    np.testing.assert_array_equal(g["out"], want["out"])
    np.testing.assert_array_equal(b["out"], want["out"])
    assert set(chosen) <= set(bad.moe_cache_state(0))


def test_counters_are_the_simulators():
    w = S.Workload("ep2", d=64, I=32, E=8, k=2, T=5, seed=9)
    ref, _ = make(w, 3)
    sim = CacheSim(w.E, 3, 6 * w.d * w.I)
    rng = np.random.default_rng(3)
    for step in range(6):
        ids = rng.choice(w.E, size=2, replace=False).tolist()
        ref.expert_cache_prefetch(0, ids)
        sim.prefetch(ids)
        wl = S.Workload("ep2", d=64, I=32, E=8, k=2, T=5, seed=9 + step)
        r = ref.moe_decode_layer(0, S.activations(wl), 5)
        sim.serve(np.nonzero(r["counts"])[0])
        assert ref.moe_cache_state(0) == sim.slot_expert
    assert ref.moe_get_stats(0) == {**sim.counters(), "layer_calls": 6}


def test_predictor_entry_is_the_pinned_scorer():
    w = S.Workload("ep3", d=64, I=32, E=8, k=2, T=3, seed=11)
    ref, _ = make(w, 2)
    x, wp = S.activations(w), S.predictor_weight(w, 0)
    s, top = ref.predictor_score(0, x, 3, wp, 3)
    s2, top2 = oracle.predictor_score(x, wp, 3)
    np.testing.assert_array_equal(s, s2)
    np.testing.assert_array_equal(top, top2)
    assert s[top[0]] == s.max()
