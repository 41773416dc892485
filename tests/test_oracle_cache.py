"""Pins of the cache oracle: the paper's closed forms on hand-computed cases,
the paper's compute-reordering example, ARC invariants and known behaviours
(LRU on a scan, frequency protection), and the full-residency special case."""
import os
import random

import pytest

from oracle import cache as C

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_cache_total_and_n_closed_forms():
    # cache_total = (memory_budget - others) / expert          (section 4.4)
    assert C.cache_total_from_budget(24 * 2**30, 8 * 2**30, 4_460_544) == (16 * 2**30) // 4_460_544
    assert C.cache_total_from_budget(100, 200, 10) == 0
    assert C.cache_total_from_budget(1000, 100, 90) == 10
    # n = T / t_expert, T = t_moe + t_attn + t_gate            (section 4.3)
    # the paper's own figures: 13 ms per MoE block against 6 ms per expert -> 2
    assert C.n_max_from_times(13.0, 0.0, 0.0, 6.0) == 2
    assert C.n_max_from_times(1.0, 2.0, 0.5, 1.0) == 3
    assert C.n_max_from_times(0.1, 0.1, 0.1, 1.0) == 0


def test_layer_capacities_golden():
    rows = [l for l in open(os.path.join(GOLD, "cache_sizing_examples.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for line in rows:
        lhs, rhs = line.split(":")
        nl, E, total, L = (int(v) for v in lhs.split())
        want = [int(v) for v in rhs.split()]
        got = C.layer_capacities(nl, E, total, L)
        assert got == want
        assert sum(got) <= total and all(0 <= c <= E for c in got)
        assert got == sorted(got, reverse=True)          # shallow layers never get less


def test_capacity_properties_random():
    rnd = random.Random(0)
    for _ in range(300):
        nl, E = rnd.randint(1, 40), rnd.randint(1, 70)
        L = rnd.randint(0, nl + 2)
        total = rnd.randint(0, nl * E + 10)
        caps = C.layer_capacities(nl, E, total, L)
        assert len(caps) == nl and all(0 <= c <= E for c in caps)
        assert sum(caps) <= total
        Lc = min(L, nl)
        if total > Lc * E and nl > Lc:
            deep = caps[Lc:]
            assert max(deep) - min(deep) <= 1
            assert caps[:Lc] == [E] * Lc
            if max(deep) < E:
                assert sum(caps) == total          # nothing wasted unless every layer is full


def test_compute_order_paper_example():
    txt = dict(l.strip().split(": ") for l in open(os.path.join(GOLD, "compute_order_example.txt"))
               if ": " in l and not l.startswith("#"))
    pre = [int(v) for v in txt["prefetched"].split()]
    loading = [int(v) for v in txt["loading"].split()]
    orig = [int(v) for v in txt["original"].split()]
    fate = [int(v) for v in txt["fate"].split()]
    # one deep layer with capacity 2 holding nothing useful; layer 1 is the one stepped.
    # popularity follows the "original" request order.
    E = 6
    sim = C.CacheOracle(num_layers=2, E=E, cache_total=0, L_shallow=0, n_max=8, staging_slots=16)
    counts = {e: 10 - i for i, e in enumerate(orig)}
    # step layer 0 with a prediction that prefetches {2, 4} for layer 1
    sim.step(0, [0], [1], pred_ids=pre, pred_pop=[1] * len(pre))
    assert sim.staged[1] == pre
    ids = sorted(counts)
    r = sim.step(1, ids, [counts[e] for e in ids])
    assert r.hit_prefetch == pre
    assert r.miss == loading
    assert r.compute_order == fate
    assert [ld[1] for ld in r.loads if ld[3]] == loading


def _check_arc(a):
    c = a.c
    lists = [a.T1, a.T2, a.B1, a.B2]
    flat = [x for l in lists for x in l]
    assert len(flat) == len(set(flat))                       # disjoint
    assert len(a.T1) + len(a.T2) <= c
    assert len(a.T1) + len(a.B1) <= c
    assert len(flat) <= 2 * c
    assert 0 <= a.p <= c


def test_arc_invariants_random_traces():
    rnd = random.Random(1)
    for trial in range(40):
        c = rnd.randint(1, 12)
        U = rnd.randint(c, 40)
        a = C.ARC(c, preload=range(min(c, U)) if trial % 2 else ())
        resident_before = None
        for _ in range(600):
            x = rnd.randrange(U) if rnd.random() < 0.7 else rnd.randrange(min(U, c + 2))
            was = a.resident(x)
            n_before = len(a.T1) + len(a.T2)
            hit, ev = a.access(x)
            assert hit == was
            assert a.resident(x)                       # the accessed item is always admitted
            assert x in a.T2 if hit else True
            if ev is not None:
                assert not a.resident(ev) and ev != x
                assert len(a.T1) + len(a.T2) == n_before
            elif not hit:
                assert len(a.T1) + len(a.T2) == n_before + 1
            _check_arc(a)


def test_arc_scan_behaves_like_lru_and_frequency_is_protected():
    # a pure scan of distinct items: each new item evicts the oldest (LRU order)
    a = C.ARC(4)
    evs = []
    for x in range(10):
        hit, ev = a.access(x)
        assert not hit
        evs.append(ev)
    assert evs == [None, None, None, None, 0, 1, 2, 3, 4, 5]
    assert a.T1 == [6, 7, 8, 9] and a.T2 == []
    # items seen twice sit in T2 and survive a following scan of one-timers
    b = C.ARC(4)
    for x in (0, 1, 0, 1):
        b.access(x)
    assert b.T2 == [0, 1]
    for x in range(100, 120):
        b.access(x)
        assert b.resident(0) and b.resident(1)
    # a ghost hit in B1 grows the recency target p.  (A scan alone leaves no
    # ghosts: with T1 full and B1 empty the LRU of T1 is dropped outright.)
    c = C.ARC(2)
    for x in (0, 0, 1, 2):     # 0 -> T2; 1 enters T1 and is demoted to B1 by 2
        c.access(x)
    assert c.T2 == [0] and c.T1 == [2] and c.B1 == [1] and c.p == 0
    hit, ev = c.access(1)
    assert not hit and c.p == 1 and c.T2 == [1] and ev == 0 and c.B2 == [0] and c.T1 == [2]
    # a ghost hit in B2 shrinks it again
    hit, ev = c.access(0)
    assert not hit and c.p == 0 and ev == 2 and c.T2 == [1, 0] and c.B1 == [2]


def test_full_layers_always_hit_and_sizing_in_simulator():
    # "cache all experts in the first layers" => those layers always hit (section 4.4)
    sim = C.CacheOracle(num_layers=4, E=8, cache_total=2 * 8 + 4, L_shallow=2, n_max=2, staging_slots=20)
    assert sim.caps == [8, 8, 2, 2]
    rnd = random.Random(2)
    for stepi in range(50):
        for l in range(4):
            ids = sorted(rnd.sample(range(8), 3))
            pred = sorted(rnd.sample(range(8), 4))
            r = sim.step(l, ids, [1, 1, 1], pred, [1] * 4)
            if l < 2:
                assert r.miss == [] and r.hit_cache == ids and r.loads == [] or all(not d for *_, d in r.loads)
                assert sorted(r.hit_cache) == ids
            assert sorted(r.hit_cache + r.hit_prefetch + r.miss) == ids
            assert set(r.compute_order) == set(ids)
            # slot accounting: no slot is owned twice, none is lost
            owned = [s for d in sim.slot for s in d.values()]
            assert len(owned) == len(set(owned))
            assert sorted(owned + sim.free + sim.pending) == list(range(sim.total_slots))
            # residents per layer never exceed the layer's capacity
            for ll in range(2, 4):
                assert len(sim.arc[ll].T1) + len(sim.arc[ll].T2) <= sim.caps[ll]
            # at most n_max prefetches, never for a resident expert
            pf = [ld for ld in r.loads if not ld[3]]
            assert len(pf) <= 2 and all(ld[0] == l + 1 for ld in pf)


def test_simulator_zero_capacity_and_zero_nmax():
    sim = C.CacheOracle(num_layers=2, E=4, cache_total=0, L_shallow=1, n_max=0, staging_slots=8)
    assert sim.caps == [0, 0]
    r = sim.step(0, [1, 3], [2, 1], [0, 1], [1, 1])
    assert r.miss == [1, 3] and r.evicted == [1, 3] and not [l for l in r.loads if not l[3]]
    r = sim.step(1, [1], [1])
    assert r.miss == [1]
    r = sim.step(0, [1], [1])
    assert r.miss == [1]                      # nothing was kept
    assert sorted(sim.free + sim.pending) == list(range(8))


def test_eap_predictor_hand_case():
    """Activation-path baseline (section 5.1): prediction from co-activation counts, worked by hand."""
    p = C.EAPPredictor(3, 4)
    # calibration: two tokens.  token A: block 0 {0,1} -> block 1 {2,3}; token B: block 0 {1,2} -> block 1 {3,0}
    p.update(0, [[0, 1], [1, 2]], [[2, 3], [3, 0]])
    assert p.freq[0][0] == [0, 0, 1, 1]
    assert p.freq[0][1] == [1, 0, 1, 2]       # expert 1 was chosen by both tokens
    assert p.freq[0][2] == [1, 0, 0, 1]
    assert p.freq[0][3] == [0, 0, 0, 0]
    # a token that chose {1, 2}: scores [2, 0, 1, 3] -> top-2 = experts 3, 0
    assert p.predict(0, [[1, 2]], 2) == [1, 0, 0, 1]
    # a token that chose {0}: scores [0, 0, 1, 1] -> tie between 2 and 3 goes to the lower id with m = 1
    assert p.predict(0, [[0]], 1) == [0, 0, 1, 0]
    # zero scores are never predicted; popularity adds up over tokens
    assert p.predict(0, [[3]], 2) == [0, 0, 0, 0]
    assert p.predict(0, [[1, 2], [0], [0]], 2) == [1, 0, 2, 3]
    # block 1 has no statistics yet, the last block predicts nothing
    assert p.predict(1, [[0, 1]], 2) == [0, 0, 0, 0] and p.predict(2, [[0, 1]], 2) == [0, 0, 0, 0]


def test_hybrid_width_hand_trace():
    """Section 4.5: of the experts predicted for the next layer, the least popular quarter moves as a
    low-width copy; such a copy is used by its layer and dropped, it never enters the 4-bit cache."""
    c = C.CacheOracle(num_layers=2, E=8, cache_total=2, L_shallow=0, n_max=8, staging_slots=12, low_percent=25)
    assert c.caps == [1, 1]                           # expert 0 preloaded in each layer
    r = c.step(0, [0], [4], pred_ids=list(range(8)), pred_pop=[8, 7, 6, 5, 4, 3, 2, 1])
    # 8 predicted experts -> the 2 least popular (6, 7) are low-width; expert 0 is resident in layer 1
    assert [(e, d) for (_, e, _, d) in r.loads] == [(e, False) for e in range(1, 8)]
    assert r.load_bits == [4, 4, 4, 4, 4, 2, 2]
    assert c.staged_low[1] == {6, 7}
    # layer 1 activates 0 (cached), 2 (staged at 4 bits) and 6 (staged at 2 bits)
    r = c.step(1, [0, 2, 6], [3, 2, 1])
    assert r.hit_cache == [0] and r.hit_prefetch == [2, 6] and r.miss == []
    assert sorted(r.wasted) == [1, 3, 4, 5, 7]
    # 2 went through ARC (capacity 1: it replaces 0), 6 was dropped without touching ARC
    assert c.resident(1, 2) and not c.resident(1, 6) and not c.resident(1, 0)
    assert 6 in r.evicted and 6 not in c.staged[1] and c.staged_low[1] == set()
    # popularity zero does not count as predicted: 3 positive -> floor(0.75) = 0 low-width copies
    c2 = C.CacheOracle(2, 8, 0, 0, 8, 12, low_percent=25)
    r = c2.step(0, [1], [1], pred_ids=[0, 1, 2, 3], pred_pop=[5, 0, 3, 1])
    assert r.load_bits == [4, 4, 4, 4]               # the demand load of expert 1, then 0, 2, 3
    # demand loads always move at the cache's width
    c3 = C.CacheOracle(2, 8, 0, 0, 8, 12, low_percent=100)
    r = c3.step(0, [1], [1], pred_ids=[2, 3], pred_pop=[2, 1])
    assert r.load_bits == [4, 2, 2]
