"""Hand traces for the two-level LRU reference model (paper Sec. 3.3.1).

Expected values below are worked out by hand from the stated rules, not
produced by running the model.
"""
from oracle.lru_model import TwoLevelLRU


def test_low_tier_is_evicted_before_high():
    c = TwoLevelLRU(4)
    c.S = 1
    # tick 0: layer 0 misses on experts 0,1 (used now); prefetch (1,2) due next layer, (3,7) due in 3 layers
    assert c.swap_in(0, 0) == "load" and c.swap_in(0, 1) == "load"
    assert c.swap_in(1, 2, due_in=1) == "load" and c.swap_in(3, 7, due_in=3) == "load"
    assert all(c.tier(*k) == "high" for k in [(0, 0), (0, 1), (1, 2), (3, 7)])
    c.advance()           # tick 1: everything still inside the window S=1 or still due
    c.advance()           # tick 2: (0,0),(0,1) last used at tick 0 -> 2 > S -> low; (1,2) was due at tick 1 -> low
    assert c.tier(0, 0) == "low" and c.tier(0, 1) == "low" and c.tier(1, 2) == "low"
    assert c.tier(3, 7) == "high"
    # a miss now takes the least recently stamped LOW entry: (0,0), not the older-or-newer HIGH one
    assert c.swap_in(2, 5) == "load"
    assert c.evictions == [(0, 0)]
    assert c.swap_in(2, 6) == "load"
    assert c.evictions == [(0, 0), (0, 1)]
    assert c.swap_in(2, 4) == "load"
    assert c.evictions == [(0, 0), (0, 1), (1, 2)]
    # only high entries remain and all are awaited: the three misses are due now (tick 2),
    # (3,7) is due at tick 3, furthest ahead, so it is the one given up
    assert c.swap_in(2, 3) == "load"
    assert c.evictions[-1] == (3, 7)


def test_touch_promotes_and_refreshes_recency():
    c = TwoLevelLRU(3)
    c.S = 1
    for e in (0, 1, 2):
        c.swap_in(0, e)
    c.advance()
    c.advance()                       # all low now
    assert [c.tier(0, e) for e in (0, 1, 2)] == ["low"] * 3
    c.touch(0, 0)                     # reuse promotes the oldest entry
    assert c.tier(0, 0) == "high"
    assert c.swap_in(1, 9) == "load"
    assert c.evictions == [(0, 1)]    # (0,0) was older but is high now
    assert c.swap_in(0, 0, due_in=2) == "hit"
    assert c.resident(0, 0)


def test_retier_when_lookahead_changes():
    c = TwoLevelLRU(4)
    c.S = 1
    c.swap_in(0, 0)
    c.advance()
    c.advance()
    c.advance()                       # clock 3, last_use 0 -> low under S=1
    assert c.tier(0, 0) == "low"
    c.set_S(3)                        # window grows: 3 - 0 <= 3 -> high again
    assert c.tier(0, 0) == "high"
    c.set_S(2)
    assert c.tier(0, 0) == "low"


def test_per_layer_cap_and_pinning():
    c = TwoLevelLRU(8, per_layer_cap=2)
    assert c.swap_in(0, 0) == "load" and c.swap_in(0, 1) == "load"
    c.pin(0, 0)
    c.pin(0, 1)
    assert c.swap_in(0, 2) == "busy"            # layer full and both pinned
    c.pin(0, 0, False)
    assert c.swap_in(0, 2) == "load"
    assert c.evictions == [(0, 0)]              # never another layer's entry, never the pinned one
    assert c.swap_in(1, 0) == "load" and len(c.entries) == 3


def test_thrash_when_lookahead_working_set_exceeds_capacity():
    """Prefetching further ahead than the pool can hold evicts entries before they are used, so
    the same experts are transferred more than once (the latency jump the paper reports once
    capacity is exceeded, Sec. 4.4).  3 experts per layer, 10 slots: a look-ahead of H needs
    3*(H+1) slots, which fits for H <= 2 and not for H = 4."""
    def run(H, slots=10, per_layer=3, layers=12):
        c = TwoLevelLRU(slots)
        c.S = H
        loads = 0
        for l in range(layers):
            for j in range(1, H + 1):
                for e in range(per_layer):
                    loads += c.swap_in(l + j, e, due_in=j) == "load"
            for e in range(per_layer):
                loads += c.swap_in(l, e) == "load"
                c.touch(l, e)
            c.advance()
        return loads
    assert run(1) == 3 * (12 + 1) and run(2) == 3 * (12 + 2)      # every expert moved exactly once
    assert run(4) > 3 * (12 + 4)


def test_pool_victim_follows_the_layer_cycle_and_the_per_layer_share():
    """One pool of 8 slots for 4 layers that run cyclically (share: 2 per layer), top_k = 1, window S = 1.
    Worked out by hand from the stated order: a layer at its share replaces its own; otherwise most crowded
    layer (above top_k) first, then the layer whose next turn is furthest away, then least recently used."""
    c = TwoLevelLRU(8, n_layers=4, top_k=1)
    c.S = 1
    for layer, experts in ((0, (0, 1, 2)), (1, (0, 1, 2)), (2, (0, 1))):     # ticks 0, 1, 2; the pool is full after them
        for e in experts:
            assert c.swap_in(layer, e) == "load"
            c.touch(layer, e)
        c.advance(layer_run=layer)
    # tick 3, layer 3 runs next.  Layers 0 and 1 were last used 3 and 2 ticks ago: low.  Layer 2: 1 tick ago: high.
    assert [c.tier(l, 0) for l in (0, 1, 2)] == ["low", "low", "high"]
    # layer 3 holds nothing.  Both low layers hold three entries.  After layer 3 the cycle continues with layer 0
    # (1 turn away), then layer 1 (2 turns away): layer 1 is needed later, its least recently used entry goes.
    # Plain recency order would have taken (0, 0), the expert needed soonest.
    assert c.swap_in(3, 5) == "load"
    assert c.evictions == [(1, 0)]
    # layer 3 holds one, still below its share; layer 0 (three entries) is more crowded than layer 1 (two) now
    assert c.swap_in(3, 6) == "load"
    assert c.evictions == [(1, 0), (0, 0)]
    # layer 3 has its share of the full pool: a third expert replaces one of its own.  Both are awaited now
    # (due at this tick): the later one goes.
    assert c.swap_in(3, 7) == "load"
    assert c.evictions == [(1, 0), (0, 0), (3, 6)]


def test_pool_rule_needs_no_cycle_when_a_per_layer_cap_is_in_force():
    """With a cap the candidates all belong to the layer being filled: least recently used, whatever the cycle."""
    c = TwoLevelLRU(8, per_layer_cap=2, n_layers=4, top_k=1)
    c.S = 1
    assert c.swap_in(2, 0) == "load" and c.swap_in(2, 1) == "load"
    c.touch(2, 1)
    c.touch(2, 0)                                  # (2, 1) is the older use now
    c.advance(layer_run=2)
    assert c.swap_in(2, 5) == "load"
    assert c.evictions == [(2, 1)]
