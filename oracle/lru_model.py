"""Reference model of the two-level expert cache (TEST INFRASTRUCTURE ONLY).

Follows the paper's expert memory management (Sec. 3.3.1): two LRU tiers,
``high`` (used within the recent window of layers, or predicted to be needed
soon) and ``low`` (everything else); eviction takes the least recently used
entry of ``low`` first and falls back to ``high`` only when ``low`` has no
candidate; tiers are re-assigned whenever the look-ahead S changes.

Readings where the paper is silent (the window length is lost in the text):
an entry is ``high`` while ``clock - last_use <= S`` or while a prediction
says it is due at a tick ``>= clock``.  The clock advances once per executed
layer.  A per-layer cap restricts the candidates to the same layer once that
layer holds ``cap`` entries.  Pinned entries (needed by the layer being run)
are never evicted.  Inside ``high`` (only reached when ``low`` has no
candidate) entries that no prediction is waiting for go first, least recently
used first; if every candidate is still awaited, the one due furthest ahead
goes (latest stamp among equals).
"""
from __future__ import annotations


class TwoLevelLRU:
    def __init__(self, slots_total: int, per_layer_cap: int = 0):
        self.slots_total = slots_total
        self.cap = per_layer_cap
        self.entries = {}      # (layer, expert) -> dict(stamp, last_use, due, high, pinned)
        self.clock = 0
        self.S = 1
        self._stamp = 0
        self.evictions = []    # (layer, expert) in eviction order

    # -- helpers -----------------------------------------------------------
    def _next_stamp(self):
        self._stamp += 1
        return self._stamp

    def resident(self, layer, expert):
        return (layer, expert) in self.entries

    def tier(self, layer, expert):
        e = self.entries[(layer, expert)]
        return "high" if e["high"] else "low"

    def _is_high(self, e):
        return (self.clock - e["last_use"] <= self.S) or (e["due"] >= self.clock)

    def retier(self):
        for e in self.entries.values():
            e["high"] = self._is_high(e)

    def advance(self, S=None):
        """One layer executed; optionally a new look-ahead S.  Re-tiers everything."""
        self.clock += 1
        if S is not None:
            self.S = S
        self.retier()

    def set_S(self, S):
        self.S = S
        self.retier()

    # -- accesses ----------------------------------------------------------
    def touch(self, layer, expert):
        """The layer being executed uses this resident expert."""
        e = self.entries[(layer, expert)]
        e["stamp"] = self._next_stamp()
        e["last_use"] = self.clock
        e["high"] = True

    def pin(self, layer, expert, on=True):
        self.entries[(layer, expert)]["pinned"] = on

    def _victim(self, layer):
        keys = list(self.entries)
        in_layer = [k for k in keys if k[0] == layer]
        if self.cap and len(in_layer) >= self.cap:
            cand = in_layer
        elif len(keys) < self.slots_total:
            return None, True
        else:
            cand = keys
        cand = [k for k in cand if not self.entries[k]["pinned"]]
        if not cand:
            return None, False
        low = [k for k in cand if not self.entries[k]["high"]]
        if low:
            return min(low, key=lambda k: self.entries[k]["stamp"]), True
        idle = [k for k in cand if self.entries[k]["due"] < self.clock]
        if idle:
            return min(idle, key=lambda k: self.entries[k]["stamp"]), True
        # every candidate is awaited by a prediction: give up the one needed last
        return max(cand, key=lambda k: (self.entries[k]["due"], self.entries[k]["stamp"])), True

    def swap_in(self, layer, expert, due_in=0):
        """Make (layer, expert) resident.  due_in = layers until it is needed
        (0 = a miss of the layer being run).  Returns 'hit', 'load' or 'busy'."""
        key = (layer, expert)
        due = self.clock + due_in
        if key in self.entries:
            e = self.entries[key]
            e["stamp"] = self._next_stamp()
            e["due"] = max(e["due"], due)
            e["high"] = True
            return "hit"
        victim, ok = self._victim(layer)
        if not ok:
            return "busy"
        if victim is not None:
            del self.entries[victim]
            self.evictions.append(victim)
        self.entries[key] = dict(stamp=self._next_stamp(), last_use=self.clock if due_in == 0 else -10**9,
                                 due=due, high=True, pinned=False)
        return "load"
