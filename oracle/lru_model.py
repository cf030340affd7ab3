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

One pool for all layers (no per-layer cap in force): a decode loop visits the
layers cyclically, so plain recency order would evict what runs next (the
premature eviction of the first layers' experts the section gives as the
motivation of the two tiers).  Once the pool is full, a layer that already
holds its share of it (``slots_total // n_layers``, at least ``top_k``) replaces
its own entries, as under a per-layer cap.  A layer below its share takes, among
the candidates of a tier, the victim from the layer holding the most entries,
provided that is more than ``top_k``; equal there, from the layer whose next
turn in the cycle is furthest away; equal there, the least recently used.
``advance(layer_run)`` tells the model which layer just ran.
"""
from __future__ import annotations


class TwoLevelLRU:
    def __init__(self, slots_total: int, per_layer_cap: int = 0, n_layers: int = 1, top_k: int = 1):
        self.slots_total = slots_total
        self.cap = per_layer_cap
        self.n_layers = n_layers
        self.top_k = top_k
        self.next_layer = 0
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

    def advance(self, S=None, layer_run=None):
        """One layer executed (layer_run: which one); optionally a new look-ahead S.  Re-tiers everything."""
        self.clock += 1
        if layer_run is not None:
            self.next_layer = (layer_run + 1) % self.n_layers
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
        pooled = False
        if self.cap and len(in_layer) >= self.cap:
            cand = in_layer
        elif len(keys) < self.slots_total:
            return None, True
        elif len(in_layer) >= max(self.top_k, self.slots_total // self.n_layers):
            cand = in_layer              # full pool and the layer has its share: it replaces its own
        else:
            cand = keys
            pooled = True
        cand = [k for k in cand if not self.entries[k]["pinned"]]
        if not cand:
            return None, False

        def order(k):
            """Smallest goes first."""
            if not pooled:
                return (0, 0, self.entries[k]["stamp"])
            held = sum(1 for q in keys if q[0] == k[0])
            crowd = held if held > self.top_k else 0
            turn = (k[0] - self.next_layer) % self.n_layers
            return (-crowd, -turn, self.entries[k]["stamp"])

        low = [k for k in cand if not self.entries[k]["high"]]
        if low:
            return min(low, key=order), True
        idle = [k for k in cand if self.entries[k]["due"] < self.clock]
        if idle:
            return min(idle, key=order), True
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
