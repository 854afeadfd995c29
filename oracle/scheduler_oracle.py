"""TEST INFRASTRUCTURE - plain Python statement of the Expert Scheduler's decisions, paper
section 3.3 (Expert Lookahead Buffer, three-phase prefetch, lookahead-aware eviction, on-demand
misses).  Only tests, smoke() and bench.py's baseline leg may import this module.

The paper leaves the policy details open; the readings are those documented at
moe_sched_plan / moe_sched_on_demand and are restated at each function here.  Data structures are
dictionaries and lists on purpose: nothing is shared with the library's implementation.
"""
from typing import Dict, List, Optional, Sequence, Tuple


class Cache:
    """Per layer: slot -> expert (None = empty), expert -> time of last use."""

    def __init__(self, n_layers: int, n_experts: int, n_slots: int):
        self.L, self.E, self.C = n_layers, n_experts, n_slots
        self.slots: List[List[Optional[int]]] = [[None] * n_slots for _ in range(n_layers)]
        self.last: List[Dict[int, int]] = [dict() for _ in range(n_layers)]
        self.protected: List[set] = [set() for _ in range(n_layers)]
        self.clock = 0
        self.hits = 0
        self.misses = 0

    def resident(self, layer: int):
        return {e for e in self.slots[layer] if e is not None}

    def place(self, layer: int, expert: int, slot: int):
        assert self.slots[layer][slot] is None and expert not in self.resident(layer)
        self.slots[layer][slot] = expert

    def slot_table(self, layer: int):
        t = [-1] * self.E
        for s, e in enumerate(self.slots[layer]):
            if e is not None:
                t[e] = s
        return t

    def use(self, layer: int, ids: Sequence[int]):
        """Section 4.4's per-step cache coverage: of the distinct experts the step needs, how many
        are resident when it starts."""
        self.clock += 1
        need = set(ids)
        res = self.resident(layer)
        hit = len(need & res)
        miss = len(need - res)
        for e in need:
            self.last[layer][e] = self.clock
        self.hits += hit
        self.misses += miss
        return hit, miss

    def end_window(self):
        self.protected = [set() for _ in range(self.L)]

    def _choose(self, layer: int, evictable):
        """Lowest empty slot; else the least recently used resident expert that may be evicted
        (never-used counts as oldest; ties go to the lowest slot); None if there is none."""
        for s, e in enumerate(self.slots[layer]):
            if e is None:
                return s
        best = None
        for s, e in enumerate(self.slots[layer]):
            if not evictable(e):
                continue
            key = self.last[layer].get(e, 0)
            if best is None or key < best[0]:
                best = (key, s)
        return None if best is None else best[1]

    def _install(self, layer: int, expert: int, slot: int):
        old = self.slots[layer][slot]
        self.slots[layer][slot] = expert
        return (layer, expert, slot, -1 if old is None else old)

    def plan(self, elb: Sequence[Sequence[Sequence[Tuple[int, float]]]], phase: int, max_fetch: int = 0,
             min_conf: float = 0.0):
        """elb[step][layer] = [(expert, confidence), ...].  Phase I (1): protect what the window
        names, fetch nothing.  Phase II (2): missing named experts by (layer, confidence
        descending, expert id), confidence >= min_conf, at most max_fetch.  Phase III (3): all
        missing named experts by (layer, expert id).  An expert named by the window is never
        evicted by the plan (Belady on the lookahead: it is needed sooner than any expert the
        window does not name); among the others the least recently used goes."""
        conf: List[Dict[int, float]] = [dict() for _ in range(self.L)]
        for step in elb:
            for layer, entries in enumerate(step):
                for e, cf in entries:
                    conf[layer][e] = max(conf[layer].get(e, -1.0), cf)
        cand = []
        for layer in range(self.L):
            self.protected[layer] |= set(conf[layer])
            if phase == 1:
                continue
            missing = [e for e in sorted(conf[layer]) if e not in self.resident(layer)]
            if phase == 2:
                missing = [e for e in missing if conf[layer][e] >= min_conf]
                missing.sort(key=lambda e: (-conf[layer][e], e))
            cand += [(layer, e) for e in missing]
        if phase == 2:
            cand = cand[:max(max_fetch, 0)]
        out = []
        for layer, e in cand:
            slot = self._choose(layer, lambda x: x not in self.protected[layer])
            if slot is None:
                continue
            out.append(self._install(layer, e, slot))
        return out

    def on_demand(self, layer: int, missing: Sequence[int]):
        """Experts the verify call found absent: each takes an empty slot or replaces the least
        recently used expert that is not itself one of the incoming ones."""
        incoming = set(missing)
        out = []
        for e in missing:
            slot = self._choose(layer, lambda x: x not in incoming)
            out.append(self._install(layer, e, slot))
        return out
