"""Checker: per-layer expert cache with LRU replacement, demand loads and prefetch
(test infrastructure).

The paper keeps a bounded set of experts per layer in GPU memory (Sec. 4.4),
replaces by least-recently-used (Sec. 6.3), loads missing experts of the
current layer on demand and prefetches the experts predicted for the following
layer (Sec. 4.3, Alg.1: the transfer set is the non-resident required experts
plus the predicted ones).  The paper does not say whether a prefetch counts as
a use, nor what happens when a layer owns fewer slots than experts run; the
readings taken here:

  * sequential semantics, independent of any timing: events are ordered by
    (token, layer, demand before prefetch, rank order e1 then e2);
  * a demand hit or a prefetch of an already-resident expert makes it the most
    recently used; a demand miss or a prefetch load inserts as most recently
    used after evicting the least recently used entry if the layer is full;
  * a layer with zero slots never holds anything: its demand misses are
    "bypass" loads and nothing is prefetched for it;
  * at most min(k_hat, slots) predicted experts are prefetched, in rank order;
  * look-ahead beyond the next layer (Sec. 4.3): the predictions for layers
    l+1, l+2, ... are served in that order, and the one for layer l+d+1 is
    served only if serving layer l+d loaded nothing (all its predicted experts
    were resident; a layer without slots loads nothing either).

Events are tuples (token, layer, kind, expert, victim) with victim = -1 when
nothing was evicted.
"""
from __future__ import annotations

HIT = "HIT"            # demanded expert resident
HIT_PF = "HIT_PF"      # demanded expert resident, brought in by a prefetch and not used since
MISS = "MISS"          # demanded expert absent -> loaded on demand (victim evicted if full)
BYPASS = "BYPASS"      # demanded expert absent and the layer owns no slot
PF_TOUCH = "PF_TOUCH"  # predicted expert already resident -> recency refreshed
PF_LOAD = "PF_LOAD"    # predicted expert absent -> loaded ahead of time


class LayerLRU:
    """Ordered set of at most `cap` expert ids; index 0 is least recently used."""

    def __init__(self, cap: int):
        self.cap = int(cap)
        self.order = []          # LRU ... MRU
        self.by_prefetch = set()  # entries whose last fill was a prefetch and that were not demanded since

    def __contains__(self, e):
        return e in self.order

    def touch(self, e):
        self.order.remove(e)
        self.order.append(e)

    def insert(self, e):
        """Insert e as MRU; returns the evicted id or -1."""
        victim = -1
        if len(self.order) >= self.cap:
            victim = self.order.pop(0)
            self.by_prefetch.discard(victim)
        self.order.append(e)
        return victim


class ExpertCache:
    def __init__(self, slots_per_layer):
        self.layers = [LayerLRU(c) for c in slots_per_layer]
        self.events = []

    def demand(self, token, layer, ids, k):
        """Experts ids[0:k] of `layer` are required now (rank order)."""
        c = self.layers[layer]
        out = []
        for j in range(int(k)):
            e = int(ids[j])
            if e in c:
                kind = HIT_PF if e in c.by_prefetch else HIT
                c.by_prefetch.discard(e)
                c.touch(e)
                ev = (token, layer, kind, e, -1)
            elif c.cap == 0:
                ev = (token, layer, BYPASS, e, -1)
            else:
                victim = c.insert(e)
                ev = (token, layer, MISS, e, victim)
            out.append(ev)
        self.events.extend(out)
        return out

    def prefetch(self, token, layer, pred_ids):
        """`pred_ids` (rank order) are predicted for `layer` (the layer after the one running)."""
        c = self.layers[layer]
        out = []
        for e in list(pred_ids)[: min(len(pred_ids), c.cap)]:
            e = int(e)
            if e in c:
                c.touch(e)
                ev = (token, layer, PF_TOUCH, e, -1)
            else:
                victim = c.insert(e)
                c.by_prefetch.add(e)
                ev = (token, layer, PF_LOAD, e, victim)
            out.append(ev)
        self.events.extend(out)
        return out

    def prefetch_lookahead(self, token, layer, preds):
        """preds[d-1] = experts predicted for layer+d (d = 1, 2, ...).  Depth d+1 is served only when
        depth d found everything resident."""
        out = []
        for d, r in enumerate(preds, start=1):
            if layer + d >= len(self.layers):
                break
            evs = self.prefetch(token, layer + d, r)
            out.extend(evs)
            if any(ev[2] == PF_LOAD for ev in evs):
                break
        return out

    def resident(self, layer):
        return list(self.layers[layer].order)


def summarise(events):
    """Counts per kind, on-demand loads (MISS + BYPASS) and prefetch usefulness."""
    n = {}
    for ev in events:
        n[ev[2]] = n.get(ev[2], 0) + 1
    demand = sum(n.get(k, 0) for k in (HIT, HIT_PF, MISS, BYPASS))
    loads = n.get(MISS, 0) + n.get(BYPASS, 0)
    return dict(counts=n, demand=demand, on_demand_loads=loads,
                hit_rate=(1.0 - loads / demand) if demand else 0.0,
                prefetch_loads=n.get(PF_LOAD, 0), prefetch_useful=n.get(HIT_PF, 0))
