"""Checker: per-layer expert cache with LRU replacement, demand loads and prefetch
(test infrastructure).

The paper keeps a bounded set of experts per layer in GPU memory (Sec. 4.4),
replaces by least-recently-used (Sec. 6.3), loads missing experts of the
current layer on demand and prefetches the experts predicted for the following
layer (Sec. 4.3, Alg.1: the transfer set is the non-resident required experts
plus the predicted ones).  The paper does not say whether a prefetch counts as
a use, nor where a prefetched expert goes when the layer owns fewer slots than
experts are predicted; the readings taken here:

  * sequential semantics, independent of any timing: events are ordered by
    (token, layer, demand before prefetch, rank order e1 then e2);
  * a demand hit or a prefetch of an already-resident expert makes it the most
    recently used; a demand miss or a prefetch load inserts as most recently
    used after evicting the least recently used entry if the layer is full;
  * a layer with zero slots never keeps anything: its demand misses are
    "bypass" loads;
  * a prefetch always has somewhere to land.  The on-demand-load model of
    Sec. 4.4.2 (Eq.11-14) counts a load only when the prefetch was wrong, also
    for a layer with no slot at all (Eq.11 at t = 0 is 1 - beta), so a
    predicted expert that cannot be given one of the layer's own slots - the
    layer has none, or the same prefetch has already filled or refreshed as
    many slots as the layer owns (it never evicts an expert predicted together
    with it) - is copied into a landing buffer outside the cache budget
    (PF_LAND).  It stays there until the layer's next demand: if it is then
    required it counts as a prefetch hit and, when the layer owns slots, moves
    into the layer's set as most recently used (evicting the least recently
    used entry, no load needed); whatever was not required is dropped;
  * look-ahead beyond the next layer (Sec. 4.3): the predictions for layers
    l+1, l+2, ... are served in that order, and the one for layer l+d+1 is
    served only if serving layer l+d loaded nothing (all its predicted experts
    were resident).  Only the prediction for the next layer may use landing
    buffers; a deeper one fills at most as many experts as the layer owns slots.

Events are tuples (token, layer, kind, expert, victim) with victim = -1 when
nothing was evicted.
"""
from __future__ import annotations

HIT = "HIT"            # demanded expert resident
HIT_PF = "HIT_PF"      # demanded expert resident (or in a landing buffer), brought in by a prefetch and not used since
MISS = "MISS"          # demanded expert absent -> loaded on demand (victim evicted if full)
BYPASS = "BYPASS"      # demanded expert absent and the layer owns no slot
PF_TOUCH = "PF_TOUCH"  # predicted expert already on the GPU -> recency refreshed
PF_LOAD = "PF_LOAD"    # predicted expert absent -> loaded ahead of time into one of the layer's slots
PF_LAND = "PF_LAND"    # predicted expert absent, no slot of the layer free for it -> loaded into a landing buffer


class LayerLRU:
    """Ordered set of at most `cap` expert ids; index 0 is least recently used.  `landing` holds
    prefetched experts kept outside the budget until the layer's next demand."""

    def __init__(self, cap: int):
        self.cap = int(cap)
        self.order = []          # LRU ... MRU
        self.by_prefetch = set()  # entries whose last fill was a prefetch and that were not demanded since
        self.landing = []

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

    def demand(self, token, layer, ids, k, release=True):
        """Experts ids[0:k] of `layer` are required now (rank order).  release=False keeps the
        layer's landing buffers for further tokens of the same step (call release_landing after
        the last one)."""
        c = self.layers[layer]
        out = []
        for j in range(int(k)):
            e = int(ids[j])
            if e in c:
                kind = HIT_PF if e in c.by_prefetch else HIT
                c.by_prefetch.discard(e)
                c.touch(e)
                ev = (token, layer, kind, e, -1)
            elif e in c.landing:
                c.landing.remove(e)
                victim = c.insert(e) if c.cap > 0 else -1
                ev = (token, layer, HIT_PF, e, victim)
            elif c.cap == 0:
                ev = (token, layer, BYPASS, e, -1)
            else:
                victim = c.insert(e)
                ev = (token, layer, MISS, e, victim)
            out.append(ev)
        self.events.extend(out)
        if release:
            self.release_landing(layer)
        return out

    def release_landing(self, layer):
        """End of a step of `layer`: prefetched experts that were not required are dropped."""
        self.layers[layer].landing = []

    def prefetch(self, token, layer, pred_ids, landing=True):
        """`pred_ids` (rank order) are predicted for `layer`.  At most as many of them as the layer
        owns slots are refreshed in or loaded into its set; the others go to landing buffers
        (landing=True, the prediction for the next layer) or are left out (deeper look-ahead)."""
        c = self.layers[layer]
        out = []
        own = 0
        for e in pred_ids:
            e = int(e)
            if e in c.landing:
                ev = (token, layer, PF_TOUCH, e, -1)
            elif own < c.cap:
                own += 1
                if e in c:
                    c.touch(e)
                    ev = (token, layer, PF_TOUCH, e, -1)
                else:
                    victim = c.insert(e)
                    c.by_prefetch.add(e)
                    ev = (token, layer, PF_LOAD, e, victim)
            elif not landing:
                continue
            elif e in c:     # only when the caller lists an expert twice: it is on the GPU already
                c.touch(e)
                ev = (token, layer, PF_TOUCH, e, -1)
            else:
                c.landing.append(e)
                ev = (token, layer, PF_LAND, e, -1)
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
            evs = self.prefetch(token, layer + d, r, landing=(d == 1))
            out.extend(evs)
            if any(ev[2] in (PF_LOAD, PF_LAND) for ev in evs):
                break
        return out

    def resident(self, layer):
        return list(self.layers[layer].order)

    def landed(self, layer):
        return list(self.layers[layer].landing)


def summarise(events):
    """Counts per kind, on-demand loads (MISS + BYPASS) and prefetch usefulness."""
    n = {}
    for ev in events:
        n[ev[2]] = n.get(ev[2], 0) + 1
    demand = sum(n.get(k, 0) for k in (HIT, HIT_PF, MISS, BYPASS))
    loads = n.get(MISS, 0) + n.get(BYPASS, 0)
    return dict(counts=n, demand=demand, on_demand_loads=loads,
                hit_rate=(1.0 - loads / demand) if demand else 0.0,
                prefetch_loads=n.get(PF_LOAD, 0) + n.get(PF_LAND, 0), prefetch_landed=n.get(PF_LAND, 0),
                prefetch_useful=n.get(HIT_PF, 0))
