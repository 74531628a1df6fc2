"""Pins for the CPU checker: each check uses something other than the checker
itself (hand-worked fixtures, closed forms, brute force, exhaustive
enumeration, a textbook reference string)."""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import cache as OC
from oracle import expert as OE
from oracle import gate as OG
from oracle import planner as OP
from oracle import stack as OS

LN = {"ln2": math.log(2), "ln3": math.log(3), "ln6": math.log(6),
      "ln6-2": math.log(6) - 2, "ln3-1": math.log(3) - 1, "-2-ln3": -2 - math.log(3)}


def _num(v):
    return LN[v] if isinstance(v, str) else float(v)


def _mat(rows):
    return np.array([[_num(v) for v in r] for r in rows])


def _load(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


# ------------------------------------------------------------------ gate ----

def test_gate_worked_example(golden_dir):
    g = _load(golden_dir, "gate_worked_example.json")
    x = np.array(g["x"])
    Wg = _mat(g["Wg_rows"])
    z = OG.router_logits(x, Wg)
    np.testing.assert_allclose(z, [_num(v) for v in g["logits"]], atol=1e-14)
    p = OG.softmax(z)
    np.testing.assert_allclose(p, np.array(g["softmax_num"]) / g["softmax_den"], rtol=1e-14)
    for case in g["cases"]:
        tau = OG.tau_from_sensitivity(case["T"], g["S"])
        r = OG.adaptive_gate(x, Wg, tau)
        assert r["ids"] == (g["top1"], g["top2"])
        assert abs(r["alpha"] - g["alpha"]) < 1e-14 and abs(r["v"] - g["v"]) < 1e-14
        assert r["k"] == case["k"]
        np.testing.assert_allclose(r["w"], case["w"], atol=1e-14)
        # Eq.8 in its printed form decides the same
        assert OG.single_expert_eq8(r["alpha"], g["S"], case["T"]) == (case["k"] == 1)


def test_gate_invariants_random():
    rng = np.random.default_rng(7)
    for trial in range(200):
        N = int(rng.integers(2, 10))
        H = int(rng.integers(1, 40))
        x = rng.standard_normal(H)
        Wg = rng.standard_normal((N, H))
        z = Wg @ x
        order = np.argsort(-z, kind="stable")
        r0 = OG.adaptive_gate(x, Wg, 0.0)
        # threshold 0 is fixed top-2: both experts run, weights from a softmax over the two logits
        assert r0["k"] == 2 and r0["ids"] == (order[0], order[1])
        a_closed = 1.0 / (1.0 + math.exp(z[order[1]] - z[order[0]]))
        assert abs(r0["w"][0] - a_closed) < 1e-12 and abs(sum(r0["w"]) - 1.0) < 1e-12
        assert r0["alpha"] >= 0.5
        # threshold >= 1/2 is top-1 with weight exactly 1 (Eq.4)
        r1 = OG.adaptive_gate(x, Wg, 0.5)
        assert r1["k"] == 1 and r1["w"] == (1.0, 0.0) and r1["ids"][0] == order[0]
        # monotone in the threshold, ids independent of it
        ks = [OG.adaptive_gate(x, Wg, t)["k"] for t in np.linspace(0, 0.5, 11)]
        assert all(b <= a for a, b in zip(ks, ks[1:]))
        # the printed Eq.8 and the threshold form agree for random S, T
        S, T = float(rng.uniform(0.1, 10)), float(rng.uniform(0.001, 1))
        rt = OG.adaptive_gate(x, Wg, OG.tau_from_sensitivity(T, S))
        if abs((1 - rt["alpha"]) ** 2 * S - T) > 1e-9:
            assert (rt["k"] == 1) == OG.single_expert_eq8(rt["alpha"], S, T)


def test_gate_tie_break_lower_index():
    Wg = np.array([[1.0], [2.0], [2.0], [1.0]])
    r = OG.adaptive_gate(np.array([1.0]), Wg, 0.0)
    assert r["ids"] == (1, 2) and abs(r["alpha"] - 0.5) < 1e-15
    r = OG.adaptive_gate(np.array([-1.0]), Wg, 0.0)
    assert r["ids"] == (0, 3)


def test_gate_constant_sensitivity_is_score_based():
    # with the same sensitivity in every layer the test depends on alpha only (Sec. 4.2, last paragraph)
    rng = np.random.default_rng(3)
    for _ in range(50):
        x, Wg = rng.standard_normal(8), rng.standard_normal((5, 8))
        alpha = OG.adaptive_gate(x, Wg, 0.0)["alpha"]
        T, S = 0.09, 1.0
        assert OG.single_expert_eq8(alpha, S, T) == (alpha >= 1 - 0.3) or abs(alpha - 0.7) < 1e-9


def test_predictor_is_next_layers_gate_on_same_input():
    rng = np.random.default_rng(11)
    x = rng.standard_normal(16)
    Wn = rng.standard_normal((8, 16))
    for tau in (0.0, 0.2, 0.5):
        g = OG.adaptive_gate(x, Wn, tau)
        assert OG.predict_next(x, Wn, tau) == list(g["ids"][: g["k"]])


def test_gate_batch_matches_python_loops():
    rng = np.random.default_rng(5)
    X, Wg = rng.standard_normal((9, 6)), rng.standard_normal((4, 6))
    out = OG.gate_batch(X, Wg, 0.3)
    for b in range(9):
        z = [sum(X[b][h] * Wg[i][h] for h in range(6)) for i in range(4)]
        m = max(z)
        e = [math.exp(v - m) for v in z]
        p = [v / sum(e) for v in e]
        i1 = max(range(4), key=lambda i: (p[i], -i))
        i2 = max((i for i in range(4) if i != i1), key=lambda i: (p[i], -i))
        v = p[i2] / (p[i1] + p[i2])
        assert tuple(out["ids"][b]) == (i1, i2)
        assert out["k"][b] == (1 if v <= 0.3 else 2)
        assert abs(out["v"][b] - v) < 1e-13


# ---------------------------------------------------------------- expert ----

def test_ffn_worked_example(golden_dir):
    g = _load(golden_dir, "ffn_worked_example.json")
    x = np.array(g["x"])
    W1, W3, W2, W2b = _mat(g["W1"]), _mat(g["W3"]), _mat(g["W2"]), _mat(g["W2b"])
    ln3 = math.log(3)
    E = OE.expert_ffn(x, W1, W3, W2)
    Eb = OE.expert_ffn(x, W1, W3, W2b)
    np.testing.assert_allclose(E / ln3, g["E_over_ln3"], rtol=1e-13)
    np.testing.assert_allclose(Eb / ln3, g["Eb_over_ln3"], rtol=1e-13)
    a = g["alpha"]
    y = OE.moe_block(x, [(W1, W3, W2), (W1, W3, W2b)], (0, 1), (a, 1 - a), 2)
    np.testing.assert_allclose(y / ln3, g["y_over_ln3"], rtol=1e-13)
    # Eq.4: a single activated expert contributes with weight one
    y1 = OE.moe_block(x, [(W1, W3, W2), (W1, W3, W2b)], (1, 0), (1.0, 0.0), 1)
    np.testing.assert_allclose(y1 / ln3, g["Eb_over_ln3"], rtol=1e-13)


def test_ffn_brute_force_loops():
    rng = np.random.default_rng(2)
    H, F = 5, 7
    x = rng.standard_normal(H)
    W1, W3, W2 = rng.standard_normal((F, H)), rng.standard_normal((F, H)), rng.standard_normal((H, F))
    a = []
    for f in range(F):
        g = sum(W1[f][h] * x[h] for h in range(H))
        u = sum(W3[f][h] * x[h] for h in range(H))
        a.append(g / (1.0 + math.exp(-g)) * u)
    y = [sum(W2[h][f] * a[f] for f in range(F)) for h in range(H)]
    np.testing.assert_allclose(OE.expert_ffn(x, W1, W3, W2), y, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(OE.expert_ffn_rows(x[None], W1, W3, W2)[0], y, rtol=1e-12, atol=1e-14)


def test_ffn_properties():
    rng = np.random.default_rng(4)
    H, F = 6, 9
    x = rng.standard_normal(H)
    W1, W3, W2 = rng.standard_normal((F, H)), rng.standard_normal((F, H)), rng.standard_normal((H, F))
    assert OE.silu(0.0) == 0.0
    assert np.all(OE.expert_ffn(np.zeros(H), W1, W3, W2) == 0.0)
    # linear in W2 and in W3, odd-symmetric pieces: silu(g) - silu(-g) = g
    np.testing.assert_allclose(OE.expert_ffn(x, W1, W3, 2 * W2), 2 * OE.expert_ffn(x, W1, W3, W2), rtol=1e-13)
    np.testing.assert_allclose(OE.expert_ffn(x, W1, 3 * W3, W2), 3 * OE.expert_ffn(x, W1, W3, W2), rtol=1e-13)
    g = rng.standard_normal(20)
    np.testing.assert_allclose(OE.silu(g) - OE.silu(-g), g, rtol=1e-13, atol=1e-15)
    # large positive gate: silu(g) -> g, so E(x) -> W2 ((W1 x) * (W3 x))
    W1big = np.abs(W1) * 50 + 40
    xpos = np.abs(x) + 1
    np.testing.assert_allclose(OE.expert_ffn(xpos, W1big, W3, W2), W2 @ ((W1big @ xpos) * (W3 @ xpos)), rtol=1e-12)


def test_moe_rows_equals_per_token_loop():
    rng = np.random.default_rng(6)
    H, F, N, B = 8, 12, 4, 10
    experts = [(rng.standard_normal((F, H)), rng.standard_normal((F, H)), rng.standard_normal((H, F))) for _ in range(N)]
    Wg = rng.standard_normal((N, H))
    X = rng.standard_normal((B, H))
    g = OG.gate_batch(X, Wg, 0.25)
    assert set(g["k"]) == {1, 2}
    Y = OE.moe_block_rows(X, experts, g["ids"], g["w"], g["k"])
    for b in range(B):
        np.testing.assert_allclose(Y[b], OE.moe_block(X[b], experts, g["ids"][b], g["w"][b], g["k"][b]), rtol=1e-12, atol=1e-13)


def test_int4_decode_hand_values():
    # codes 0..15 with scale 0.5 and zero -2 decode to -2, -1.5, ..., 5.5; second group scale 0.25 zero 1
    codes = np.arange(128).reshape(1, 128) % 16
    scale = np.array([[0.5, 0.25]], dtype=np.float16)
    zero = np.array([[-2.0, 1.0]], dtype=np.float16)
    w = OE.decode_int4(codes, scale, zero, group=64)
    exp0 = -2.0 + 0.5 * (np.arange(64) % 16)
    exp1 = 1.0 + 0.25 * (np.arange(64) % 16)
    np.testing.assert_array_equal(w[0, :64], exp0)
    np.testing.assert_array_equal(w[0, 64:], exp1)
    packed = np.array([[0x21, 0xF0]], dtype=np.uint8)
    np.testing.assert_array_equal(OE.unpack_nibbles(packed), [[1, 2, 0, 15]])


def test_two_bit_decode_hand_values():
    # the same decode with 2-bit codes (Sec. 6.3, 2-bit MoE blocks): 0..3 with scale 0.5, zero -1 -> -1, -0.5, 0, 0.5
    codes = np.arange(64).reshape(1, 64) % 4
    w = OE.decode_int4(codes, np.array([[0.5]], dtype=np.float16), np.array([[-1.0]], dtype=np.float16), group=64)
    np.testing.assert_array_equal(w[0, :8], [-1.0, -0.5, 0.0, 0.5, -1.0, -0.5, 0.0, 0.5])
    # a quantised expert evaluated from decoded weights equals the one evaluated from the formula per element
    rng = np.random.default_rng(3)
    q = rng.integers(0, 4, (2, 128))
    sc = rng.uniform(0.01, 0.1, (2, 2)).astype(np.float16)
    zr = rng.uniform(-0.1, 0.0, (2, 2)).astype(np.float16)
    x = rng.standard_normal(128)
    ref = [sum((float(q[r, c]) * float(sc[r, c // 64]) + float(zr[r, c // 64])) * x[c] for c in range(128)) for r in range(2)]
    np.testing.assert_allclose(OE.decode_int4(q, sc, zr) @ x, ref, rtol=1e-12)


# ----------------------------------------------------------------- cache ----

class _StampLRU:
    """Independent LRU: last-use timestamps, evict the smallest."""

    def __init__(self, cap):
        self.cap, self.stamp, self.clock = cap, {}, 0

    def access(self, e):
        self.clock += 1
        if e in self.stamp:
            self.stamp[e] = self.clock
            return True, -1
        victim = -1
        if self.cap == 0:
            return False, -1
        if len(self.stamp) >= self.cap:
            victim = min(self.stamp, key=self.stamp.get)
            del self.stamp[victim]
        self.stamp[e] = self.clock
        return False, victim


def test_lru_textbook_reference_string(golden_dir):
    g = _load(golden_dir, "lru_reference_string.json")
    c = OC.ExpertCache([g["frames"]])
    for n, page in enumerate(g["reference_string"]):
        c.demand(n, 0, [page], 1)
    faults = sum(1 for ev in c.events if ev[2] == OC.MISS)
    assert faults == g["lru_faults"]


def test_lru_exhaustive_against_timestamp_simulator():
    for cap in range(0, 4):
        for length in range(1, 7):
            for trace in itertools.product(range(3), repeat=length):
                c = OC.ExpertCache([cap])
                ref = _StampLRU(cap)
                for n, e in enumerate(trace):
                    ev = c.demand(n, 0, [e], 1)[0]
                    hit, victim = ref.access(e)
                    assert (ev[2] in (OC.HIT, OC.HIT_PF)) == hit
                    assert ev[4] == victim
                    assert (ev[2] == OC.BYPASS) == (cap == 0)
                assert sorted(c.resident(0)) == sorted(ref.stamp)


def test_lru_inclusion_and_capacity_properties():
    rng = np.random.default_rng(9)
    trace = rng.integers(0, 8, size=400)
    misses = []
    for cap in range(0, 9):
        c = OC.ExpertCache([cap])
        for n, e in enumerate(trace):
            c.demand(n, 0, [int(e)], 1)
        misses.append(sum(ev[2] in (OC.MISS, OC.BYPASS) for ev in c.events))
    assert misses[0] == len(trace)                       # no slot: always loads
    assert misses[8] == len(set(trace.tolist()))         # room for every expert: only first touches miss
    assert all(b <= a for a, b in zip(misses, misses[1:]))   # LRU stack (inclusion) property


def test_cache_prefetch_hand_trace(golden_dir):
    g = _load(golden_dir, "cache_prefetch_trace.json")
    c = OC.ExpertCache(g["slots"])
    for s in g["steps"]:
        c.demand(s["token"], s["layer"], s["demand"], s["k"])
        if s["layer"] + 1 < len(g["slots"]):
            c.prefetch(s["token"], s["layer"] + 1, s["pred_for_next"])
    assert [list(e) for e in c.events] == g["events"]
    assert [c.resident(l) for l in range(len(g["slots"]))] == g["final_resident"]
    s = OC.summarise(c.events)
    assert s["on_demand_loads"] == 4 and s["prefetch_loads"] == 2 and s["prefetch_useful"] == 2


def test_cache_lookahead_hand_trace(golden_dir):
    g = _load(golden_dir, "cache_lookahead_trace.json")
    c = OC.ExpertCache(g["slots"])
    for s in g["steps"]:
        c.demand(s["token"], s["layer"], s["demand"], s["k"])
        c.prefetch_lookahead(s["token"], s["layer"], s["ahead"])
    assert [list(e) for e in c.events] == g["events"]
    assert [c.resident(l) for l in range(len(g["slots"]))] == g["final_resident"]


def test_cache_lookahead_depth_one_is_plain_prefetch_and_deeper_never_loads_after_a_load():
    rng = np.random.default_rng(5)
    L, N = 5, 6
    slots = [2, 0, 3, 1, 2]
    a, b, d3 = OC.ExpertCache(slots), OC.ExpertCache(slots), OC.ExpertCache(slots)
    for n in range(80):
        for l in range(L):
            ids = rng.choice(N, size=2, replace=False)
            k = int(rng.integers(1, 3))
            ahead = [list(rng.choice(N, size=int(rng.integers(1, 3)), replace=False)) for _ in range(3)]
            a.demand(n, l, ids, k)
            b.demand(n, l, ids, k)
            d3.demand(n, l, ids, k)
            if l + 1 < L:
                a.prefetch(n, l + 1, ahead[0])
            b.prefetch_lookahead(n, l, ahead[:1])
            evs = d3.prefetch_lookahead(n, l, ahead)
            # within one step: layers appear in increasing order, nothing beyond the stack, and
            # only the deepest layer served may contain a load
            layers = [ev[1] for ev in evs]
            assert layers == sorted(layers) and all(l < x < L for x in layers)
            for ev in evs:
                if ev[2] in (OC.PF_LOAD, OC.PF_LAND):
                    assert ev[1] == max(layers)
                if ev[2] == OC.PF_LAND:
                    assert ev[1] == l + 1      # only the prediction for the next layer uses landing buffers
    assert a.events == b.events


class _StampCacheWithLanding:
    """Independent model of one layer: last-use timestamps for the layer's own slots plus a set of
    landed experts that lives until the end of the next demand."""

    def __init__(self, cap):
        self.cap, self.stamp, self.clock, self.landed = cap, {}, 0, set()

    def _use(self, e):
        self.clock += 1
        self.stamp[e] = self.clock

    def _make_room(self):
        if len(self.stamp) >= self.cap:
            del self.stamp[min(self.stamp, key=self.stamp.get)]

    def demand(self, ids):
        loads = 0
        for e in ids:
            if e in self.stamp:
                self._use(e)
            elif e in self.landed:
                self.landed.discard(e)
                if self.cap:
                    self._make_room()
                    self._use(e)
            else:
                loads += 1
                if self.cap:
                    self._make_room()
                    self._use(e)
        self.landed = set()
        return loads

    def prefetch(self, pred):
        copies = 0
        for i, e in enumerate(pred):
            if e in self.landed:
                continue
            if i < self.cap:                 # distinct ids: the first cap of them use the layer's own slots
                if e not in self.stamp:
                    copies += 1
                    self._make_room()
                self._use(e)
            else:
                assert e not in self.stamp   # the cap own slots hold the cap experts predicted before it
                self.landed.add(e)
                copies += 1
        return copies


def test_cache_prefetch_against_timestamp_simulator():
    rng = np.random.default_rng(12)
    for trial in range(60):
        cap = int(rng.integers(0, 5))
        c = OC.ExpertCache([cap])
        ref = _StampCacheWithLanding(cap)
        for n in range(60):
            k = int(rng.integers(1, 3))
            ids = rng.choice(6, size=2, replace=False)
            want_loads = ref.demand([int(e) for e in ids[:k]])
            evs = c.demand(n, 0, ids, k)
            assert sum(ev[2] in (OC.MISS, OC.BYPASS) for ev in evs) == want_loads
            assert c.landed(0) == []                       # nothing survives the demand
            pred = list(rng.choice(6, size=int(rng.integers(0, 4)), replace=False))
            want_copies = ref.prefetch([int(e) for e in pred])
            evs = c.prefetch(n, 0, pred)
            assert sum(ev[2] in (OC.PF_LOAD, OC.PF_LAND) for ev in evs) == want_copies
            assert sorted(c.resident(0)) == sorted(ref.stamp)
            assert sorted(c.landed(0)) == sorted(ref.landed)
            assert len(c.resident(0)) <= cap
            assert len(evs) == len(pred)                   # every predicted expert is on the GPU afterwards
            assert all(e in c.resident(0) or e in c.landed(0) for e in pred)


def test_cache_landing_hand_trace(golden_dir):
    g = _load(golden_dir, "cache_landing_trace.json")
    for sc in g["scenarios"]:
        c = OC.ExpertCache(sc["slots"])
        for s in sc["steps"]:
            c.demand(s["token"], s["layer"], s["demand"], s["k"])
            if s["layer"] + 1 < len(sc["slots"]):
                c.prefetch(s["token"], s["layer"] + 1, s["pred_for_next"])
        assert [list(e) for e in c.events] == sc["events"]
        assert [c.resident(l) for l in range(len(sc["slots"]))] == sc["final_resident"]
        s = OC.summarise(c.events)
        assert s["on_demand_loads"] == sc["on_demand_loads"] and s["prefetch_loads"] == sc["prefetch_loads"]
        assert s["prefetch_landed"] == sc["prefetch_landed"] and s["prefetch_useful"] == sc["prefetch_useful"]


def test_cache_without_slots_loads_on_demand_only_when_the_prefetch_was_wrong():
    """The on-demand-load model counts, for a token that needs one expert, a load when the cache
    misses and the prefetch was wrong: (1 - t/N)(1 - beta), which is 1 - beta for a layer without
    slots (Sec. 4.4.2, Eq.11).  A layer with zero slots must therefore load on demand exactly for
    the tokens whose prediction was wrong, and for two required experts exactly the wrongly
    predicted ones."""
    n_tok, N = 200, 8
    rng = np.random.default_rng(3)
    need = rng.integers(0, N, size=n_tok)
    right = rng.random(n_tok) < 0.7
    c = OC.ExpertCache([4, 0])
    for n in range(n_tok):
        c.demand(n, 0, [0, 1], 1)
        c.prefetch(n, 1, [int(need[n]) if right[n] else int((need[n] + 1) % N)])
        c.demand(n, 1, [int(need[n]), 0], 1)
    l1 = [ev for ev in c.events if ev[1] == 1]
    assert sum(ev[2] == OC.BYPASS for ev in l1) == int((~right).sum())
    assert sum(ev[2] == OC.HIT_PF for ev in l1) == int(right.sum())
    assert sum(ev[2] == OC.PF_LAND for ev in l1) == n_tok and c.resident(1) == [] and c.landed(1) == []
    # two required, one of them predicted: one on-demand load (the case of Eq.13)
    c = OC.ExpertCache([0])
    c.prefetch(0, 0, [5])
    evs = c.demand(0, 0, [5, 2], 2)
    assert [ev[2] for ev in evs] == [OC.HIT_PF, OC.BYPASS]
    # several tokens in one step share the landing buffers until the step ends
    c = OC.ExpertCache([0])
    c.prefetch(0, 0, [5, 6, 7])
    a = c.demand(0, 0, [6, 1], 1, release=False)
    b = c.demand(0, 0, [5, 6], 2, release=False)
    c.release_landing(0)
    assert [ev[2] for ev in a + b] == [OC.HIT_PF, OC.HIT_PF, OC.BYPASS] and c.landed(0) == []


# --------------------------------------------------------------- planner ----

def _expected_loads_by_enumeration(N, t, a, beta):
    """Expected on-demand loads when a uniformly random set of t of N experts is
    cached (Sec. 4.4.2), using the per-case load counts the text gives:
    one required: miss and wrong prefetch -> 1;
    two required: both miss -> 2 if the prefetch is wrong, 1 if it is right for one;
                  one hits  -> 1 if the prefetch is wrong."""
    sets = list(itertools.combinations(range(N), t))
    one = sum((0 not in S) for S in sets) / len(sets) * (1 - beta)
    two = 0.0
    for S in sets:
        miss = (0 not in S) + (1 not in S)          # experts 0 and 1 are the two "given" experts
        if miss == 2:
            two += 2 * (1 - beta) + 1 * beta
        elif miss == 1:
            two += 1 * (1 - beta)
    two /= len(sets)
    return a * one + (1 - a) * two


def test_cost_model_by_enumeration():
    for N in (2, 3, 5, 8):
        for t in range(N + 1):
            assert abs(OP.p_both_miss(N, t) + OP.p_one_hit(N, t) + OP.p_both_hit(N, t) - 1.0) < 1e-14
            for a, beta in ((0.0, 0.0), (0.24, 0.9), (1.0, 0.3), (0.5, 1.0)):
                assert abs(OP.cost(N, t, a, beta) - _expected_loads_by_enumeration(N, t, a, beta)) < 1e-13


def test_cost_model_closed_forms_and_shape():
    N = 8
    for a, beta in ((0.24, 0.9), (0.5, 0.5), (0.0, 0.0), (1.0, 1.0)):
        f = [OP.cost(N, t, a, beta) for t in range(N + 1)]
        assert f[N] == 0.0
        assert abs(f[0] - (a * (1 - beta) + (1 - a) * (2 - beta))) < 1e-14
        d = np.diff(f)
        assert np.all(d <= 1e-15) and np.all(np.diff(d) >= -1e-15)   # non-increasing, convex


def _brute_plan(L, N, C, f):
    best, arg = math.inf, None
    for t in itertools.product(range(N + 1), repeat=L):
        if sum(t) <= C:
            c = sum(f[i][t[i]] for i in range(L))
            if c < best - 1e-12:
                best, arg = c, t
    return best, arg


def test_plan_brute_force_and_greedy():
    rng = np.random.default_rng(21)
    for trial in range(40):
        L, N = int(rng.integers(1, 5)), int(rng.integers(2, 5))
        C = int(rng.integers(0, 11))
        a = np.round(rng.uniform(0, 1, L) * 1024) / 1024
        beta = np.round(rng.uniform(0, 1, L) * 1024) / 1024
        t, cst = OP.plan(L, N, C, a, beta)
        f = OP.cost_table(N, a, beta)
        best, _ = _brute_plan(L, N, C, f)
        assert abs(cst - best) < 1e-12
        assert sum(t) <= C and all(0 <= v <= N for v in t)
        assert abs(sum(f[i][t[i]] for i in range(L)) - cst) < 1e-12
        # f is convex in t, so handing out slots by largest marginal gain reaches the same cost
        g = [0] * L
        for _ in range(min(C, L * N)):
            gains = [(f[i][g[i]] - f[i][g[i] + 1]) if g[i] < N else -1 for i in range(L)]
            i = int(np.argmax(gains))
            if gains[i] <= 0:
                break
            g[i] += 1
        assert abs(sum(f[i][g[i]] for i in range(L)) - cst) < 1e-12


def test_plan_special_cases():
    L, N = 5, 8
    a, beta = np.full(L, 0.25), np.full(L, 0.75)
    t, c = OP.plan(L, N, L * N + 7, a, beta)
    assert c == 0.0 and t == [N] * L
    t, c = OP.plan(L, N, 0, a, beta)
    assert t == [0] * L and abs(c - L * (0.25 * 0.25 + 0.75 * 1.25)) < 1e-13
    # a layer that is predicted perfectly and always runs one expert needs no slot
    a2, b2 = np.array([1.0, 0.0]), np.array([1.0, 0.0])
    t, c = OP.plan(2, 8, 8, a2, b2)
    assert t == [0, 8] and c == 0.0


def test_profile_from_trace():
    dec = [[[1, 2], [3]], [[1], [3, 4]]]
    pred = [[[], [3]], [[], [5, 4]]]
    a, b = OP.profile_from_trace(dec, pred, 2)
    np.testing.assert_allclose(a, [0.5, 0.5])
    np.testing.assert_allclose(b, [0.0, 2 / 3])


# ----------------------------------------------------------------- stack ----

def test_stack_wiring():
    rng = np.random.default_rng(31)
    H, F, N, L = 8, 6, 4, 3
    routers = [rng.standard_normal((N, H)) for _ in range(L)]
    W = [[(rng.standard_normal((F, H)), rng.standard_normal((F, H)), rng.standard_normal((H, F))) for _ in range(N)] for _ in range(L)]
    h0 = rng.standard_normal((4, H)) * 3
    ex = lambda l, e, x: OE.expert_ffn(x, *W[l][e])
    x = OS.rmsnorm(h0[0])
    assert abs(np.sqrt(np.mean(x * x)) - 1.0) < 1e-6
    # gamma = 0: the residual stream never changes
    r0 = OS.run_stack(h0, routers, [0.2] * L, ex, 0.0)
    for l in range(L + 1):
        np.testing.assert_array_equal(r0["h"][:, l], h0)
    # one layer: h1 = h0 + gamma * block(x0), gate taken on x0
    r1 = OS.run_stack(h0[:1], routers[:1], [0.2], ex, 0.5)
    g = OG.adaptive_gate(x, routers[0], 0.2)
    y = OE.moe_block(x, W[0], g["ids"], g["w"], g["k"])
    np.testing.assert_allclose(r1["h"][0, 1], h0[0] + 0.5 * y, rtol=1e-13)
    # predictions for layer l+1 use layer l+1's gate on layer l's input
    r = OS.run_stack(h0, routers, [0.2] * L, ex, 0.3, collect_x=True)
    for n in range(4):
        for l in range(L - 1):
            assert r["pred"][n][l + 1] == OG.predict_next(r["x"][n, l], routers[l + 1], 0.2)
        assert r["pred"][n][0] == []


def test_first_layer_predictive_gate_is_exact_when_inputs_repeat():
    """With gamma = 0 and the same token repeated, the last layer's input of token n equals the first
    layer's input of token n+1, so a predictive gate equal to the first router predicts layer 0 exactly
    (Sec. 4.3): after the first token, layer 0 never loads on demand.  With two alternating tokens the
    same gate always predicts the wrong pair and the two-slot LRU set keeps missing."""
    from oracle import stack as OS
    rng = np.random.default_rng(21)
    L, N, H = 3, 6, 16
    routers = [rng.standard_normal((N, H)) for _ in range(L)]
    taus = [0.0] * L                      # always two experts
    # two tokens alternate, so layer 0 needs two different expert pairs in turn
    t0, t1 = rng.standard_normal(H), rng.standard_normal(H)
    h0 = [t0, t1] * 6
    zero = lambda l, e, x: np.zeros(H)

    def loads_layer0(first_gate):
        c = OC.ExpertCache([2, 2, 2])
        OS.run_stack(h0, routers, taus, zero, gamma=0.0, cache=c, first_gate=first_gate)
        return [ev for ev in c.events if ev[1] == 0 and ev[2] == OC.MISS], c

    e0 = set(OG.adaptive_gate(OS.rmsnorm(t0), routers[0], 0.0)["ids"])
    e1 = set(OG.adaptive_gate(OS.rmsnorm(t1), routers[0], 0.0)["ids"])
    assert e0 != e1                        # the seed gives two different pairs, otherwise the test is void
    miss_without, _ = loads_layer0(None)
    assert len(miss_without) >= 6          # LRU with 2 slots thrashes on the alternation
    # a predictive gate applied to token n's last-layer input predicts token n's own layer-0 pair
    # (inputs repeat across layers), not token n+1's: with alternating tokens it is always wrong
    miss_self, _ = loads_layer0(routers[0])
    assert len(miss_self) >= 6
    # constant stream: prediction exact, so after the first token layer 0 only hits
    c = OC.ExpertCache([2, 2, 2])
    out = OS.run_stack([t0] * 5, routers, taus, zero, gamma=0.0, cache=c, first_gate=routers[0])
    l0 = [ev for ev in c.events if ev[1] == 0]
    assert [ev[2] for ev in l0 if ev[0] == 0 and ev[2] in (OC.MISS, OC.HIT)] == [OC.MISS, OC.MISS]
    assert all(ev[2] in (OC.HIT, OC.HIT_PF, OC.PF_TOUCH) for ev in l0 if not (ev[0] == 0 and ev[2] == OC.MISS))
    assert all(sorted(out["pred"][n][0]) == sorted(e0) for n in range(1, 5))
