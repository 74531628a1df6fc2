"""Checker: multi-layer decode loop around the MoE block (test infrastructure).

The paper's model has attention and normalisation between MoE blocks; this
path has neither, so the multi-layer workloads wire the blocks with a residual
stream of this build's own choosing (NOT from the paper; parity unpinned for
the wiring):

    x_l     = store( h_l / sqrt(mean(h_l^2) + 1e-6) )   input of MoE block l
    h_{l+1} = h_l + gamma * MoE_l(x_l)

`store` rounds to the activation storage format (identity for fp32).  The
residual keeps successive block inputs similar, the property the paper's
predictor relies on (Sec. 3, observation 2).  Per token and layer the loop
follows Alg.1: gate (Eq.1, Eq.8), predict for the following layer with that
layer's gate on the same x_l (Sec. 4.3), demand the activated experts from the
cache, prefetch the predicted ones, evaluate (Eq.2-4).
"""
from __future__ import annotations

import numpy as np

from . import gate as G

F64 = np.float64
EPS = 1e-6


def rmsnorm(h):
    h = np.asarray(h, dtype=F64)
    return h / np.sqrt(np.mean(h * h) + EPS)


def run_stack(h0, routers, taus, expert_out, gamma, store=lambda a: a, cache=None,
              collect_x=False, depth=1, first_gate=None):
    """Run tokens h0[n] through L layers.

    routers[l]            W_g of layer l, [N,H]
    taus[l]               threshold of layer l
    expert_out(l, e, x)   E_e^{(l)}(x), float64 [H]
    cache                 optional oracle.cache.ExpertCache driven alongside
    depth                 look-ahead: layers l+1 .. l+depth are predicted from x_l (Sec. 4.3)
    first_gate            optional predictive gate [N,H] for layer 0 (Sec. 4.3, Eq.9): applied to the last
                          layer's block input, with layer 0's threshold; its prediction is prefetched
                          into layer 0's cache for the following token
    Returns dict of per (token, layer): ids, k, w, v, pred (pred[n][l] = list predicted for
    layer l by layer l-1; pred[n][0] = list predicted by the predictive gate during token n-1), ahead (ahead[n][l][d-1] = list predicted at layer l for layer l+d),
    h (block input residual, [n,L+1,H]) and, if collect_x, x [n,L,H].
    """
    n_tok = len(h0)
    L = len(routers)
    H = len(h0[0])
    ids = np.zeros((n_tok, L, 2), np.int32)
    ks = np.zeros((n_tok, L), np.int32)
    ws = np.zeros((n_tok, L, 2), F64)
    vs = np.zeros((n_tok, L), F64)
    gap23 = np.zeros((n_tok, L), F64)
    preds = [[[] for _ in range(L)] for _ in range(n_tok)]   # preds[n][l] = predicted FOR layer l
    ahead = [[[] for _ in range(L)] for _ in range(n_tok)]
    hs = np.zeros((n_tok, L + 1, H), F64)
    xs = np.zeros((n_tok, L, H), F64) if collect_x else None
    for n in range(n_tok):
        h = np.asarray(h0[n], dtype=F64)
        for l in range(L):
            hs[n, l] = h
            x = np.asarray(store(rmsnorm(h)), dtype=F64)
            if collect_x:
                xs[n, l] = x
            g = G.adaptive_gate(x, routers[l], taus[l])
            ids[n, l], ks[n, l], ws[n, l], vs[n, l] = g["ids"], g["k"], g["w"], g["v"]
            zs = np.sort(g["z"])[::-1]
            gap23[n, l] = zs[1] - zs[2] if len(zs) > 2 else np.inf
            rs = [G.predict_next(x, routers[l + d], taus[l + d]) for d in range(1, depth + 1) if l + d < L]
            ahead[n][l] = rs
            if rs:
                preds[n][l + 1] = rs[0]
            if cache is not None:
                cache.demand(n, l, g["ids"], g["k"])
                cache.prefetch_lookahead(n, l, rs)
            if first_gate is not None and l == L - 1:
                r0 = G.predict_next(x, first_gate, taus[0])
                if n + 1 < n_tok:
                    preds[n + 1][0] = r0
                if cache is not None:
                    cache.prefetch(n, 0, r0)
            y = np.zeros(H, F64)
            for j in range(g["k"]):
                y += F64(g["w"][j]) * expert_out(l, int(g["ids"][j]), x)
            h = h + F64(gamma) * y
        hs[n, L] = h
    return dict(ids=ids, k=ks, w=ws, v=vs, gap23=gap23, pred=preds, ahead=ahead, h=hs, x=xs)
