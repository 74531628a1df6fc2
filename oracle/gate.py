"""Checker: router, softmax, top-2 and the adaptive gating test (test infrastructure).

Follows the paper's gating definition (Sec. 2.1, Eq.1), the two-expert /
one-expert outputs (Sec. 4.2, Eq.3 and Eq.4) and the activation rule (Eq.8).
All arithmetic is float64.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def router_logits(x, Wg):
    """z_i = sum_h x_h * W_g[i,h]  (the product x.W_g inside Eq.1); Wg is [N,H]."""
    return np.asarray(Wg, dtype=F64) @ np.asarray(x, dtype=F64)


def softmax(z):
    """Softmax over all N logits (max subtracted first)."""
    z = np.asarray(z, dtype=F64)
    e = np.exp(z - z.max())
    return e / e.sum()


def top2(p):
    """Indices of the largest and second-largest entries; equal values -> lower index first."""
    p = np.asarray(p)
    e1 = int(np.argmax(p))
    q = p.copy()
    q[e1] = -np.inf
    e2 = int(np.argmax(q))
    return e1, e2


def normalised_scores(p, e1, e2):
    """alpha = normalised score of the top-1 expert and 1-alpha of the top-2
    (Sec. 4.2: Eq.3 weighs f1 by alpha and f2 by 1-alpha; normalising the two
    selected softmax scores is the same as a softmax over the two selected
    logits, which is how Eq.1 states it)."""
    s = p[e1] + p[e2]
    return p[e1] / s, p[e2] / s


def tau_from_sensitivity(T, S):
    """Per-layer threshold on the second weight implied by Eq.8:
    (1-alpha)^2 * S <= T  <=>  (1-alpha) <= sqrt(T/S)   (S = sum diag(F) > 0)."""
    return np.sqrt(F64(T) / F64(S))


def single_expert_eq8(alpha, S, T):
    """Eq.8 literally: only one expert is activated iff (1-alpha)^2 * sum diag(F) <= T."""
    return (1.0 - F64(alpha)) ** 2 * F64(S) <= F64(T)


def adaptive_gate(x, Wg, tau):
    """One token, one layer.

    Returns dict with
      ids   (e1, e2)      top-1 and top-2 expert (always both reported)
      k     1 or 2        experts that run (Eq.8 with tau = sqrt(T/S))
      w     (w1, w2)      (1, 0) if k == 1 (Eq.4) else (alpha, 1-alpha) (Eq.3)
      alpha, v            normalised top-1 score and test value v = 1-alpha
      z, p                logits and full softmax (for diagnostics)
    """
    z = router_logits(x, Wg)
    p = softmax(z)
    e1, e2 = top2(p)
    alpha, v = normalised_scores(p, e1, e2)
    k = 1 if v <= F64(tau) else 2
    w = (1.0, 0.0) if k == 1 else (float(alpha), float(v))
    return dict(ids=(e1, e2), k=k, w=w, alpha=float(alpha), v=float(v), z=z, p=p)


def predict_next(x, Wg_next, tau_next):
    """Expert prediction for the following layer (Sec. 4.3): the following
    layer's gate, adaptive test included, applied to the *current* layer's
    MoE-block input.  Returns the list of predicted experts in rank order
    (length k_hat)."""
    g = adaptive_gate(x, Wg_next, tau_next)
    return list(g["ids"][: g["k"]])


def gate_batch(X, Wg, tau):
    """adaptive_gate over rows of X; returns ids[B,2] int32, w[B,2] f64, k[B] int32, v[B] f64,
    gap23[B] f64 (difference between 2nd and 3rd largest logit, for near-tie reporting)."""
    X = np.asarray(X)
    B = X.shape[0]
    N = np.asarray(Wg).shape[0]
    ids = np.zeros((B, 2), np.int32)
    w = np.zeros((B, 2), F64)
    k = np.zeros(B, np.int32)
    v = np.zeros(B, F64)
    gap12 = np.zeros(B, F64)
    gap23 = np.full(B, np.inf, F64)
    for b in range(B):
        g = adaptive_gate(X[b], Wg, tau)
        ids[b] = g["ids"]
        w[b] = g["w"]
        k[b] = g["k"]
        v[b] = g["v"]
        zs = np.sort(g["z"])[::-1]
        gap12[b] = zs[0] - zs[1]
        if N > 2:
            gap23[b] = zs[1] - zs[2]
    return dict(ids=ids, w=w, k=k, v=v, gap12=gap12, gap23=gap23)
