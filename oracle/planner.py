"""Checker: on-demand-loading cost model and cache-size allocation (test infrastructure).

Sec. 4.4 of the paper: the expected number of on-demand expert loads of layer
i with t cached experts, f_{i,t} (Eq.10-15), from the layer's single-expert
probability a_i and prefetch accuracy beta_i; the allocation minimises
sum_i f_{i,t_i} subject to sum t_i <= C and 0 <= t_i <= N (Eq.16-18) by a
knapsack dynamic programme (Eq.19) followed by a traceback from the last
layer.  float64 throughout.

Readings where the text is silent: ties in the traceback go to the smallest
slot count (two candidates tie when they differ by at most 1e-12); the
printed probability that two given experts are both cached, "t*t-1 over
N*(N-1)", is read as t(t-1)/(N(N-1)).
"""
from __future__ import annotations

import numpy as np

TIE = 1e-12


def p_both_miss(N, t):
    """Probability that two given experts are both absent from a cache of t of N (Sec. 4.4.2)."""
    return max((N - t) * (N - t - 1), 0) / (N * (N - 1))


def p_one_hit(N, t):
    """Probability that exactly one of two given experts is cached (coefficient of Eq.14)."""
    return 2.0 * (N - t) * t / (N * (N - 1))


def p_both_hit(N, t):
    return t * (t - 1) / (N * (N - 1))


def cost_single(N, t, beta):
    """Eq.11: one expert required; a load happens on a cache miss with a wrong prefetch."""
    return (1.0 - t / N) * (1.0 - beta)


def cost_double(N, t, beta):
    """Eq.12 + Eq.13 + Eq.14: two experts required."""
    m2 = p_both_miss(N, t)
    f2 = 2.0 * m2 * (1.0 - beta)          # both miss, prefetch wrong: two loads
    f3 = m2 * beta                        # both miss, prefetch right for one: one load
    f4 = p_one_hit(N, t) * (1.0 - beta)   # one hits, prefetch wrong: one load
    return f2 + f3 + f4


def cost(N, t, a, beta):
    """Eq.15: f_{i,t} = a * f^1 + (1-a) * (f^2 + f^3 + f^4)."""
    return a * cost_single(N, t, beta) + (1.0 - a) * cost_double(N, t, beta)


def cost_table(N, a, beta):
    """f[i][t] for every layer i and 0 <= t <= N."""
    L = len(a)
    return np.array([[cost(N, t, float(a[i]), float(beta[i])) for t in range(N + 1)] for i in range(L)])


def plan(L, N, C, a, beta):
    """Eq.19 and the traceback.  Returns (t[L] ints, total cost)."""
    f = cost_table(N, a, beta)
    C = int(C)
    Fm = np.zeros((L + 1, C + 1))
    for i in range(1, L + 1):
        for j in range(C + 1):
            best = np.inf
            for k in range(min(j, N) + 1):
                v = Fm[i - 1][j - k] + f[i - 1][k]
                if v < best:
                    best = v
            Fm[i][j] = best
    t = [0] * L
    j = C
    for i in range(L, 0, -1):
        for k in range(min(j, N) + 1):
            if Fm[i - 1][j - k] + f[i - 1][k] <= Fm[i][j] + TIE:
                t[i - 1] = k
                j -= k
                break
    return t, float(Fm[L][C])


def profile_from_trace(decisions, predictions, L):
    """a_l and beta_l from a profiling run (Sec. 4.4.1: both come from offline tracing).

    decisions[n][l]   = list of experts activated for token n in layer l (length k)
    predictions[n][l] = list of experts predicted for layer l while layer l-1 ran
                        (empty for layer 0, which has no predecessor)
    a_l    = fraction of tokens with one activated expert in layer l
    beta_l = activated experts that had been predicted / activated experts
    """
    a = np.zeros(L)
    beta = np.zeros(L)
    for l in range(L):
        single = tot = inter = 0
        for n in range(len(decisions)):
            E = decisions[n][l]
            r = predictions[n][l]
            single += (len(E) == 1)
            tot += len(E)
            inter += len(set(E) & set(r))
        a[l] = single / len(decisions)
        beta[l] = inter / tot if tot else 0.0
    return a, beta
