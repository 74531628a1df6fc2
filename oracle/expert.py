"""Checker: expert feed-forward network and the weighted combine (test infrastructure).

The MoE output is the gate-weighted sum of expert outputs (Sec. 2.1, Eq.2);
with adaptive gating it is alpha*f1(x) + (1-alpha)*f2(x) when two experts run
(Eq.3) and f1(x) when one runs (Eq.4).  The expert body is the evaluation
model's (Mixtral, Sec. 6.1): a bias-free SwiGLU FFN,
E(x) = W2 . ( silu(W1 x) * (W3 x) ),  silu(g) = g / (1 + exp(-g)).
All arithmetic is float64.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def silu(g):
    g = np.asarray(g, dtype=F64)
    return g / (1.0 + np.exp(-g))


def expert_ffn(x, W1, W3, W2):
    """E(x) for one token.  W1,W3: [F,H]; W2: [H,F]; x: [H] -> [H]."""
    x = np.asarray(x, dtype=F64)
    g = np.asarray(W1, dtype=F64) @ x
    u = np.asarray(W3, dtype=F64) @ x
    a = silu(g) * u
    return np.asarray(W2, dtype=F64) @ a


def expert_ffn_rows(X, W1, W3, W2):
    """E applied to every row of X [B,H] -> [B,H] (same definition, one matmul per matrix)."""
    X = np.asarray(X, dtype=F64)
    g = X @ np.asarray(W1, dtype=F64).T
    u = X @ np.asarray(W3, dtype=F64).T
    a = silu(g) * u
    return a @ np.asarray(W2, dtype=F64).T


def combine(ids, w, k, expert_out):
    """y = sum_{j<k} w_j * E_{ids_j}(x)  (Eq.2 restricted to the activated experts, Eq.3-4).
    `expert_out(e)` returns E_e(x)."""
    y = None
    for j in range(int(k)):
        t = F64(w[j]) * expert_out(int(ids[j]))
        y = t if y is None else y + t
    return y


def moe_block(x, experts, ids, w, k):
    """Output of the MoE block for one token given the gate's decision.
    `experts[e]` is (W1, W3, W2)."""
    return combine(ids, w, k, lambda e: expert_ffn(x, *experts[e]))


def moe_block_rows(X, experts, ids, w, k):
    """moe_block for every row of X, evaluated expert by expert: for each expert
    the rows that activated it are gathered, passed through E, scaled by their
    weight and added into their output rows."""
    X = np.asarray(X, dtype=F64)
    B = X.shape[0]
    Y = np.zeros_like(X)
    ids = np.asarray(ids)
    for e in range(len(experts)):
        for j in range(2):
            rows = np.nonzero((ids[:, j] == e) & (np.asarray(k) > j))[0]
            if rows.size == 0:
                continue
            out = expert_ffn_rows(X[rows], *experts[e])
            Y[rows] += np.asarray(w, dtype=F64)[rows, j][:, None] * out
    return Y


# ---------------------------------------------------------------------------
# 4-bit group-quantised storage (the paper runs 4-bit experts, Sec. 6.3; this
# build's storage format is asymmetric round-to-nearest with groups of 64
# along the reduction axis and fp16 scale / zero per group)
# ---------------------------------------------------------------------------


def decode_int4(codes, scale, zero, group=64):
    """w_hat[r, c] = codes[r, c] * scale[r, c//group] + zero[r, c//group], float64.
    codes: [rows, cols] integers 0..15 (unpacked); scale, zero: [rows, cols/group]."""
    codes = np.asarray(codes)
    rows, cols = codes.shape
    s = np.repeat(np.asarray(scale, dtype=F64), group, axis=1)
    z = np.repeat(np.asarray(zero, dtype=F64), group, axis=1)
    return codes.astype(F64) * s + z


def unpack_nibbles(packed):
    """[rows, cols/2] bytes -> [rows, cols] codes; low nibble is the even element."""
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty((p.shape[0], p.shape[1] * 2), dtype=np.uint8)
    out[:, 0::2] = p & 0xF
    out[:, 1::2] = p >> 4
    return out
