"""CPU oracle O-std: the textbook top-k mixture-of-experts layer.

TEST INFRASTRUCTURE ONLY (see oracle/routing.py for who may import this).

Definition followed (paper, Preliminary, Eq. 0 and Eq. 1):

    MoE(x) = sum_i R(x)_i * E_i(x),   R(x) = TopK(Softmax(g(x)), k)

with every expert a SwiGLU feed-forward network (fixed by the build's baseline
file; the paper's pipeline listing only names two weight tensors),

    E_i(v) = W_down,i ( silu(W_gate,i v) * (W_up,i v) ),   silu(z) = z / (1 + exp(-z)),

and S shared experts that every token uses with weight 1 (the paper mentions
them once, as a DeepSeek-MoE feature; they take no part in routing).

There is no dispatch, no device and no deduplication in this file: every
(token, selected expert) pair is evaluated on its own and summed.  It is the
result the deduplicated path must reproduce exactly when pruning is off.
All arithmetic is float64 from the stored inputs.
"""
from __future__ import annotations

import numpy as np


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def expert_ffn(v: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray,
               acc=np.float64) -> np.ndarray:
    """E_i(v) for rows v [n, d]; weights [f, d], [f, d], [d, f]."""
    v = v.astype(acc)
    g = v @ w_gate.astype(acc).T
    u = v @ w_up.astype(acc).T
    return (silu(g) * u) @ w_down.astype(acc).T


def topk_by_definition(logits: np.ndarray, k: int, renorm: int):
    """Eq. 1 written out: softmax over all experts, keep the k largest.
    Equal scores: lower expert index first (same reading as oracle/routing.py, written
    independently: a lexicographic sort on (-score, index))."""
    lg = logits.astype(np.float64)
    T, E = lg.shape
    p = np.exp(lg - lg.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    ids = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k), dtype=np.float64)
    idx = np.arange(E)
    for t in range(T):
        order = np.lexsort((idx, -lg[t]))      # primary key -score, secondary key index
        ids[t] = order[:k]
        w[t] = p[t, order[:k]]
    if renorm:
        w /= w.sum(axis=1, keepdims=True)
    return ids, w


def moe_layer(x: np.ndarray, ids: np.ndarray, w: np.ndarray, w_gate: np.ndarray,
              w_up: np.ndarray, w_down: np.ndarray, E: int, S: int = 0,
              tokens: np.ndarray | None = None, acc=np.float64) -> np.ndarray:
    """y[t] = sum_s w[t,s] * E_{ids[t,s]}(x[t]) + sum_{shared} E_shared(x[t]).

    ``tokens`` restricts the evaluation to a subset of rows (sampled parity at full size);
    the result then has one row per entry of ``tokens``.
    Grouped by expert so that BLAS does the products; the sum over a token's experts is
    accumulated in expert-index order in float64.
    """
    if tokens is None:
        tokens = np.arange(x.shape[0])
    tokens = np.asarray(tokens)
    xs = x[tokens].astype(acc)
    ids_s = ids[tokens]
    w_s = w[tokens].astype(acc)
    y = np.zeros((len(tokens), x.shape[1]), dtype=acc)
    for e in range(E):
        rows, slots = np.nonzero(ids_s == e)
        if rows.size == 0:
            continue
        out = expert_ffn(xs[rows], w_gate[e], w_up[e], w_down[e], acc)
        y[rows] += w_s[rows, slots][:, None] * out
    for s in range(S):
        y += expert_ffn(xs, w_gate[E + s], w_up[E + s], w_down[E + s], acc)
    return y


def moe_layer_loops(x, ids, w, w_gate, w_up, w_down, E, S=0) -> np.ndarray:
    """The same definition with explicit per-token, per-expert loops (tiny inputs only)."""
    T, d = x.shape
    k = ids.shape[1]
    y = np.zeros((T, d), dtype=np.float64)
    for t in range(T):
        v = x[t].astype(np.float64)
        chosen = [(int(ids[t, s]), float(w[t, s])) for s in range(k)]
        chosen += [(E + s, 1.0) for s in range(S)]
        for e, gate in chosen:
            g = w_gate[e].astype(np.float64) @ v
            u = w_up[e].astype(np.float64) @ v
            h = g / (1.0 + np.exp(-g)) * u
            y[t] += gate * (w_down[e].astype(np.float64) @ h)
    return y
