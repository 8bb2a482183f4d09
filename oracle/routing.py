"""CPU oracle: softmax top-k routing with optional collaboration pruning.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this file;
only tests/, the smoke check and the benchmark's cpu_baseline leg may call it.
It shares no code with the HIP path.

What is computed (paper, Preliminary, Eq. 1 and Section 3.3 "Expert
Collaboration Pruning", routing-score-based variant):

* gate scores  p = Softmax(g(x)) over all E experts; the router scores g(x)
  ("logits") are an input;
* the k experts of highest score are selected; their gates are their softmax
  values, optionally divided by their sum (``renorm``);
* with pruning (n_d > 0) each token may use experts of at most n_d devices.
  The surviving devices are chosen either
    mode 1: by the summed gate score of the token's unpruned top-k experts per
            device (highest n_d sums; the rule of this build's benchmark configurations), or
    mode 2: by walking the unpruned top-k in descending score order and keeping
            the first n_d distinct devices met (the paper's wording);
  then the k highest-scoring experts *on the surviving devices* are selected
  (Section 3.3, steps 1-2).  Tokens whose top-k already lies on <= n_d devices
  keep their selection (footnote of Section 3.3).

Readings where the paper is silent:
* selection compares the raw float32 router scores (softmax is monotone, so
  the order is that of the softmax values, without any exp in the comparison);
  larger first, equal scores -> lower expert index first; -0.0 equals +0.0;
  slot 0 holds the highest-scoring selected expert;
* mode-1 device sums decide an integer (which devices survive), so they are
  taken in one fixed float32 arithmetic that the GPU kernel repeats step by
  step: q_i = exp_ref(l_i - max_j l_j), summed sequentially in slot order into a
  float32 accumulator per device; highest sum first, equal sums -> lower device;
  exp_ref is defined below.  Unnormalised q has the same order as p.
* gates after pruning are still softmax values over all E experts (no second
  softmax), then renormalised if asked.

Gate *values* are computed in float64 from the float32 scores (the definition);
only decisions use exp_ref.

Expert-similarity-based pruning (Section 3.3, second criterion; Appendix "Similarity Table
Construction") is ``prune_mode=3``.  The table comes from profiled router scores H [N, E]:
squared cosine similarity of the expert columns, T2[i,j] = <H_i,H_j>^2 / (|H_i|^2 |H_j|^2)
(`similarity`), which only needs the Gram matrix H^T H, summed over batches (`gram`).  Readings:
* the integer table lists, for every expert i, the other experts by descending T2 (equal values ->
  lower expert index first): `similarity_table` ([E, E-1]);
* the devices that survive are found as in mode 2 (walk the top-k in descending score, keep the
  first n_d distinct devices);
* then the k routed experts are walked in descending score: an expert on a surviving device
  stays in its slot; any other is replaced by the first expert of its table row that sits on a
  surviving device and is not selected - where "selected" covers every routed expert that stays
  (also those later in the walk) and the replacements made so far, so the result is k distinct
  experts;
* gates are the softmax values of the final experts (their own scores), renormalised if asked;
  slots keep the walk order, so after a replacement slot order is no longer score order.

Router scores themselves (Eq. 1: g is a single linear projection of the hidden
state) are `router_scores`: the plain product x W_r^T in float64 from the stored
inputs.  A second implementation of that product sums in another order, so its
float32 scores differ in the last bits and selections whose deciding scores are
closer than that may legitimately differ; `selection_margin` measures, per token,
the gap that decides its selection, which is what a test needs to audit such
differences.
"""
from __future__ import annotations

import numpy as np

# ---- exp_ref: the fixed float32 sequence that decides device sums -----------------------
# z <= 0.  z < -80 -> 0.  n = rint(z * LOG2E) (ties to even); r = (z - n*LN2_HI) - n*LN2_LO;
# Horner polynomial of degree 7 with Taylor coefficients 1/i!, every multiply and every add
# rounded to float32 on its own (no fused multiply-add); result = poly * 2**n (exact).
_F = np.float32
LOG2E = _F(1.4426950408889634)
LN2_HI = _F(0.693359375)            # 355/512, exact in 9 bits: n*LN2_HI is exact for |n| < 2**15
LN2_LO = _F(-2.12194440054690583e-4)  # ln 2 - LN2_HI
EXP_CUTOFF = _F(-80.0)
EXP_COEF = [_F(1.0), _F(1.0), _F(0.5), _F(1.0 / 6.0), _F(1.0 / 24.0), _F(1.0 / 120.0),
            _F(1.0 / 720.0), _F(1.0 / 5040.0)]


def exp_ref(z: np.ndarray) -> np.ndarray:
    """exp(z) for z <= 0 in the fixed float32 sequence described above (vectorised)."""
    z = np.asarray(z, dtype=np.float32)
    with np.errstate(over="ignore", under="ignore", invalid="ignore"):
        zc = np.maximum(z, EXP_CUTOFF)            # keep the arithmetic finite for masked lanes
        n = np.rint(zc * LOG2E).astype(np.float32)
        t = (n * LN2_HI).astype(np.float32)
        r = (zc - t).astype(np.float32)
        t = (n * LN2_LO).astype(np.float32)
        r = (r - t).astype(np.float32)
        p = np.full_like(r, EXP_COEF[7])
        for i in range(6, -1, -1):
            p = (p * r).astype(np.float32)
            p = (p + EXP_COEF[i]).astype(np.float32)
        scale = ((n.astype(np.int32) + 127) << 23).astype(np.int32).view(np.float32)
        out = (p * scale).astype(np.float32)
    return np.where(z < EXP_CUTOFF, _F(0.0), out).astype(np.float32)


def _topk_rows(scores: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries per row, largest first, ties -> lower index.
    Entries equal to -inf are never selected before finite ones."""
    # stable sort of the negated scores keeps equal scores in ascending index order;
    # adding 0.0 turns -0.0 into +0.0 so that the two compare (and sort) as equal
    neg = -(scores + np.float32(0.0))
    order = np.argsort(neg, axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


def softmax64(logits: np.ndarray) -> np.ndarray:
    lg = logits.astype(np.float64)
    lg = lg - lg.max(axis=1, keepdims=True)
    e = np.exp(lg)
    return e / e.sum(axis=1, keepdims=True)


def device_sums_mode1(logits: np.ndarray, ids0: np.ndarray, expert_device: np.ndarray,
                      D: int) -> np.ndarray:
    """float32 per-device sums of exp_ref(l - max) over the unpruned top-k, slot order."""
    T, k = ids0.shape
    mx = logits.max(axis=1, keepdims=True).astype(np.float32)
    sums = np.zeros((T, D), dtype=np.float32)
    rows = np.arange(T)
    for s in range(k):                                  # sequential in slot order
        e = ids0[:, s]
        q = exp_ref((logits[rows, e] - mx[:, 0]).astype(np.float32))
        dev = expert_device[e]
        sums[rows, dev] = (sums[rows, dev] + q).astype(np.float32)
    return sums


def route(logits: np.ndarray, k: int, D: int, expert_pos: np.ndarray | None = None,
          n_d: int = 0, prune_mode: int = 1, renorm: int = 1, sim_table: np.ndarray | None = None):
    """Return (ids [T,k] int32, w [T,k] float64).

    expert_pos[e] is expert e's placement position; its device is pos // (E/D).
    sim_table [E, E-1] is the similarity table of prune_mode 3.
    """
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    assert E % D == 0 and 1 <= k <= E
    G = E // D
    if expert_pos is None:
        expert_pos = np.arange(E, dtype=np.int32)
    expert_device = (np.asarray(expert_pos) // G).astype(np.int64)

    ids = _topk_rows(logits, k)
    if n_d and n_d > 0:
        assert n_d * G >= k, "pruned range must hold k experts"
        assert prune_mode in (1, 2, 3)
        if prune_mode == 1:
            sums = device_sums_mode1(logits, ids, expert_device, D)
            kept_idx = _topk_rows(sums, n_d)            # highest sums, ties -> lower device
            kept = np.zeros((T, D), dtype=bool)
            np.put_along_axis(kept, kept_idx.astype(np.int64), True, axis=1)
        else:
            kept = np.zeros((T, D), dtype=bool)
            n_kept = np.zeros(T, dtype=np.int64)
            for s in range(k):                          # descending score order
                dev = expert_device[ids[:, s]]
                new = ~kept[np.arange(T), dev] & (n_kept < n_d)
                kept[np.arange(T)[new], dev[new]] = True
                n_kept += new
        if prune_mode == 3:
            assert sim_table is not None and sim_table.shape == (E, E - 1)
            ids = np.array([_replace_by_similarity(ids[t], kept[t], expert_device, sim_table)
                            for t in range(T)], dtype=np.int32).reshape(T, k)
        else:
            allowed = kept[:, expert_device]                # [T, E]
            masked = np.where(allowed, logits, np.float32(-np.inf)).astype(np.float32)
            ids = _topk_rows(masked, k)

    p = softmax64(logits)
    w = np.take_along_axis(p, ids.astype(np.int64), axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    return ids, w


def gram(logits: np.ndarray) -> np.ndarray:
    """H^T H of profiled router scores H [N, E] in float64 (batches add up)."""
    h = np.asarray(logits, dtype=np.float64)
    return h.T @ h


def similarity(g: np.ndarray) -> np.ndarray:
    """Squared cosine similarity of expert columns from their Gram matrix:
    T2[i,j] = g[i,j]^2 / (g[i,i] * g[j,j]), each operation rounded in float64 in this order."""
    g = np.asarray(g, dtype=np.float64)
    dg = np.diag(g)
    return (g * g) / (dg[:, None] * dg[None, :])


def similarity_table(g: np.ndarray) -> np.ndarray:
    """[E, E-1] int32: row i lists the experts j != i by descending T2[i,j], equal -> lower j first."""
    t2 = similarity(g)
    E = t2.shape[0]
    out = np.empty((E, E - 1), dtype=np.int32)
    for i in range(E):
        others = [j for j in range(E) if j != i]
        others.sort(key=lambda j: (-t2[i, j], j))
        out[i] = others
    return out


def _replace_by_similarity(ids_row, kept_dev, expert_device, table):
    """One token of prune_mode 3: ids_row in descending score order -> final ids in walk order."""
    stays = [int(e) for e in ids_row if kept_dev[expert_device[e]]]
    selected = set(stays)
    out = []
    for e in ids_row:
        e = int(e)
        if kept_dev[expert_device[e]]:
            out.append(e)
            continue
        for c in table[e]:
            c = int(c)
            if kept_dev[expert_device[c]] and c not in selected:
                selected.add(c)
                out.append(c)
                break
        else:
            raise AssertionError("no replacement available: n_d * G < k?")
    return out


def router_scores(x: np.ndarray, w_router: np.ndarray) -> np.ndarray:
    """g(x) of Eq. 1 for every token: x [T, d] times w_router [E, d] transposed, in float64."""
    return np.asarray(x, dtype=np.float64) @ np.asarray(w_router, dtype=np.float64).T


def router_scores_loops(x: np.ndarray, w_router: np.ndarray) -> np.ndarray:
    """The same by explicit loops (tiny inputs)."""
    T, d = x.shape
    E = w_router.shape[0]
    out = np.zeros((T, E), dtype=np.float64)
    for t in range(T):
        for e in range(E):
            acc = 0.0
            for i in range(d):
                acc += float(x[t, i]) * float(w_router[e, i])
            out[t, e] = acc
    return out


def selection_margin(logits: np.ndarray, k: int) -> np.ndarray:
    """Per token, the smallest gap between two adjacent scores among the k+1 highest (unpruned
    selection): the k-th/(k+1)-th gap decides membership, the gaps above it decide slot order.
    A perturbation of the scores smaller than half this margin cannot change ids."""
    lg = np.asarray(logits, dtype=np.float64)
    E = lg.shape[1]
    top = -np.sort(-lg, axis=1)[:, :min(k + 1, E)]
    if top.shape[1] < 2:
        return np.full(lg.shape[0], np.inf)
    return np.min(top[:, :-1] - top[:, 1:], axis=1)


def route_loops(logits: np.ndarray, k: int, D: int, expert_pos=None, n_d: int = 0,
                prune_mode: int = 1, renorm: int = 1):
    """The same rules written token by token with explicit loops (small inputs only)."""
    logits = np.asarray(logits, dtype=np.float32)
    T, E = logits.shape
    G = E // D
    pos = list(range(E)) if expert_pos is None else [int(v) for v in expert_pos]
    dev_of = [pos[e] // G for e in range(E)]

    def pick(cands, row):
        chosen = []
        pool = list(cands)
        for _ in range(k):
            best = None
            for e in pool:
                if best is None or row[e] > row[best] or (row[e] == row[best] and e < best):
                    best = e
            chosen.append(best)
            pool.remove(best)
        return chosen

    ids = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k), dtype=np.float64)
    for t in range(T):
        row = logits[t]
        sel = pick(range(E), row)
        if n_d and n_d > 0:
            if prune_mode == 1:
                mx = np.float32(max(float(v) for v in row))
                sums = [np.float32(0.0)] * D
                for e in sel:
                    q = exp_ref(np.array([np.float32(row[e] - mx)], dtype=np.float32))[0]
                    sums[dev_of[e]] = np.float32(sums[dev_of[e]] + q)
                kept = []
                pool = list(range(D))
                for _ in range(n_d):
                    best = None
                    for j in pool:
                        if best is None or sums[j] > sums[best]:
                            best = j
                    kept.append(best)
                    pool.remove(best)
            else:
                kept = []
                for e in sel:
                    if dev_of[e] not in kept and len(kept) < n_d:
                        kept.append(dev_of[e])
            sel = pick([e for e in range(E) if dev_of[e] in kept], row)
        r64 = row.astype(np.float64)
        ex = np.exp(r64 - r64.max())
        p = ex / ex.sum()
        g = np.array([p[e] for e in sel])
        if renorm:
            g = g / g.sum()
        ids[t] = sel
        w[t] = g
    return ids, w
