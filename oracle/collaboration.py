"""CPU oracle: expert co-activation counts, collaboration statistics and the greedy
collaboration-aware expert placement.

TEST INFRASTRUCTURE ONLY (see oracle/routing.py for who may import this).

Followed passages (paper):
  * co-activation graph C_ij = number of tokens that select both expert i and expert j
    (Preliminary, equation after Eq. 1); the diagonal (i = j) is the expert's load;
  * intra- / inter-collaboration averages of a placement (Section 3.2);
  * "Building expert placement" (Section 3.2, Algorithm 1): device 0 starts from the most
    collaborative pair; every later device starts from the unused expert that collaborates
    least with the experts already placed; a device is then grown with the unused expert
    that collaborates most with the experts already on it.

Readings where the printed algorithm is off or silent:
  * a device is filled to exactly N_e / N_d experts (the printed loop bound would add one more);
  * the divisor of the intra score is the size of the device's list; all candidates of one
    step share their divisor (and the normalisation C -> P is one positive scale), so
    candidates are compared by integer sums of C: no floats, no rounding questions;
  * the diagonal of C never takes part (arg-max over off-diagonal pairs only);
  * ties: most collaborative pair -> smallest (i, j) with i < j; minimal / maximal candidate
    -> lowest expert index;
  * needs at least 2 experts per device.
"""
from __future__ import annotations

import numpy as np


def coactivation_loops(ids: np.ndarray, E: int) -> np.ndarray:
    """Triple loop: for every token, every ordered pair of its selected experts."""
    C = np.zeros((E, E), dtype=np.int64)
    for t in range(ids.shape[0]):
        for a in ids[t]:
            for b in ids[t]:
                C[int(a), int(b)] += 1
    return C


def coactivation(ids: np.ndarray, E: int) -> np.ndarray:
    """C = A^T A with A[t, e] = 1 if token t selects expert e."""
    T = ids.shape[0]
    A = np.zeros((T, E), dtype=np.int64)
    A[np.arange(T)[:, None], ids] = 1
    return A.T @ A


def collaboration_stats(C: np.ndarray, expert_pos: np.ndarray, D: int):
    """Fraction of co-activated pairs (off-diagonal mass of C) that sit on one device, and the
    paper's per-device / per-device-pair averages of P = C / max offdiag C."""
    E = C.shape[0]
    G = E // D
    dev = np.asarray(expert_pos) // G
    off = C.astype(np.float64).copy()
    np.fill_diagonal(off, 0.0)
    same = dev[:, None] == dev[None, :]
    total = off.sum()
    intra_frac = float(off[same].sum() / total) if total > 0 else 0.0
    P = off / off.max() if off.max() > 0 else off
    c_intra = np.zeros(D)
    c_inter = np.zeros((D, D))
    for a in range(D):
        ia = np.nonzero(dev == a)[0]
        pairs = [(i, j) for i in ia for j in ia if i != j]
        c_intra[a] = np.mean([P[i, j] for i, j in pairs]) if pairs else 0.0
        for b in range(D):
            if a != b:
                ib = np.nonzero(dev == b)[0]
                c_inter[a, b] = P[np.ix_(ia, ib)].mean()
    return {"intra_fraction": intra_frac, "inter_fraction": 1.0 - intra_frac,
            "c_intra": c_intra, "c_inter": c_inter}


def greedy_placement(C: np.ndarray, D: int):
    """Algorithm 1 on integer counts.  Returns (L, expert_pos): L[d] lists device d's experts in
    the order they were pushed (= slot order); expert_pos[e] = d * G + slot."""
    C = np.asarray(C, dtype=np.int64)
    E = C.shape[0]
    assert E % D == 0
    G = E // D
    assert G >= 2, "needs at least two experts per device"
    used = []
    L = [[] for _ in range(D)]
    for d in range(D):
        if d == 0:
            best = None
            for i in range(E):
                for j in range(i + 1, E):
                    if best is None or C[i, j] > C[best[0], best[1]]:
                        best = (i, j)
            L[d] += [best[0], best[1]]
            used += [best[0], best[1]]
        else:
            cand, cand_val = None, None
            for e in range(E):
                if e in used:
                    continue
                val = sum(int(C[t, e]) for t in used)
                if cand is None or val < cand_val:
                    cand, cand_val = e, val
            L[d].append(cand)
            used.append(cand)
        while len(L[d]) < G:
            cand, cand_val = None, None
            for e in range(E):
                if e in used:
                    continue
                val = sum(int(C[t, e]) for t in L[d])
                if cand is None or val > cand_val:
                    cand, cand_val = e, val
            L[d].append(cand)
            used.append(cand)
    expert_pos = np.zeros(E, dtype=np.int32)
    for d in range(D):
        for s, e in enumerate(L[d]):
            expert_pos[e] = d * G + s
    return L, expert_pos
