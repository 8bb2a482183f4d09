"""CPU oracle O-occ: the deduplicated ("collaboration-aware") expert-parallel MoE layer,
step by step in the paper's order and notation.

TEST INFRASTRUCTURE ONLY (see oracle/routing.py for who may import this).

Followed passages (paper, Section 3.1 and Appendix A):
  * three tensor states ORI / SFD / EPD and the two re-index matrices (Section 3.1);
  * pipeline order: router -> BRIM_0 -> Dispatch -> all-to-all -> BRIM_1 ->
    SMM-scattering -> weight modulation -> SMM-merging -> all-to-all -> Combine
    (Appendix A.1, pipeline pseudo-code);
  * "Building BRIM_0", "Dispatch", "Building BRIM_1", "SMM with Scattering",
    "Weight Modulation", "SMM with Merging", "Combine" (Appendix A.2);
  * replica count C_T = N_sfd / N_ori and its bounds (Section 2.2).

Readings:
  * one source rank is simulated: segment d of the send buffer *is* what device d
    receives, and the return trip is the identity;
  * the BRIM_0 counter runs over all devices (device-major, token-ascending), so its
    values are global rows of the send buffer; absent entries are -1 and the count of
    SFD rows is the number of non-negative entries (0 is a valid row);
  * BRIM_1 is built per receiving device over that device's SFD segment, local experts in
    placement-slot order; its values are EPD rows local to the device;
  * Dispatch / Combine skip the -1 entries (the printed loops do not mask them);
  * the expert is SwiGLU: the first SMM produces gate and up projections, the
    intermediate is silu(gate) * up; routing weights multiply the intermediate
    (weight modulation), not the output;
  * merging accumulates serially over local experts in slot order (the paper's
    "serially aggregating" alternative to atomic adds), into a zeroed SFD tensor;
  * shared experts are replicated on every device, cost no dispatch bytes, and are added
    to the combined output.
Float arithmetic is float64 (or the ``acc`` type given) from the stored inputs.
"""
from __future__ import annotations

import dataclasses
from typing import List

import numpy as np


def silu(z):
    return z / (1.0 + np.exp(-z))


def placement_lists(expert_pos: np.ndarray, D: int) -> List[List[int]]:
    """L[d] = experts kept on device d, in slot order."""
    E = len(expert_pos)
    G = E // D
    L = [[-1] * G for _ in range(D)]
    for e in range(E):
        p = int(expert_pos[e])
        L[p // G][p % G] = e
    assert all(v >= 0 for row in L for v in row), "expert_pos must be a permutation"
    return L


# ------------------------------------------------------------------ BRIM_0 (Appendix A.2)
def _running_index(present: list) -> list:
    """Row-major numbering of the True cells of a list of rows: the n-th True cell (counting from
    0 across rows, left to right) gets n, every False cell gets -1."""
    flat = [c for row in present for c in row]
    seen = np.cumsum(flat)
    width = len(present[0]) if present else 0
    return [[int(seen[r * width + c]) - 1 if flat[r * width + c] else -1 for c in range(width)]
            for r in range(len(present))]


def build_brim_0_loops(ids: np.ndarray, L: List[List[int]]) -> np.ndarray:
    """Pure-Python twin: the (device x token) membership table, then its row-major numbering
    (device-major, token-ascending, one count across all devices)."""
    present = [[bool(set(int(e) for e in ids[t]) & set(L[d])) for t in range(ids.shape[0])]
               for d in range(len(L))]
    return np.asarray(_running_index(present), dtype=np.int64).reshape(len(L), ids.shape[0])


def build_brim_0(ids: np.ndarray, L: List[List[int]]) -> np.ndarray:
    """Same matrix; the inner token loop is a running count over a boolean vector."""
    T = ids.shape[0]
    D = len(L)
    brim_0 = np.full((D, T), -1, dtype=np.int64)
    ctr = 0
    for d in range(D):
        activates = np.isin(ids, np.asarray(L[d])).any(axis=1)
        n = int(activates.sum())
        brim_0[d, activates] = ctr + np.arange(n)
        ctr += n
    return brim_0


# ------------------------------------------------------------------ Dispatch (Appendix A.2)
def dispatch(x, ids, w, brim_0):
    """ORI -> SFD: row t is written to every non-negative BRIM_0[d, t]; ids and w ride along."""
    n_sfd = int((brim_0 >= 0).sum())
    x_sfd = np.empty((n_sfd, x.shape[1]), dtype=x.dtype)
    ids_sfd = np.empty((n_sfd, ids.shape[1]), dtype=ids.dtype)
    w_sfd = np.empty((n_sfd, w.shape[1]), dtype=w.dtype)
    for d in range(brim_0.shape[0]):
        v = brim_0[d]
        present = v >= 0
        x_sfd[v[present]] = x[present]
        ids_sfd[v[present]] = ids[present]
        w_sfd[v[present]] = w[present]
    return x_sfd, ids_sfd, w_sfd


# ------------------------------------------------------------------ BRIM_1 (Appendix A.2)
def build_brim_1_loops(ids_sfd: np.ndarray, w_sfd: np.ndarray, L_loc: List[int]):
    """Pure-Python twin: the (local expert x SFD row) membership table, its row-major numbering
    (local-expert-major), and beside it the routing weight of the matching slot."""
    n_sfd, k = ids_sfd.shape
    slot = [[next((s for s in range(k) if int(ids_sfd[t, s]) == expert), None) for t in range(n_sfd)]
            for expert in L_loc]
    brim_1 = np.asarray(_running_index([[s is not None for s in row] for row in slot]),
                        dtype=np.int64).reshape(len(L_loc), n_sfd)
    brim_w = np.zeros((len(L_loc), n_sfd), dtype=np.float64)
    for e, row in enumerate(slot):
        for t, s in enumerate(row):
            if s is not None:
                brim_w[e, t] = w_sfd[t, s]
    return brim_1, brim_w


def build_brim_1(ids_sfd: np.ndarray, w_sfd: np.ndarray, L_loc: List[int]):
    n_sfd = ids_sfd.shape[0]
    brim_1 = np.full((len(L_loc), n_sfd), -1, dtype=np.int64)
    brim_w = np.zeros((len(L_loc), n_sfd), dtype=np.float64)
    ctr = 0
    for e, expert in enumerate(L_loc):
        hit = ids_sfd == expert
        activates = hit.any(axis=1)
        n = int(activates.sum())
        brim_1[e, activates] = ctr + np.arange(n)
        brim_w[e, activates] = w_sfd[activates][hit[activates]]
        ctr += n
    return brim_1, brim_w


# ------------------------------------------------------------------ expert computing
def smm_scattering(x_sfd, w_gate_loc, w_up_loc, brim_1, acc):
    """SFD -> EPD: for local expert e, rows t with BRIM_1[e,t] >= 0 are projected and written
    to EPD row BRIM_1[e,t].  Returns the SwiGLU intermediate [n_epd, f]."""
    n_epd = int((brim_1 >= 0).sum())
    f = w_gate_loc[0].shape[0]
    x_epd = np.zeros((n_epd, f), dtype=acc)
    for e in range(brim_1.shape[0]):
        v = brim_1[e]
        present = v >= 0
        if not present.any():
            continue
        a = x_sfd[present].astype(acc)
        g = a @ w_gate_loc[e].astype(acc).T
        u = a @ w_up_loc[e].astype(acc).T
        x_epd[v[present]] = silu(g) * u
    return x_epd


def weight_modulate(x_epd, brim_1, brim_w):
    out = x_epd.copy()
    for e in range(brim_1.shape[0]):
        v = brim_1[e]
        present = v >= 0
        out[v[present]] = x_epd[v[present]] * brim_w[e, present][:, None]
    return out


def smm_merging(x_epd, w_down_loc, brim_1, d_out, acc):
    """EPD -> SFD: zeroed SFD tensor, local experts added one after another (slot order)."""
    n_sfd = brim_1.shape[1]
    x_sfd = np.zeros((n_sfd, d_out), dtype=acc)
    for e in range(brim_1.shape[0]):
        v = brim_1[e]
        present = v >= 0
        if not present.any():
            continue
        x_sfd[present] += x_epd[v[present]] @ w_down_loc[e].astype(acc).T
    return x_sfd


# ------------------------------------------------------------------ Combine (Appendix A.2)
def combine(x_sfd, brim_0, acc):
    D, T = brim_0.shape
    x_ori = np.zeros((T, x_sfd.shape[1]), dtype=acc)
    for d in range(D):                       # sequential over devices
        v = brim_0[d]
        present = v >= 0
        x_ori[present] += x_sfd[v[present]]
    return x_ori


@dataclasses.dataclass
class OccultTrace:
    brim_0: np.ndarray            # [D, T] global SFD rows, -1 absent
    dev_count: np.ndarray         # [D]
    brim_1: list                  # per device [G, n_sfd_d] local EPD rows, -1 absent
    brim_w: list                  # per device [G, n_sfd_d]
    n_sfd: int
    n_epd: int
    c_t: float
    x_sfd: np.ndarray | None      # dispatched hidden rows (the all-to-all payload)
    y_sfd: np.ndarray | None      # merged expert outputs per SFD row (the return payload)
    y: np.ndarray | None          # layer output, ORI order
    ids_sfd: np.ndarray | None = None   # routing of each dispatched row's token (rides along with the payload)
    w_sfd: np.ndarray | None = None


def moe_forward(x, ids, w, expert_pos, D, w_gate=None, w_up=None, w_down=None, S=0,
                acc=np.float64, bypass_scale=None) -> OccultTrace:
    """One forward pass of the refactored pipeline for one simulated source rank.

    With ``bypass_scale`` (one number per expert) the expert network is replaced by
    E_e(v) = bypass_scale[e] * v, which makes every sum exact for small-integer inputs and
    power-of-two gates: the bit-exactness pin for dispatch + two-stage combine.
    """
    T, d = x.shape
    E = len(expert_pos)
    L = placement_lists(expert_pos, D)
    # (2) BRIM_0, (3) Dispatch
    brim_0 = build_brim_0(ids, L)
    x_sfd, ids_sfd, w_sfd = dispatch(x, ids, w, brim_0)
    dev_count = (brim_0 >= 0).sum(axis=1)
    # (4) first all-to-all: device j receives rows [offset_j, offset_j + count_j)
    offs = np.concatenate([[0], np.cumsum(dev_count)])
    brim_1_all, brim_w_all = [], []
    y_sfd = None
    compute = bypass_scale is not None or w_gate is not None
    if compute:
        y_sfd = np.zeros((x_sfd.shape[0], d), dtype=acc)
    n_epd = 0
    for j in range(D):
        seg = slice(int(offs[j]), int(offs[j + 1]))
        # (5) BRIM_1 on the receiver
        brim_1, brim_w = build_brim_1(ids_sfd[seg], w_sfd[seg], L[j])
        brim_1_all.append(brim_1)
        brim_w_all.append(brim_w)
        n_epd += int((brim_1 >= 0).sum())
        if not compute:
            continue
        # (6) computing with local experts
        if bypass_scale is not None:
            xs = x_sfd[seg].astype(acc)
            x_epd = np.zeros((int((brim_1 >= 0).sum()), d), dtype=acc)
            for e in range(len(L[j])):
                v = brim_1[e]
                present = v >= 0
                x_epd[v[present]] = xs[present]
            x_epd = weight_modulate(x_epd, brim_1, brim_w)
            out = np.zeros((xs.shape[0], d), dtype=acc)
            for e in range(len(L[j])):
                v = brim_1[e]
                present = v >= 0
                out[present] += x_epd[v[present]] * acc(bypass_scale[L[j][e]])
            y_sfd[seg] = out
        else:
            wg = [w_gate[e] for e in L[j]]
            wu = [w_up[e] for e in L[j]]
            wd = [w_down[e] for e in L[j]]
            x_epd = smm_scattering(x_sfd[seg], wg, wu, brim_1, acc)
            x_epd = weight_modulate(x_epd, brim_1, brim_w)
            y_sfd[seg] = smm_merging(x_epd, wd, brim_1, d, acc)
    y = None
    if compute:
        # (7) return trip = identity, (8) Combine
        y = combine(y_sfd, brim_0, acc)
        if S and w_gate is not None:
            xs = x.astype(acc)
            for s in range(S):
                g = xs @ w_gate[E + s].astype(acc).T
                u = xs @ w_up[E + s].astype(acc).T
                y += (silu(g) * u) @ w_down[E + s].astype(acc).T
    n_sfd = int(dev_count.sum())
    return OccultTrace(brim_0, dev_count, brim_1_all, brim_w_all, n_sfd, n_epd, n_sfd / T,
                       x_sfd, y_sfd, y, ids_sfd, w_sfd)


def exchange_bytes(T: int, k: int, n_sfd: int, row_bytes: int):
    """Hidden-row bytes over the two trips: standard k replicas per token vs one per device."""
    return {"bytes_std": 2 * T * k * row_bytes, "bytes_occ": 2 * n_sfd * row_bytes,
            "bytes_meta": n_sfd * k * 8}
