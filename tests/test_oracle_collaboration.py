"""Pins for oracle/collaboration.py: counting identities of the co-activation graph and the
greedy placement (hand trace, partition property, planted blocks)."""
import numpy as np
import pytest

from inputs import workloads as wl
from oracle import collaboration, occult_ref, routing


def test_coactivation_identities_and_loop_twin():
    E, k, T = 16, 4, 400
    ids, _ = routing.route(wl.random_logits(T, E, seed=2), k, D=4)
    C = collaboration.coactivation(ids, E)
    assert np.array_equal(C, collaboration.coactivation_loops(ids, E))
    assert np.array_equal(C, C.T)
    load = np.bincount(ids.reshape(-1), minlength=E)
    assert np.array_equal(np.diag(C), load)
    assert np.trace(C) == T * k
    assert C.sum() == T * k * k
    assert np.array_equal(C.sum(axis=1), k * load)


def test_coactivation_tiny_by_hand():
    ids = np.array([[0, 1], [1, 2], [0, 1]], dtype=np.int32)
    C = collaboration.coactivation(ids, 3)
    assert C.tolist() == [[2, 2, 0], [2, 3, 1], [0, 1, 1]]


def test_placement_hand_trace(golden_dir):
    pairs, L_want, pos_want = [], None, None
    for line in open(f"{golden_dir}/placement_e6_d3.txt"):
        tok = line.split()
        if not tok or tok[0].startswith("#"):
            continue
        if tok[0] == "pair":
            pairs.append(tuple(int(v) for v in tok[1:]))
        elif tok[0] == "L":
            L_want = [[int(v) for v in part.split()] for part in " ".join(tok[1:]).split("/")]
        elif tok[0] == "expert_pos":
            pos_want = [int(v) for v in tok[1:]]
    C = np.zeros((6, 6), dtype=np.int64)
    for i, j, v in pairs:
        C[i, j] = C[j, i] = v
    np.fill_diagonal(C, 1000)                   # loads on the diagonal must not matter
    L, pos = collaboration.greedy_placement(C, 3)
    assert L == L_want
    assert pos.tolist() == pos_want


@pytest.mark.parametrize("E,D", [(16, 4), (64, 16), (60, 4), (12, 6)])
def test_placement_is_a_partition(E, D):
    rng = np.random.default_rng(E)
    A = rng.integers(0, 50, size=(E, E))
    C = A + A.T
    L, pos = collaboration.greedy_placement(C, D)
    G = E // D
    assert sorted(e for row in L for e in row) == list(range(E))
    assert all(len(row) == G for row in L)
    assert sorted(pos.tolist()) == list(range(E))
    for d in range(D):
        for s, e in enumerate(L[d]):
            assert pos[e] == d * G + s


def test_planted_blocks_are_recovered_and_replicas_drop_to_lower_bound():
    # routing that always picks its k experts inside one hidden group of G experts
    E, D, k, T = 32, 8, 4, 4000
    G = E // D
    rng = np.random.default_rng(6)
    hidden = rng.permutation(E).reshape(D, G)              # hidden groups
    grp = rng.integers(0, D, size=T)
    ids = np.stack([rng.permutation(hidden[g])[:k] for g in grp]).astype(np.int32)
    w = np.full((T, k), 1.0 / k)
    C = collaboration.coactivation(ids, E)
    L, pos = collaboration.greedy_placement(C, D)
    assert sorted(sorted(r) for r in L) == sorted(sorted(r.tolist()) for r in hidden)
    tr = occult_ref.moe_forward(np.zeros((T, 1)), ids, w, pos, D)
    assert tr.c_t == 1.0                                    # = ceil(k / G), the lower bound
    tr0 = occult_ref.moe_forward(np.zeros((T, 1)), ids, w, wl.contiguous_placement(E, D), D)
    assert tr0.c_t > 2.0
    st = collaboration.collaboration_stats(C, pos, D)
    assert st["intra_fraction"] == 1.0 and st["inter_fraction"] == 0.0


def test_collaboration_stats_fraction_matches_pair_count():
    E, D, k, T = 16, 4, 4, 300
    G = E // D
    ids, _ = routing.route(wl.random_logits(T, E, seed=12), k, D)
    pos = wl.random_placement(E, D, seed=4)
    C = collaboration.coactivation(ids, E)
    st = collaboration.collaboration_stats(C, pos, D)
    same = diff = 0
    for t in range(T):
        for a in ids[t]:
            for b in ids[t]:
                if a != b:
                    if pos[a] // G == pos[b] // G:
                        same += 1
                    else:
                        diff += 1
    assert np.isclose(st["intra_fraction"], same / (same + diff))
