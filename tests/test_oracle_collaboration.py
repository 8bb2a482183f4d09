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


def test_collaboration_stats_by_hand_two_experts_per_device():
    """Sec. 3.2 formulas on a 4-expert, 2-device case worked by hand.  Experts {0, 2} sit on device 0
    and {1, 3} on device 1.  Off-diagonal counts: C01=4 C02=8 C03=2 C12=6 C13=1 C23=3, largest 8, so
    P = C / 8.  S_0 = {(0,2), (2,0)}: C_intra^0 = (8+8)/8 / 2 = 1.  S_1 = {(1,3), (3,1)}:
    C_intra^1 = (1+1)/8 / 2 = 1/8.  C_inter^{0,1} = (P01 + P03 + P21 + P23) / (2*2)
    = (4+2+6+3)/8 / 4 = 15/32, and C_inter^{1,0} is the same by symmetry of C.
    Intra share of the off-diagonal mass: 2*(8+1) / (2*24) = 3/8."""
    C = np.zeros((4, 4), dtype=np.int64)
    for (i, j), v in {(0, 1): 4, (0, 2): 8, (0, 3): 2, (1, 2): 6, (1, 3): 1, (2, 3): 3}.items():
        C[i, j] = C[j, i] = v
    np.fill_diagonal(C, [14, 11, 17, 6])            # loads: must not enter any of the figures
    pos = np.array([0, 2, 1, 3])                    # expert -> placement position (G = 2)
    st = collaboration.collaboration_stats(C, pos, 2)
    assert np.allclose(st["c_intra"], [1.0, 0.125], rtol=0, atol=1e-15)
    assert np.allclose(st["c_inter"], [[0.0, 15 / 32], [15 / 32, 0.0]], rtol=0, atol=1e-15)
    assert np.isclose(st["intra_fraction"], 3 / 8) and np.isclose(st["inter_fraction"], 5 / 8)


def test_collaboration_stats_by_hand_three_experts_per_device():
    """6 experts, 2 devices of 3, asymmetric blocks.  Device 0 = {0, 1, 2}, device 1 = {3, 4, 5}.
    Inside device 0: C01=6 C02=2 C12=4 (sum 12); inside device 1: C34=12 C35=3 C45=0 (sum 15);
    across: C03=1 C04=2 C05=3 C13=4 C14=5 C15=6 C23=7 C24=8 C25=9 (sum 45).  Largest count 12.
    |S_d| = 3*2 = 6 ordered pairs: C_intra^0 = 2*12/12 / 6 = 1/3, C_intra^1 = 2*15/12 / 6 = 5/12.
    C_inter^{0,1} = 45/12 / 9 = 5/12.  Intra share = 2*(12+15) / (2*(12+15+45)) = 27/72 = 3/8."""
    vals = {(0, 1): 6, (0, 2): 2, (1, 2): 4, (3, 4): 12, (3, 5): 3, (4, 5): 0,
            (0, 3): 1, (0, 4): 2, (0, 5): 3, (1, 3): 4, (1, 4): 5, (1, 5): 6, (2, 3): 7, (2, 4): 8, (2, 5): 9}
    C = np.zeros((6, 6), dtype=np.int64)
    for (i, j), v in vals.items():
        C[i, j] = C[j, i] = v
    np.fill_diagonal(C, 99)
    st = collaboration.collaboration_stats(C, np.arange(6), 2)
    assert np.allclose(st["c_intra"], [1 / 3, 5 / 12], rtol=0, atol=1e-15)
    assert np.allclose(st["c_inter"], [[0.0, 5 / 12], [5 / 12, 0.0]], rtol=0, atol=1e-15)
    assert np.isclose(st["intra_fraction"], 3 / 8)
    # a permuted placement moves experts, not the definition: swap experts 2 and 3 between the devices
    pos = np.array([0, 1, 3, 2, 4, 5])              # device 0 = {0, 1, 3}, device 1 = {2, 4, 5}
    st = collaboration.collaboration_stats(C, pos, 2)
    # device 0: C01=6 C03=1 C13=4 -> 11; device 1: C24=8 C25=9 C45=0 -> 17; across: 72 - 28 = 44
    assert np.allclose(st["c_intra"], [2 * 11 / 12 / 6, 2 * 17 / 12 / 6], rtol=0, atol=1e-15)
    assert np.allclose(st["c_inter"][0, 1], 44 / 12 / 9, rtol=0, atol=1e-15)
    assert np.isclose(st["intra_fraction"], 28 / 72)
