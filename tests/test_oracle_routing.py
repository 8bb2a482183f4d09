"""Pins for oracle/routing.py: library reductions, loop twin, pruning special cases
(paper Section 3.3 and Table 1) and the exp_ref decision arithmetic."""
import itertools

import numpy as np
import pytest
import torch

from inputs import workloads as wl
from oracle import moe_std, routing


def test_exp_ref_matches_libm_within_float32_rounding():
    z = -np.abs(np.random.default_rng(0).standard_normal(200000).astype(np.float32)) * 12
    z = np.concatenate([z, np.float32([0.0, -1e-8, -79.99, -80.0, -80.01, -200.0])])
    got = routing.exp_ref(z).astype(np.float64)
    want = np.exp(z.astype(np.float64))
    live = z >= routing.EXP_CUTOFF
    rel = np.abs(got[live] - want[live]) / want[live]
    assert rel.max() < 4e-7
    assert np.all(got[~live] == 0.0)
    assert routing.exp_ref(np.float32([0.0]))[0] == np.float32(1.0)
    # monotone (the decision only needs order): non-decreasing on a fine grid
    g = np.linspace(-80, 0, 400001).astype(np.float32)
    assert np.all(np.diff(routing.exp_ref(g).astype(np.float64)) >= -1e-12 * 1.0)


def test_exp_ref_is_fma_free_sequence():
    # one value worked through in float64 steps rounded to float32 after every operation
    z = np.float32(-3.3)
    f = np.float32
    n = f(np.rint(f(z * routing.LOG2E)))
    r = f(f(z - f(n * routing.LN2_HI)) - f(n * routing.LN2_LO))
    p = routing.EXP_COEF[7]
    for i in range(6, -1, -1):
        p = f(f(float(p) * float(r)))          # product rounded once ...
        p = f(float(p) + float(routing.EXP_COEF[i]))   # ... then the sum rounded once
    want = f(float(p) * 2.0 ** float(n))
    assert routing.exp_ref(np.array([z]))[0] == want


@pytest.mark.parametrize("renorm", [0, 1])
def test_unpruned_values_match_torch_softmax_topk(renorm):
    lg = wl.random_logits(512, 64, seed=3, scale=1.5)
    ids, w = routing.route(lg, k=8, D=8, renorm=renorm)
    p = torch.softmax(torch.from_numpy(lg).double(), dim=1)
    tv, ti = torch.topk(p, 8, dim=1)
    if renorm:
        tv = tv / tv.sum(dim=1, keepdim=True)
    # no exact ties in continuous scores: indices agree too
    assert np.array_equal(ids, ti.numpy().astype(np.int32))
    assert np.allclose(w, tv.numpy(), rtol=1e-12, atol=0)
    if renorm:
        assert np.allclose(w.sum(axis=1), 1.0, atol=1e-14)
    assert np.all(np.diff(w, axis=1) <= 0)        # slot 0 = highest


def test_selection_equals_independent_definition_in_moe_std():
    lg = wl.random_logits(300, 16, seed=5, ties=True)
    ids_a, w_a = routing.route(lg, k=4, D=4, renorm=1)
    ids_b, w_b = moe_std.topk_by_definition(lg, 4, 1)
    assert np.array_equal(ids_a, ids_b)
    assert np.allclose(w_a, w_b, rtol=1e-13)


def test_tie_rule_lower_index_first_and_signed_zero():
    lg = np.zeros((1, 8), dtype=np.float32)
    lg[0, 2] = -0.0
    ids, w = routing.route(lg, k=3, D=4)
    assert ids.tolist() == [[0, 1, 2]]
    lg = np.float32([[1, 3, 3, 2, 3, 0, 2, 1]])
    ids, _ = routing.route(lg, k=5, D=4)
    assert ids.tolist() == [[1, 2, 4, 3, 6]]


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("ties", [False, True])
def test_vectorised_route_equals_loop_twin(mode, ties):
    E, D, k = 12, 4, 3
    lg = wl.random_logits(200, E, seed=11 + mode, ties=ties)
    pos = wl.random_placement(E, D, seed=2)
    for n_d in (0, 1, 2, 3):
        a = routing.route(lg, k, D, pos, n_d=n_d, prune_mode=mode, renorm=1)
        b = routing.route_loops(lg, k, D, pos, n_d=n_d, prune_mode=mode, renorm=1)
        assert np.array_equal(a[0], b[0])
        assert np.allclose(a[1], b[1], rtol=1e-13)


def _devices_touched(ids, pos, G):
    dev = (np.asarray(pos)[ids] // G)
    return np.array([len(set(r)) for r in dev.tolist()])


@pytest.mark.parametrize("mode", [1, 2])
def test_pruning_special_cases(mode, golden_dir):
    E, D, k = 64, 8, 8
    G = E // D
    lg = wl.random_logits(2048, E, seed=21, scale=1.1)
    pos = wl.contiguous_placement(E, D)
    ids0, w0 = routing.route(lg, k, D, pos)
    c0 = _devices_touched(ids0, pos, G)
    for n_d in (1, 2, 4, 8):
        ids, w = routing.route(lg, k, D, pos, n_d=n_d, prune_mode=mode)
        c = _devices_touched(ids, pos, G)
        assert np.all(c <= n_d)                                   # at most n_d devices
        assert all(len(set(r)) == k for r in ids.tolist())        # still k distinct experts
        assert np.allclose(w.sum(axis=1), 1.0, atol=1e-13)
        untouched = c0 <= n_d                                     # footnote of Section 3.3
        assert np.array_equal(ids[untouched], ids0[untouched])
        assert np.allclose(w[untouched], w0[untouched], rtol=1e-13)
        if n_d >= min(k, D):                                      # full range = plain top-k
            assert np.array_equal(ids, ids0)
        if n_d == 1:                                              # Table 1, last column
            assert np.all(c == 1)
    # Table 1 upper bounds per pruned column
    rows = [l.split() for l in open(f"{golden_dir}/table1_replicas.txt") if l[0] != "#"]
    ub = {r[0]: float(r[1]) for r in rows}
    assert ub["occult_prune_2"] == 2 and ub["occult_prune_1"] == 1


def test_mode2_keeps_first_distinct_devices_in_score_order():
    # E=8, D=4 (G=2); scores descending on experts 6,0,7,2,4 -> devices 3,0,3,1,2
    lg = np.float32([[5.0, 0.1, 3.0, 0.0, 2.0, 0.2, 6.0, 4.0]])
    # kept devices {3, 0}: candidates 6,7,0,1
    ids, _ = routing.route(lg, k=4, D=4, n_d=2, prune_mode=2)
    assert ids.tolist() == [[6, 0, 7, 1]]
    # mode 1 on the same token: top-4 = 6,0,7,2; sums dev3 = q6+q7, dev0 = q0, dev1 = q2
    ids1, _ = routing.route(lg, k=4, D=4, n_d=2, prune_mode=1)
    assert ids1.tolist() == [[6, 0, 7, 1]]
    # a case where the two rules differ: device 1 holds two mid experts whose sum beats device 0
    lg = np.float32([[4.0, -9.0, 3.9, 3.9, -9.0, -9.0, 5.0, -9.0]])
    a, _ = routing.route(lg, k=4, D=4, n_d=2, prune_mode=1)   # sums: dev3=q6, dev1=q2+q3, dev0=q0
    b, _ = routing.route(lg, k=4, D=4, n_d=2, prune_mode=2)   # order 6,0,... -> devices 3,0
    assert set((np.array(a[0]) // 2).tolist()) == {3, 1}
    assert set((np.array(b[0]) // 2).tolist()) == {3, 0}


def test_mode1_device_choice_brute_force_float64_margin():
    # wherever float64 sums separate the devices clearly, the float32 decision agrees
    E, D, k, n_d = 16, 4, 4, 2
    lg = wl.random_logits(4000, E, seed=8)
    pos = wl.contiguous_placement(E, D)
    ids0, _ = routing.route(lg, k, D, pos)
    ids, _ = routing.route(lg, k, D, pos, n_d=n_d, prune_mode=1)
    p = routing.softmax64(lg)
    G = E // D
    checked = 0
    for t in range(lg.shape[0]):
        s = np.zeros(D)
        for e in ids0[t]:
            s[e // G] += p[t, e]
        order = np.argsort(-s, kind="stable")
        if s[order[n_d - 1]] - s[order[n_d]] > 1e-6 * s[order[0]]:
            kept = set(order[:n_d].tolist())
            assert set((ids[t] // G).tolist()) <= kept
            checked += 1
    assert checked > 3900


def test_all_subsets_single_token():
    # every possible top-k set of one token is produced by suitable scores and is returned as-is
    E, k = 6, 3
    for sub in itertools.combinations(range(E), k):
        lg = np.full((1, E), -1.0, dtype=np.float32)
        for rank, e in enumerate(sub):
            lg[0, e] = 3.0 - rank
        ids, w = routing.route(lg, k, D=3)
        assert ids[0].tolist() == list(sub)


# ---- router scores (Eq. 1: g(x) is a linear projection) ---------------------------------------

def test_router_scores_match_loops_and_pick_columns():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((5, 7))
    wr = rng.standard_normal((4, 7))
    got = routing.router_scores(x, wr)
    assert np.allclose(got, routing.router_scores_loops(x, wr), rtol=1e-13, atol=1e-13)
    # a one-hot hidden state reads one column of W_r; the projection is linear
    eye = np.eye(7)
    assert np.array_equal(routing.router_scores(eye, wr), wr.T)
    assert np.allclose(routing.router_scores(2.0 * x + eye[:5], wr), 2.0 * got + wr.T[:5], rtol=1e-13, atol=1e-13)
    # not transposed: a rectangular case with distinct T, E, d has the right shape
    assert got.shape == (5, 4)


def test_workload_logits_are_the_router_scores():
    shape = wl.CONFIGS["tiny_f32"]
    wk = wl.make_workload(shape, with_experts=False)
    ref = routing.router_scores(wk.x, wk.w_router)
    assert np.max(np.abs(wk.logits - ref)) <= 1e-5 * np.sqrt(np.mean(ref ** 2))


def test_selection_margin_bounds_what_a_perturbation_can_change():
    rng = np.random.default_rng(11)
    lg = rng.standard_normal((400, 16)).astype(np.float32)
    k = 4
    margin = routing.selection_margin(lg, k)
    assert margin.shape == (400,) and np.all(margin >= 0)
    ids0, _ = routing.route(lg, k, 4)
    # hand-made rows: gap structure known
    row = np.array([[5.0, 4.0, 3.5, 1.0, 0.0, -1.0]], dtype=np.float32)
    assert routing.selection_margin(row, 2)[0] == 0.5      # min(5-4, 4-3.5)
    assert routing.selection_margin(row, 3)[0] == 0.5      # min(1, .5, 2.5)
    # perturbations below half the margin never change the selection; tokens that do change under a
    # larger perturbation all have a margin below twice its size
    for eps in (1e-4, 1e-2):
        noise = rng.uniform(-eps, eps, lg.shape).astype(np.float32)
        ids1, _ = routing.route(lg + noise, k, 4)
        changed = np.any(ids0 != ids1, axis=1)
        assert np.all(margin[changed] <= 2 * eps + 1e-6)


# ---- expert-similarity-based pruning (Section 3.3, second criterion; similarity table appendix) ----

def test_similarity_is_squared_cosine_of_columns():
    rng = np.random.default_rng(2)
    h = rng.standard_normal((300, 6))
    h[:, 3] = -2.5 * h[:, 1]                 # anti-parallel columns count as identical (the square)
    h[:, 5] = h[:, 0] - (h[:, 0] @ h[:, 2]) / (h[:, 2] @ h[:, 2]) * h[:, 2]   # orthogonal to column 2
    t2 = routing.similarity(routing.gram(h))
    for i in range(6):
        for j in range(6):
            cos = (h[:, i] @ h[:, j]) / (np.linalg.norm(h[:, i]) * np.linalg.norm(h[:, j]))
            assert abs(t2[i, j] - cos * cos) < 1e-12
    assert np.allclose(np.diag(t2), 1.0) and np.allclose(t2, t2.T)
    assert abs(t2[1, 3] - 1.0) < 1e-12 and t2[2, 5] < 1e-20
    # batches add up; rescaling an expert's scores changes nothing
    g2 = routing.gram(h[:100]) + routing.gram(h[100:])
    assert np.allclose(g2, routing.gram(h), rtol=1e-13)
    assert np.allclose(routing.similarity(routing.gram(h * np.array([1, 7, 1, .1, 3, 1.]))), t2, rtol=1e-12, atol=1e-30)


def test_similarity_table_rows_are_sorted_and_complete():
    rng = np.random.default_rng(4)
    h = rng.standard_normal((200, 9))
    h[:, 7] = h[:, 4]                          # an exact tie for everybody: 4 before 7
    g = routing.gram(h)
    tab = routing.similarity_table(g)
    t2 = routing.similarity(g)
    assert tab.shape == (9, 8)
    for i in range(9):
        assert sorted(tab[i].tolist()) == [j for j in range(9) if j != i]
        vals = t2[i, tab[i]]
        assert np.all(vals[:-1] >= vals[1:])
        for a, b in zip(tab[i][:-1], tab[i][1:]):
            if t2[i, a] == t2[i, b]:
                assert a < b
    assert tab[4][0] == 7 and tab[7][0] == 4
    pos4, pos7 = list(tab[0]).index(4), list(tab[0]).index(7)
    assert pos7 == pos4 + 1


def _route3_brute(logits, k, D, pos, n_d, t2):
    """Mode 3 for one batch without the table: kept devices by the walk, replacements by a direct
    arg-max of the similarity over the experts that are allowed and free."""
    T, E = logits.shape
    G = E // D
    dev = [int(pos[e]) // G for e in range(E)]
    out = []
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-float(logits[t, e]), e))[:k]
        kept = []
        for e in order:
            if dev[e] not in kept and len(kept) < n_d:
                kept.append(dev[e])
        taken = {e for e in order if dev[e] in kept}
        final = []
        for e in order:
            if dev[e] in kept:
                final.append(e)
                continue
            cands = [c for c in range(E) if c != e and dev[c] in kept and c not in taken]
            best = min(cands, key=lambda c: (-t2[e, c], c))
            taken.add(best)
            final.append(best)
        out.append(final)
    return np.array(out, dtype=np.int32)


@pytest.mark.parametrize("E,D,k,n_d,seed", [(8, 4, 3, 2, 0), (12, 3, 4, 1, 1), (16, 4, 4, 2, 2), (6, 3, 2, 1, 3),
                                            (16, 8, 6, 3, 4)])
def test_similarity_pruning_against_direct_search(E, D, k, n_d, seed):
    rng = np.random.default_rng(seed)
    T = 150
    lg = rng.standard_normal((T, E)).astype(np.float32)
    prof = rng.standard_normal((500, E)) + rng.standard_normal((500, 1))   # profiling scores, correlated columns
    g = routing.gram(prof)
    tab = routing.similarity_table(g)
    pos = wl.random_placement(E, D, seed=seed + 10)
    ids, w = routing.route(lg, k, D, pos, n_d=n_d, prune_mode=3, renorm=1, sim_table=tab)
    assert np.array_equal(ids, _route3_brute(lg, k, D, pos, n_d, routing.similarity(g)))
    G = E // D
    ids0, _ = routing.route(lg, k, D, pos)
    ids2, _ = routing.route(lg, k, D, pos, n_d=n_d, prune_mode=2)
    p = routing.softmax64(lg)
    for t in range(T):
        assert len(set(ids[t].tolist())) == k                                   # k distinct experts
        devs = set((pos[ids[t]] // G).tolist())
        assert len(devs) <= n_d                                                 # at most n_d devices
        kept_devs = set((pos[ids2[t]] // G).tolist())                           # same walk as mode 2
        assert devs <= kept_devs
        for s in range(k):                                                      # survivors keep their slot
            if (pos[ids0[t, s]] // G) in kept_devs:
                assert ids[t, s] == ids0[t, s]
        if len(set((pos[ids0[t]] // G).tolist())) <= n_d:                       # nothing to prune: unchanged
            assert np.array_equal(ids[t], ids0[t])
        assert abs(w[t].sum() - 1.0) < 1e-12
        assert np.allclose(w[t], p[t, ids[t]] / p[t, ids[t]].sum(), rtol=1e-12)  # gates = own softmax values
    # a range that cannot prune anything leaves routing as it was
    ids_all, w_all = routing.route(lg, k, D, pos, n_d=min(k, D), prune_mode=3, sim_table=tab)
    ids_ref, w_ref = routing.route(lg, k, D, pos)
    assert np.array_equal(ids_all, ids_ref) and np.allclose(w_all, w_ref)
