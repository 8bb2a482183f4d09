"""GPU parity, integer side: occult_route, occult_plan, occult_coactivation, plan statistics.
Every index, offset, count and table must equal the oracle's bit for bit; gate values within
1e-5 relative."""
import numpy as np
import pytest
import torch

from inputs import workloads as wl
from oracle import collaboration, occult_ref, routing
from paper_2505_13345_amd import binding as B
from paper_2505_13345_amd.layer import OccultLayer
from tests.helpers import check_plan_against_trace, expand_plan, require_gpu, say

pytestmark = pytest.mark.gpu


def _route_gpu(lg, k, D, E, pos, n_d, mode, renorm):
    dev = require_gpu()
    T = lg.shape[0]
    layer = OccultLayer(T, 64, 64, E, 0, k, D, "bf16", n_d, mode, renorm, pos, with_ffn=False)
    layer.route(torch.from_numpy(lg).to(dev))
    torch.cuda.synchronize()
    return layer, layer.ids.cpu().numpy(), layer.w.cpu().numpy()


ROUTE_CASES = [
    # E, D, k, T, n_d, mode, renorm, ties, placement
    (16, 4, 4, 256, 0, 1, 1, False, "contig"),
    (16, 4, 4, 1000, 2, 1, 1, True, "random"),
    (16, 4, 4, 1000, 2, 2, 0, True, "random"),
    (60, 4, 4, 128, 0, 1, 1, False, "contig"),
    (60, 4, 4, 777, 1, 1, 1, False, "random"),
    (64, 8, 8, 4099, 2, 1, 1, False, "contig"),
    (64, 8, 8, 4099, 2, 2, 1, True, "random"),
    (64, 8, 8, 513, 8, 1, 1, False, "contig"),
    (64, 16, 6, 2050, 3, 1, 0, True, "random"),
    (128, 8, 8, 1500, 2, 1, 1, True, "random"),
    (256, 64, 32, 900, 8, 2, 1, True, "random"),
    (256, 16, 8, 900, 4, 1, 1, False, "contig"),
    (8, 8, 2, 65, 0, 1, 1, True, "contig"),
    (4, 1, 4, 10, 1, 1, 1, False, "contig"),
]


@pytest.mark.parametrize("E,D,k,T,n_d,mode,renorm,ties,placement", ROUTE_CASES)
def test_route_matches_oracle(E, D, k, T, n_d, mode, renorm, ties, placement):
    say(f"route case E={E} D={D} k={k} T={T} n_d={n_d} mode={mode} ties={ties} {placement}")
    lg = wl.random_logits(T, E, seed=E * 7 + k + n_d, scale=1.3, ties=ties)
    pos = None if placement == "contig" else wl.random_placement(E, D, seed=E + D)
    ids_ref, w_ref = routing.route(lg, k, D, pos, n_d=n_d, prune_mode=mode, renorm=renorm)
    _, ids, w = _route_gpu(lg, k, D, E, pos, n_d, mode, renorm)
    assert np.array_equal(ids, ids_ref)
    rel = np.abs(w.astype(np.float64) - w_ref) / w_ref
    assert rel.max() <= 1e-5, rel.max()


@pytest.mark.parametrize("name", ["tiny_f32", "decode_bf16", "prefill_bf16", "prefill_pruned_bf16",
                                  "large_bf16"])
def test_route_and_plan_at_config_sizes(name):
    shape = wl.CONFIGS[name]
    say(f"config {name}: generating")
    wk = wl.make_workload(shape, with_experts=False)
    dev = require_gpu()
    ids_ref, w_ref = routing.route(wk.logits, shape.k, shape.D, None, shape.n_d, shape.prune_mode,
                                   shape.renorm)
    layer = OccultLayer(shape.T, shape.d, shape.f, shape.E, shape.S, shape.k, shape.D, shape.dtype,
                        shape.n_d, shape.prune_mode, shape.renorm, None, with_ffn=False)
    say(f"config {name}: route + plan on GPU")
    layer.route(torch.from_numpy(wk.logits).to(dev))
    layer.make_plan()
    torch.cuda.synchronize()
    ids, w = layer.ids.cpu().numpy(), layer.w.cpu().numpy()
    assert np.array_equal(ids, ids_ref)
    assert (np.abs(w - w_ref) / w_ref).max() <= 1e-5
    # the plan is built from the GPU's own float32 gates; feed the oracle the same values
    trace = occult_ref.moe_forward(np.zeros((shape.T, 1)), ids, w.astype(np.float64),
                                   wl.contiguous_placement(shape.E, shape.D), shape.D)
    exp = expand_plan(layer.tables(), shape.T, shape.E, shape.D, shape.k)
    check_plan_against_trace(exp, trace, ids, w, None, shape.T, shape.E, shape.D, shape.k)
    st = layer.stats()
    row = shape.d * (2 if shape.dtype == "bf16" else 4)
    ref_bytes = occult_ref.exchange_bytes(shape.T, shape.k, trace.n_sfd, row)
    assert st.n_sfd == trace.n_sfd and st.n_epd == shape.T * shape.k
    assert st.bytes_occ == ref_bytes["bytes_occ"] and st.bytes_std == ref_bytes["bytes_std"]
    assert st.bytes_meta == ref_bytes["bytes_meta"]
    assert abs(st.c_t - trace.c_t) < 1e-12
    if shape.n_d:
        assert st.c_t <= shape.n_d
    say(f"config {name}: C_T={st.c_t:.4f} bytes/token occ={st.bytes_occ / shape.T:.0f} "
        f"std={st.bytes_std / shape.T:.0f}")


PLAN_CASES = [
    # E, D, k, T, placement
    (4, 2, 2, 4, "contig"),
    (12, 3, 4, 97, "random"),
    (16, 4, 4, 255, "random"),
    (16, 4, 4, 256, "contig"),
    (16, 4, 4, 257, "random"),
    (60, 4, 4, 1031, "random"),
    (64, 64, 8, 700, "contig"),       # one expert per device: standard dispatch, C_T = k
    (64, 1, 8, 700, "contig"),        # one device: every token once
    (256, 64, 32, 600, "random"),
    (256, 4, 3, 1300, "random"),
    (8, 2, 8, 300, "contig"),         # k = E: every token on every device
    # one block of tokens (T <= 256): the single-launch planner built on per-column token sets
    (8, 2, 2, 1, "contig"),
    (60, 4, 4, 63, "random"),
    (60, 4, 4, 64, "contig"),
    (60, 4, 4, 65, "random"),
    (64, 8, 8, 129, "random"),
    (64, 64, 8, 200, "contig"),       # one expert per device
    (64, 1, 8, 256, "contig"),        # one device
    (256, 64, 32, 256, "random"),     # the largest layer the planner takes, full block
    (256, 4, 3, 191, "random"),
    (8, 2, 8, 100, "contig"),         # k = E
    (32, 4, 16, 77, "random"),
]


@pytest.mark.parametrize("E,D,k,T,placement", PLAN_CASES)
def test_plan_matches_oracle_brims(E, D, k, T, placement):
    say(f"plan case E={E} D={D} k={k} T={T} {placement}")
    dev = require_gpu()
    lg = wl.random_logits(T, E, seed=T + E, ties=True)
    pos = None if placement == "contig" else wl.random_placement(E, D, seed=T)
    ids, w = routing.route(lg, k, D, pos)
    w32 = w.astype(np.float32)
    layer = OccultLayer(T, 64, 64, E, 0, k, D, "bf16", expert_pos=pos, with_ffn=False)
    layer.make_plan(torch.from_numpy(ids).to(dev), torch.from_numpy(w32).to(dev))
    torch.cuda.synchronize()
    pos_arr = wl.contiguous_placement(E, D) if pos is None else pos
    trace = occult_ref.moe_forward(np.zeros((T, 1)), ids, w32.astype(np.float64), pos_arr, D)
    exp = expand_plan(layer.tables(), T, E, D, k)
    check_plan_against_trace(exp, trace, ids, w32, pos, T, E, D, k)
    if D == E:
        assert exp["n_sfd"] == T * k
    if D == 1:
        assert exp["n_sfd"] == T


def test_plan_fig2_instance(golden_dir):
    dev = require_gpu()
    ids = np.array([[0, 1], [2, 3], [0, 2], [1, 3]], dtype=np.int32)
    w = np.full((4, 2), 0.5, dtype=np.float32)
    layer = OccultLayer(4, 64, 64, 4, 0, 2, 2, "bf16", with_ffn=False)
    layer.make_plan(torch.from_numpy(ids).to(dev), torch.from_numpy(w).to(dev))
    torch.cuda.synchronize()
    exp = expand_plan(layer.tables(), 4, 4, 2, 2)
    assert exp["brim_0"].tolist() == [[0, -1, 1, 2], [-1, 3, 4, 5]]
    assert exp["brim_1"][0].tolist() == [[0, 1, -1], [2, -1, 3]]
    assert exp["brim_1"][1].tolist() == [[0, 1, -1], [2, -1, 3]]
    assert exp["sfd_token"][:6].tolist() == [0, 2, 3, 1, 2, 3]
    assert layer.stats().c_t == 1.5


def test_empty_batch_is_a_no_op():
    dev = require_gpu()
    layer = OccultLayer(0, 64, 64, 16, 0, 4, 4, "bf16", with_ffn=False)
    layer.route(torch.zeros((0, 16), device=dev))
    layer.make_plan()
    torch.cuda.synchronize()
    tabs = layer.tables()
    assert tabs["dev_offset"].cpu().tolist() == [0] * 5
    assert tabs["exp_offset"].cpu().tolist() == [0] * 17
    st = layer.stats()
    assert st.n_sfd == 0 and st.c_t == 0.0


@pytest.mark.parametrize("E,k,T", [(16, 4, 256), (64, 8, 16384), (64, 6, 65536), (128, 8, 3000),
                                    (256, 8, 3000), (60, 4, 128)])
def test_coactivation_counts(E, k, T):
    say(f"coactivation E={E} k={k} T={T}")
    dev = require_gpu()
    ids, _ = routing.route(wl.random_logits(T, E, seed=E + k, scale=2.0), k, 1)
    C_ref = collaboration.coactivation(ids, E)
    cfg = B.make_cfg(T, 64, 64, E, 0, k, 1, "bf16")
    C = torch.full((E, E), 7, dtype=torch.int32, device=dev)
    ids_d = torch.from_numpy(ids).to(dev)
    B.occult_coactivation(cfg, ids_d, C, False)
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy(), C_ref)
    B.occult_coactivation(cfg, ids_d, C, True)       # accumulate over a second batch
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy(), 2 * C_ref)


# ---- expert-similarity-based pruning (prune_mode 3) -------------------------------------------

SIM_CASES = [
    # E, D, k, T, n_d, renorm, placement
    (16, 4, 4, 1000, 2, 1, "random"),
    (60, 4, 4, 777, 1, 1, "contig"),
    (64, 8, 8, 4099, 2, 1, "contig"),
    (64, 8, 8, 2000, 3, 0, "random"),
    (128, 8, 8, 1500, 2, 1, "random"),
    (256, 16, 8, 900, 4, 1, "random"),
    (8, 4, 2, 65, 1, 1, "contig"),
]


@pytest.mark.parametrize("E,D,k,T,n_d,renorm,placement", SIM_CASES)
def test_similarity_pruning_matches_oracle(E, D, k, T, n_d, renorm, placement):
    say(f"similarity pruning case E={E} D={D} k={k} T={T} n_d={n_d} {placement}")
    dev = require_gpu()
    prof = wl.random_logits(3000, E, seed=E + 1, scale=1.0)
    prof = (prof + np.random.default_rng(E).standard_normal((3000, 1)).astype(np.float32)).astype(np.float32)
    # Gram matrix on the GPU in two accumulated batches against the oracle's
    cfg = B.make_cfg(2000, 64, 64, E, 0, k, D, "bf16")
    gram = torch.full((E, E), 123.0, dtype=torch.float64, device=dev)
    prof_d = torch.from_numpy(prof).to(dev)
    B.occult_similarity_gram(cfg, prof_d[:2000].contiguous(), gram, accumulate=False)
    cfg2 = B.make_cfg(1000, 64, 64, E, 0, k, D, "bf16")
    B.occult_similarity_gram(cfg2, prof_d[2000:].contiguous(), gram, accumulate=True)
    torch.cuda.synchronize()
    g_gpu = gram.cpu().numpy()
    g_ref = routing.gram(prof)
    assert np.max(np.abs(g_gpu - g_ref)) <= 1e-11 * np.max(np.abs(g_ref))
    # the host table builder is exact: same table as the oracle from the same Gram matrix
    tab = B.occult_similarity_table(g_gpu)
    assert np.array_equal(tab, routing.similarity_table(g_gpu))
    # and from the oracle's Gram matrix the table may differ only where similarities are as good as equal
    tab_ref = routing.similarity_table(g_ref)
    if not np.array_equal(tab, tab_ref):
        t2 = routing.similarity(g_ref)
        i, q = np.argwhere(tab != tab_ref)[0]
        assert abs(t2[i, tab[i, q]] - t2[i, tab_ref[i, q]]) <= 1e-10
    # routing with that table
    lg = wl.random_logits(T, E, seed=E * 5 + k, scale=1.3)
    pos = None if placement == "contig" else wl.random_placement(E, D, seed=E + D)
    ids_ref, w_ref = routing.route(lg, k, D, pos, n_d=n_d, prune_mode=3, renorm=renorm, sim_table=tab)
    layer = OccultLayer(T, 64, 64, E, 0, k, D, "bf16", n_d, 3, renorm, pos, with_ffn=False, sim_table=tab)
    layer.route(torch.from_numpy(lg).to(dev))
    torch.cuda.synchronize()
    ids, w = layer.ids.cpu().numpy(), layer.w.cpu().numpy()
    assert np.array_equal(ids, ids_ref)
    assert np.max(np.abs(w.astype(np.float64) - w_ref) / w_ref) <= 1e-5
    # and the plan built on it keeps every token within n_d devices
    layer.make_plan()
    torch.cuda.synchronize()
    mask = layer.tables()["tok_devmask"].cpu().numpy().astype(np.uint64)
    assert max(bin(int(m)).count("1") for m in mask) <= n_d


@pytest.mark.parametrize("E,D,k,n_d,mode", [(16, 4, 4, 0, 1), (64, 8, 8, 2, 1), (60, 4, 4, 2, 2), (256, 16, 8, 4, 1)])
def test_route_non_finite_scores_give_in_range_distinct_ids(E, D, k, n_d, mode):
    """Scores are documented as finite; NaN / -inf / +inf entries are read as the extreme finite values, so
    the routing of such a token is still k distinct experts below E (within n_d devices under pruning),
    the plan built from it is consistent, and the finite tokens of the batch are untouched."""
    say(f"non-finite scores E={E} D={D} k={k} n_d={n_d} mode={mode}")
    T = 300
    lg = wl.random_logits(T, E, seed=E + k, scale=1.3)
    rng = np.random.default_rng(E)
    bad = rng.choice(T, size=60, replace=False)
    for i, t in enumerate(bad):
        cols = rng.choice(E, size=[1, E // 2, E - 1, E][i % 4], replace=False)
        lg[t, cols] = [np.nan, -np.inf, np.inf][i % 3]
        if i % 5 == 0:
            lg[t, [15 % E, 31 % E, 47 % E]] = np.nan
    layer, ids, w = _route_gpu(lg, k, D, E, None, n_d, mode, 1)
    good = np.setdiff1d(np.arange(T), bad)
    ids_ref, _ = routing.route(lg[good], k, D, None, n_d=n_d, prune_mode=mode, renorm=1)
    assert np.array_equal(ids[good], ids_ref)
    assert ids.min() >= 0 and ids.max() < E
    assert all(len(set(row)) == k for row in ids.tolist())
    assert np.isfinite(w).all()
    if n_d:
        assert (np.array([len(set(e // (E // D) for e in row)) for row in ids.tolist()]) <= n_d).all()
    layer.make_plan()
    torch.cuda.synchronize()
    trace = occult_ref.moe_forward(np.zeros((T, 1)), ids, w.astype(np.float64), np.arange(E), D)
    check_plan_against_trace(expand_plan(layer.tables(), T, E, D, k), trace, ids, w, None, T, E, D, k)
