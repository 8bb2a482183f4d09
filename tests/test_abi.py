"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, validates
arguments before touching a GPU, lays the plan block out as documented, and its host-side
placement equals the oracle's Algorithm 1.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from inputs import workloads as wl
from oracle import collaboration, routing
from paper_2505_13345_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return B.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "occult.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(occult_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert lib.occult_version() == 100


def test_cfg_validation_reports_errors_without_a_gpu(lib):
    good = dict(T=64, d=128, f=256, E=16, S=0, k=4, D=4, dtype="f32")
    pb, wb = B.occult_plan_sizes(B.make_cfg(**good))
    assert pb > 0 and wb > 0 and pb % 256 == 0
    cases = [
        (dict(good, D=5), -2),            # E % D
        (dict(good, k=17), -1),           # k > E
        (dict(good, E=512, D=4), -1),     # E above the limit
        (dict(good, n_d=1, k=8), -2),     # pruned range cannot hold k
        (dict(good, n_d=2, prune_mode=4), -1),
        (dict(good, T=-1), -1),
        (dict(good, renorm=2), -1),
    ]
    for kw, code in cases:
        with pytest.raises(B.OccultError) as ei:
            B.occult_plan_sizes(B.make_cfg(**kw))
        assert ei.value.code == code
        assert len(B.occult_last_error()) > 0
    # NULL pointers are refused before any launch
    cfg = B.make_cfg(**good)
    rc = lib.occult_route(ctypes.byref(cfg), None, None, None, None)
    assert rc == -4
    rc = lib.occult_dispatch(ctypes.byref(cfg), None, None, None, None)
    assert rc == -4
    # the host similarity-table builder: exact against the oracle, bad input refused
    import numpy as np
    from oracle import routing
    h = np.random.default_rng(0).standard_normal((50, 7))
    g = routing.gram(h)
    assert np.array_equal(B.occult_similarity_table(g), routing.similarity_table(g))
    g[3, 3] = 0.0
    with pytest.raises(B.OccultError):
        B.occult_similarity_table(g)


def test_plan_bind_layout_is_aligned_and_disjoint(lib):
    cfg = B.make_cfg(T=1000, d=64, f=64, E=60, S=0, k=4, D=4, dtype="bf16")
    pb, _ = B.occult_plan_sizes(cfg)
    base = 0x10000000
    plan = B.occult_plan_t()
    rc = lib.occult_plan_bind(ctypes.byref(cfg), base, pb, ctypes.byref(plan))
    assert rc == 0
    T, D, E, k = 1000, 4, 60, 4
    sizes = dict(tok_devmask=T * 8, dev_count=D * 4, dev_offset=(D + 1) * 4, tok_sfd_row=T * D * 4,
                 sfd_token=T * 4 * 4, exp_count=E * 4, exp_offset=(E + 1) * 4, pos_expert=E * 4,
                 epd_sfd_row=T * k * 4, epd_gate=T * k * 4, sfd_epd_rows=T * 4 * 4 * 4, counters=64)
    spans = []
    for name, sz in sizes.items():
        p = getattr(plan, name)
        assert p % 256 == 0 and base <= p and p + sz <= base + pb
        spans.append((p, p + sz))
    spans.sort()
    for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
        assert a1 <= b0
    assert lib.occult_plan_bind(ctypes.byref(cfg), base + 8, pb, ctypes.byref(plan)) == -3
    assert lib.occult_plan_bind(ctypes.byref(cfg), base, pb - 1, ctypes.byref(plan)) == -5


@pytest.mark.parametrize("E,D,k,seed", [(16, 4, 4, 0), (64, 16, 6, 1), (60, 4, 4, 2), (12, 6, 2, 3)])
def test_host_placement_equals_oracle_algorithm(E, D, k, seed):
    ids, _ = routing.route(wl.random_logits(3000, E, seed=seed, scale=2.0), k, D)
    C = collaboration.coactivation(ids, E)
    L_ref, pos_ref = collaboration.greedy_placement(C, D)
    L, pos = B.occult_placement_greedy(C.astype(np.int32), D)
    assert L.tolist() == L_ref
    assert pos.tolist() == pos_ref.tolist()
    # ties everywhere: constant matrix
    L, pos = B.occult_placement_greedy(np.ones((E, E), dtype=np.int32), D)
    L_ref, pos_ref = collaboration.greedy_placement(np.ones((E, E), dtype=np.int64), D)
    assert L.tolist() == L_ref and pos.tolist() == pos_ref.tolist()


def test_host_placement_rejects_bad_shapes():
    with pytest.raises(B.OccultError):
        B.occult_placement_greedy(np.zeros((8, 8), dtype=np.int32), 8)     # one expert per device
    with pytest.raises(B.OccultError):
        B.occult_placement_greedy(np.zeros((8, 8), dtype=np.int32), 3)


def test_backward_and_packing_entry_points_validate_on_the_host(lib):
    """Argument errors of the newer entry points are reported before any HIP call."""
    good = dict(T=64, d=128, f=256, E=16, S=0, k=4, D=4, dtype="bf16")
    cfg = B.make_cfg(**good)
    # sizes: host, pure
    assert B.occult_pack_weights_bytes(cfg) == 16 * 3 * 128 * 256 * 2
    assert B.occult_pack_weights_bytes(B.make_cfg(**dict(good, dtype="f32"))) == 0
    assert B.occult_expert_ffn_ws_bytes(cfg) == 0            # no shared experts: no scratch
    # NULL arguments
    assert lib.occult_combine_backward(ctypes.byref(cfg), None, None, None, None, None, None, None, None) == -4
    assert lib.occult_dispatch_backward(ctypes.byref(cfg), None, None, None, None, None, None) == -4
    assert lib.occult_route_backward(ctypes.byref(cfg), None, None, None, None, None) == -4
    assert lib.occult_transpose_weights(ctypes.byref(cfg), None, None, None, None) == -4
    assert lib.occult_pack_weights(ctypes.byref(cfg), None, None, 0, None) == -4
    args11 = [None] * 11
    assert lib.occult_expert_ffn_backward(ctypes.byref(cfg), None, None, None, None, *([None] * 10), 0, None) == -4
    assert lib.occult_expert_ffn_backward_weights(ctypes.byref(cfg), None, *args11, 0, None) == -4
    assert lib.occult_expert_ffn_backward_weights(ctypes.byref(cfg), None, *args11, 2, None) in (-1, -4)
    # a bad configuration is refused by every one of them
    bad = B.make_cfg(**dict(good, D=5))
    for call in (lambda: lib.occult_combine_backward(ctypes.byref(bad), None, None, None, None, None, None, None, None),
                 lambda: lib.occult_transpose_weights(ctypes.byref(bad), None, None, None, None),
                 lambda: lib.occult_pack_weights(ctypes.byref(bad), None, None, 0, None)):
        assert call() == -2
    # the bf16 expert kernels need d and f in multiples of 64
    odd = B.make_cfg(**dict(good, d=72))
    w = B.occult_weights_t(1 << 20, 1 << 20, 1 << 20)     # never dereferenced: the shape check comes first
    assert lib.occult_pack_weights(ctypes.byref(odd), ctypes.byref(w), 1 << 20, 1 << 30, None) == -2


@pytest.mark.parametrize("E,seed", [(2, 0), (5, 1), (16, 2), (60, 3), (128, 4), (256, 5)])
def test_host_similarity_table_equals_oracle(E, seed):
    """The host table builder on random Gram matrices, with tied similarities (a zero-norm column is refused:
    checked with the configuration errors above)."""
    rng = np.random.default_rng(seed)
    prof = rng.standard_normal((400, E))
    if E >= 5:
        prof[:, 3] = prof[:, 1]          # identical columns: equal similarities to everyone else -> index order
    g = routing.gram(prof.astype(np.float32))
    tab = B.occult_similarity_table(g)
    assert tab.shape == (E, E - 1)
    assert np.array_equal(tab, routing.similarity_table(g))
    for i in range(E):                   # every row lists every other expert exactly once
        assert sorted(tab[i].tolist()) == [j for j in range(E) if j != i]
    # placement with more random shapes, including zero co-activation
    if E % 4 == 0 and E >= 8:
        C = rng.integers(0, 50, (E, E))
        C = (C + C.T).astype(np.int32)
        L, pos = B.occult_placement_greedy(C, 4)
        L_ref, pos_ref = collaboration.greedy_placement(C.astype(np.int64), 4)
        assert L.tolist() == L_ref and pos.tolist() == pos_ref.tolist()
        L, pos = B.occult_placement_greedy(np.zeros((E, E), dtype=np.int32), 4)
        L_ref, pos_ref = collaboration.greedy_placement(np.zeros((E, E), dtype=np.int64), 4)
        assert L.tolist() == L_ref and pos.tolist() == pos_ref.tolist()


@pytest.mark.parametrize("E,D,seed", [(4, 2, 0), (16, 4, 1), (64, 16, 2), (60, 4, 3), (8, 8, 4), (6, 1, 5)])
def test_host_collaboration_stats_equal_the_oracle(E, D, seed):
    """occult_collaboration_stats (Sec. 3.2 averages) against the pinned oracle, contiguous and permuted."""
    rng = np.random.default_rng(seed)
    A = rng.integers(0, 200, (E, E))
    C = (A + A.T).astype(np.int32)
    for pos in (None, wl.random_placement(E, D, seed=seed)):
        ci, cx, frac = B.occult_collaboration_stats(C, D, pos)
        want = collaboration.collaboration_stats(C.astype(np.int64), np.arange(E) if pos is None else pos, D)
        assert np.allclose(ci, want["c_intra"], rtol=1e-12, atol=0)
        assert np.allclose(cx, want["c_inter"], rtol=1e-12, atol=0)
        assert np.isclose(frac, want["intra_fraction"], rtol=1e-12, atol=0)
    ci, cx, frac = B.occult_collaboration_stats(np.zeros((E, E), dtype=np.int32), D)
    assert not ci.any() and not cx.any() and frac == 0.0
    with pytest.raises(B.OccultError):
        B.occult_collaboration_stats(C, D + 1 if E % (D + 1) else E + 1)


def test_plan_static_refuses_layers_beyond_its_built_in_scratch(lib):
    """The size check of occult_plan_static comes before any HIP call: a layer needing more than
    OCCULT_PLAN_STATIC_MAX_BYTES of planner scratch gets OCCULT_EWORKSPACE and a message naming the limit."""
    big = B.make_cfg(T=20_000_000, d=64, f=64, E=256, S=0, k=1, D=64, dtype="bf16")
    _, ws = B.occult_plan_sizes(big)
    assert ws > 4 << 20
    assert lib.occult_plan_static(ctypes.byref(big), None, None, None, None) == -5
    assert "4194304" in B.occult_last_error()
    ok = B.make_cfg(T=4096, d=64, f=64, E=64, S=0, k=8, D=8, dtype="bf16")
    assert lib.occult_plan_static(ctypes.byref(ok), None, None, None, None) == -4     # NULL plan, still on the host
