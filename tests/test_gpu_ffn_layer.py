"""GPU parity for occult_expert_ffn and the whole hot path (route -> plan -> dispatch -> expert
FFN -> combine) against the textbook layer O-std in float64.

Bars: f32 outputs within max-rel 1e-5 (relative to
max(|o|, rms(o)) so that entries near zero do not dominate), bf16 outputs within max-abs 2e-2
and mean-abs 2e-3 of the oracle's exactly accumulated result.
"""
import numpy as np
import pytest
import torch

from inputs import workloads as wl
from oracle import moe_std, occult_ref, routing
from paper_2505_13345_amd.layer import OccultLayer
from tests.helpers import (assert_one_rounding, bf16_errors, cached_workload, chain_mean_bar, f32_rel_error, require_gpu, say,
                           to_dev)

pytestmark = pytest.mark.gpu


def _run_layer(shape, wk, pos=None):
    dev = require_gpu()
    layer = OccultLayer(shape.T, shape.d, shape.f, shape.E, shape.S, shape.k, shape.D, shape.dtype,
                        shape.n_d, shape.prune_mode, shape.renorm, pos)
    x = to_dev(wk.x, shape.dtype, dev)
    wg, wu, wd = (to_dev(a, shape.dtype, dev) for a in (wk.w_gate, wk.w_up, wk.w_down))
    y = layer.forward(torch.from_numpy(wk.logits).to(dev), x, wg, wu, wd)
    torch.cuda.synchronize()
    return layer, y.float().cpu().numpy()


SMALL = [
    # name, T, d, f, E, S, k, D, dtype   (several tiles and ragged tails in M, N and groups)
    ("f32_a", 300, 96, 80, 8, 0, 2, 4, "f32"),
    ("f32_shared", 130, 128, 256, 16, 2, 4, 4, "f32"),
    ("bf16_a", 700, 256, 192, 8, 0, 2, 4, "bf16"),
    ("bf16_shared", 333, 512, 320, 12, 2, 3, 3, "bf16"),
    ("bf16_one_row_experts", 9, 128, 64, 16, 1, 2, 8, "bf16"),
    ("bf16_big_expert", 1500, 192, 448, 4, 0, 1, 2, "bf16"),
    # ~20 rows per expert (weight-streaming kernel, some experts over 32 rows = two row tiles, some
    # empty), shared experts as uniform groups of the small-tile kernel
    ("bf16_few_rows_ragged", 80, 256, 192, 16, 2, 4, 4, "bf16"),
    # 256-row tiles with three K tiles, shared experts as uniform groups of the same kernel
    ("bf16_big_shared", 1100, 192, 128, 4, 3, 1, 4, "bf16"),
    # hidden rows of 14 KiB (two column chunks in combine), long K in the first product
    ("bf16_wide_rows", 200, 7168, 128, 32, 1, 4, 8, "bf16"),
    # outputs narrower than a wave tile of the 256-row kernel (d = 64 forward, f = 64 backward): the store
    # range must end inside the group's last row
    ("bf16_narrow_d", 900, 64, 128, 8, 0, 3, 2, "bf16"),
    ("bf16_narrow_f", 1100, 192, 64, 8, 0, 3, 1, "bf16"),
]


@pytest.mark.parametrize("name,T,d,f,E,S,k,D,dtype", SMALL)
def test_small_layers_elementwise(name, T, d, f, E, S, k, D, dtype):
    say(f"small layer {name}")
    shape = wl.LayerShape(name, T=T, d=d, f=f, E=E, S=S, k=k, D=D, dtype=dtype,
                          components=4 if dtype == "bf16" else 0)
    wk = wl.make_workload(shape, seed=17)
    pos = wl.random_placement(E, D, seed=2)
    layer, y = _run_layer(shape, wk, pos)
    ids, w = layer.ids.cpu().numpy(), layer.w.cpu().numpy().astype(np.float64)
    ids_ref, _ = routing.route(wk.logits, k, D, pos)
    assert np.array_equal(ids, ids_ref)
    y_ref = moe_std.moe_layer(wk.x, ids, w, wk.w_gate, wk.w_up, wk.w_down, E, S)
    # the deduplicated oracle reaches the same numbers (exactness), and gives the intermediates
    tr = occult_ref.moe_forward(wk.x, ids, w, pos, D, wk.w_gate, wk.w_up, wk.w_down, S)
    assert np.allclose(tr.y, y_ref, rtol=1e-9, atol=1e-11)
    n_sfd = tr.n_sfd
    sfd_y = layer.sfd_y[:n_sfd].float().cpu().numpy()
    if dtype == "f32":
        assert f32_rel_error(y, y_ref) <= 1e-5
        assert f32_rel_error(sfd_y, tr.y_sfd) <= 1e-5
    else:
        mx, mean = bf16_errors(y, y_ref)
        say(f"  y max-abs {mx:.3e} mean-abs {mean:.3e}")
        assert mx <= 2e-2 and mean <= 2e-3
        mx, mean = bf16_errors(sfd_y, tr.y_sfd)
        assert mx <= 2e-2 and mean <= 2e-3


def test_tiny_f32_config_full_layer():
    shape = wl.CONFIGS["tiny_f32"]
    wk = wl.make_workload(shape)
    layer, y = _run_layer(shape, wk)
    ids, w = layer.ids.cpu().numpy(), layer.w.cpu().numpy().astype(np.float64)
    ids_ref, w_ref = routing.route(wk.logits, shape.k, shape.D)
    assert np.array_equal(ids, ids_ref)
    y_ref = moe_std.moe_layer(wk.x, ids_ref, w_ref, wk.w_gate, wk.w_up, wk.w_down, shape.E, 0)
    err = f32_rel_error(y, y_ref)
    say(f"tiny_f32 normalised max-rel {err:.3e}; plain max-rel "
        f"{np.max(np.abs(y - y_ref) / np.maximum(np.abs(y_ref), 1e-30)):.3e}")
    assert err <= 1e-5


def test_decode_config_full_layer():
    shape = wl.CONFIGS["decode_bf16"]
    say("decode_bf16: generating")
    wk = wl.make_workload(shape)
    layer, y = _run_layer(shape, wk)
    ids, w = layer.ids.cpu().numpy(), layer.w.cpu().numpy().astype(np.float64)
    y_ref = moe_std.moe_layer(wk.x, ids, w, wk.w_gate, wk.w_up, wk.w_down, shape.E, shape.S)
    mx, mean = bf16_errors(y, y_ref)
    say(f"decode_bf16: y max-abs {mx:.3e} mean-abs {mean:.3e} |y|max {np.abs(y_ref).max():.2f}")
    assert mx <= 2e-2 and mean <= 2e-3


_refs = {}


def _std_reference(shape, wk, ids, w):
    """The textbook layer on every token, cached per routing (placement does not change it)."""
    key = (shape.T, shape.E, shape.S, shape.k, ids.tobytes()[:4096], float(w.sum()))
    if key not in _refs:
        say(f"{shape.name}: textbook oracle on all {shape.T} tokens")
        _refs.clear()
        _refs[key] = moe_std.moe_layer(wk.x, ids, w, wk.w_gate, wk.w_up, wk.w_down, shape.E, shape.S)
    return _refs[key]


def _check_expert_rows(layer, shape, wk):
    """Both products of every expert against float64 products of their stored operands, every EPD row:
    epd_h = one bf16 rounding of silu(X W_gate^T) * (X W_up^T) with X the gathered rows of sfd_x, and
    epd_y = one bf16 rounding of (stored epd_h) W_down^T."""
    tabs = layer.tables()
    exp_off = tabs["exp_offset"].cpu().numpy()
    pos_expert = tabs["pos_expert"].cpu().numpy()
    src = tabs["epd_sfd_row"].long()
    for P in range(shape.E):
        q0, q1 = int(exp_off[P]), int(exp_off[P + 1])
        if q1 == q0:
            continue
        e = int(pos_expert[P])
        X = layer.sfd_x[src[q0:q1]].double().cpu().numpy()
        g = X @ wk.w_gate[e].astype(np.float64).T
        u = X @ wk.w_up[e].astype(np.float64).T
        assert_one_rounding(layer.epd_h[q0:q1].float().cpu().numpy(), g / (1.0 + np.exp(-g)) * u, f"epd_h, position {P}")
        H = layer.epd_h[q0:q1].double().cpu().numpy()
        assert_one_rounding(layer.epd_y[q0:q1].float().cpu().numpy(), H @ wk.w_down[e].astype(np.float64).T,
                            f"epd_y, position {P}")
    if shape.S:
        X = wk.x.astype(np.float64)
        for s_ in range(shape.S):
            e = shape.E + s_
            g = X @ wk.w_gate[e].astype(np.float64).T
            u = X @ wk.w_up[e].astype(np.float64).T
            assert_one_rounding(layer.h_shared[:, s_ * shape.f:(s_ + 1) * shape.f].float().cpu().numpy(),
                                g / (1.0 + np.exp(-g)) * u, f"h_shared, shared expert {s_}")


def _full_parity(name, pos=None, payload=True, expert_rows=True):
    """One configuration at full size: routing bit-exact; y of every token against the textbook oracle;
    the dispatched rows (bit-exact) and the return payload sfd_y of every SFD row against the
    deduplicated oracle; every EPD row of both products against float64 products of its stored operands."""
    shape = wl.CONFIGS[name]
    wk = cached_workload(shape)
    say(f"{name}: running on GPU")
    layer, y = _run_layer(shape, wk, pos)
    ids, w = layer.ids.cpu().numpy(), layer.w.cpu().numpy().astype(np.float64)
    ids_ref, _ = routing.route(wk.logits, shape.k, shape.D, pos, shape.n_d, shape.prune_mode, shape.renorm)
    assert np.array_equal(ids, ids_ref)
    y_ref = _std_reference(shape, wk, ids, w)
    mx, mean = bf16_errors(y, y_ref)
    rms = float(np.sqrt(np.mean(y_ref ** 2)))
    say(f"{name}: all {shape.T} rows of y: max-abs {mx:.3e} mean-abs {mean:.3e}; |y| rms {rms:.3f} max "
        f"{np.abs(y_ref).max():.2f}; mean-abs / rms {mean / rms:.2e}")
    assert mx <= 2e-2 and mean <= 2e-3
    # scale-free: y passed through four stored bf16 tensors (epd_h, epd_y, sfd_y, y)
    assert mean / rms <= chain_mean_bar(4)
    if payload:
        say(f"{name}: deduplicated oracle on all tokens")
        pos_arr = wl.contiguous_placement(shape.E, shape.D) if pos is None else pos
        tr = occult_ref.moe_forward(wk.x, ids, w, pos_arr, shape.D, wk.w_gate, wk.w_up, wk.w_down, shape.S)
        n_sfd = tr.n_sfd
        assert layer.stats().n_sfd == n_sfd
        assert np.array_equal(layer.sfd_x[:n_sfd].float().cpu().numpy(), tr.x_sfd)
        got = layer.sfd_y[:n_sfd].float().cpu().numpy()
        mx, mean = bf16_errors(got, tr.y_sfd)
        rms_s = float(np.sqrt(np.mean(tr.y_sfd ** 2)))
        say(f"{name}: all {n_sfd} rows of sfd_y: max-abs {mx:.3e} mean-abs {mean:.3e}; mean-abs / rms {mean / rms_s:.2e}")
        assert mx <= 2e-2 and mean <= 2e-3 and mean / rms_s <= chain_mean_bar(3)
        assert np.abs(tr.y - y_ref).max() <= 1e-9 * max(1.0, np.abs(y_ref).max())     # the two oracles agree
        del tr, got
    if expert_rows:
        say(f"{name}: both products of every expert on their stored operands")
        _check_expert_rows(layer, shape, wk)
    return wk, layer, y


def test_prefill_config_all_rows():
    _full_parity("prefill_bf16")


def test_prefill_pruned_config_all_rows_and_difference_from_unpruned():
    wk, layer, y = _full_parity("prefill_bf16", payload=False, expert_rows=False)
    st = layer.stats()
    del layer
    torch.cuda.empty_cache()
    # same tensors with collaboration pruning to 2 devices
    wk2, layer2, y2 = _full_parity("prefill_pruned_bf16")
    st2 = layer2.stats()
    assert st2.c_t <= 2.0 < st.c_t
    diff = np.abs(y2.astype(np.float64) - y)
    rel_fro = np.linalg.norm(y2.astype(np.float64) - y) / np.linalg.norm(y)
    say(f"pruned vs unpruned: C_T {st.c_t:.3f} -> {st2.c_t:.3f}; bytes/token {st.bytes_occ / 16384:.0f} -> "
        f"{st2.bytes_occ / 16384:.0f} (standard {st.bytes_std / 16384:.0f}); output diff max-abs "
        f"{diff.max():.3f} mean-abs {diff.mean():.4f} rel-Frobenius {rel_fro:.3f}")
    assert 0.0 < rel_fro < 1.0


_large = {}


def test_large_config_all_rows_of_y():
    wk, layer, y = _full_parity("large_bf16", payload=False, expert_rows=False)
    _large["y"], _large["c_t"], _large["bytes_occ"] = y, layer.stats().c_t, layer.stats().bytes_occ


def test_large_config_payload_and_expert_rows():
    _full_parity("large_bf16", payload=True, expert_rows=False)


def test_large_config_expert_rows():
    _full_parity("large_bf16", payload=False, expert_rows=True)


def test_large_config_greedy_placement_all_rows():
    from oracle import collaboration
    from paper_2505_13345_amd import binding as B
    shape = wl.CONFIGS["large_bf16"]
    dev = require_gpu()
    wk = cached_workload(shape)
    ids, _ = routing.route(wk.logits, shape.k, shape.D)
    cfg = B.make_cfg(shape.T, shape.d, shape.f, shape.E, shape.S, shape.k, shape.D, "bf16")
    C = torch.zeros((shape.E, shape.E), dtype=torch.int32, device=dev)
    B.occult_coactivation(cfg, torch.from_numpy(ids).to(dev), C, False)
    torch.cuda.synchronize()
    C_host = C.cpu().numpy()
    assert np.array_equal(C_host, collaboration.coactivation(ids, shape.E))
    L, pos = B.occult_placement_greedy(C_host, shape.D)
    L_ref, pos_ref = collaboration.greedy_placement(C_host, shape.D)
    assert pos.tolist() == pos_ref.tolist()
    # the same layer under the greedy placement: every row of y and of the payload against the oracles
    wk, layer2, y2 = _full_parity("large_bf16", pos=pos, payload=True, expert_rows=False)
    st2 = layer2.stats()
    contig = occult_ref.moe_forward(np.zeros((shape.T, 1)), ids, np.ones(ids.shape), wl.contiguous_placement(shape.E, shape.D),
                                    shape.D)
    say(f"large: C_T contiguous {contig.c_t:.3f} -> greedy {st2.c_t:.3f}; bytes/token "
        f"{2 * contig.n_sfd * shape.d * 2 / shape.T:.0f} -> {st2.bytes_occ / shape.T:.0f} (standard {st2.bytes_std / shape.T:.0f})")
    assert st2.c_t < contig.c_t
    if "y" in _large:
        # placement never changes the layer output beyond rounding (exactness): both runs are within the
        # bars of the same oracle rows, so they differ by at most twice the bar
        mx, mean = bf16_errors(y2, _large["y"])
        assert mx <= 4e-2 and mean <= 2e-3


def test_shared_down_projection_split_over_k_matches_unsplit():
    """occult_expert_ffn_ws (the shared experts' down projection as f32 partial products in scratch, summed in a
    fixed order and rounded once) against occult_expert_ffn on the decode layer with 160 tokens (above the batch
    sizes whose shared experts run inside the routed experts' launches): the same numbers up to one bf16 rounding of
    differently ordered f32 sums, and each within the bars of the oracle."""
    import dataclasses
    shape = dataclasses.replace(wl.CONFIGS["decode_bf16"], name="decode_160", T=160)
    say("decode shape, 160 tokens, split-K: generating")
    wk = wl.make_workload(shape)
    dev = require_gpu()
    layer = OccultLayer(shape.T, shape.d, shape.f, shape.E, shape.S, shape.k, shape.D, shape.dtype)
    assert layer.ffn_ws is not None            # this shape asks for scratch
    x = to_dev(wk.x, shape.dtype, dev)
    wg, wu, wd = (to_dev(a, shape.dtype, dev) for a in (wk.w_gate, wk.w_up, wk.w_down))
    layer.route(torch.from_numpy(wk.logits).to(dev)); layer.make_plan(); layer.dispatch(x)
    outs = []
    for use_ws in (False, True, True):          # twice with scratch: the buffer's old contents do not matter
        layer.y_shared.fill_(7.0)
        layer.expert_ffn(x, wg, wu, wd, use_ws=use_ws)
        torch.cuda.synchronize()
        outs.append(layer.y_shared.float().cpu().numpy().copy())
    assert np.array_equal(outs[1], outs[2])
    xs = wk.x.astype(np.float64)
    ref = np.zeros((shape.T, shape.d))
    for s_ in range(shape.S):
        e = shape.E + s_
        g = xs @ wk.w_gate[e].astype(np.float64).T
        u = xs @ wk.w_up[e].astype(np.float64).T
        ref += (g / (1.0 + np.exp(-g)) * u) @ wk.w_down[e].astype(np.float64).T
    for o in outs[:2]:
        mx, mean = bf16_errors(o, ref)
        say(f"  shared experts: max-abs {mx:.3e} mean-abs {mean:.3e}")
        assert mx <= 2e-2 and mean <= 2e-3
    assert np.max(np.abs(outs[0] - outs[1])) <= 2e-2


@pytest.mark.parametrize("T,S,k,E,d,f,packed", [(128, 4, 4, 60, 512, 320, False), (45, 2, 2, 16, 256, 192, True),
                                                 (1, 1, 2, 8, 128, 64, False), (33, 3, 4, 32, 256, 128, True),
                                                 (97, 1, 6, 64, 128, 256, False),
                                                 # one K stage for the gate/up product, two for the shared down
                                                 # projection: some waves of a K-splitting workgroup have no stage
                                                 (20, 2, 2, 8, 64, 64, False), (20, 2, 2, 8, 64, 64, True),
                                                 (128, 3, 2, 16, 192, 64, True)])
def test_small_batch_shared_experts_ride_in_the_routed_launches(T, S, k, E, d, f, packed):
    """Small batches: the shared experts' two products run inside the routed experts' weight-streaming launches (the
    down projection as one product whose K walks the S matrices, its four K quarters added in order).  h_shared and
    y_shared against the float64 definition, element by element; the call gives the same bits with and without
    scratch and with the repacked weights, whatever the scratch held."""
    say(f"paired shared experts T={T} S={S} k={k} E={E} d={d} f={f} packed={packed}")
    dev = require_gpu()
    D = 4
    shape = wl.LayerShape("pair", T=T, d=d, f=f, E=E, S=S, k=k, D=D, dtype="bf16", components=4)
    wk = wl.make_workload(shape, seed=T + S)
    layer = OccultLayer(T, d, f, E, S, k, D, "bf16")
    from paper_2505_13345_amd import binding as B
    assert B.occult_expert_ffn_ws_bytes(layer.cfg) == 0 and layer.ffn_ws is None     # nothing to split here
    layer.ffn_ws = torch.full((1024,), float("nan"), dtype=torch.float32, device=dev)   # passed along, never read
    x = to_dev(wk.x, "bf16", dev)
    wg, wu, wd = (to_dev(a, "bf16", dev) for a in (wk.w_gate, wk.w_up, wk.w_down))
    layer.route(torch.from_numpy(wk.logits).to(dev)); layer.make_plan(); layer.dispatch(x)
    res = {}
    for tag, use_ws in (("plain", False), ("scratch", True), ("scratch again", True)):
        if packed and use_ws and getattr(layer, "packed", None) is None:
            assert layer.pack_weights(wg, wu, wd) is not None
        layer.h_shared.fill_(7.0); layer.y_shared.fill_(7.0); layer.epd_y.fill_(7.0); layer.epd_h.fill_(7.0)
        layer.expert_ffn(x, wg, wu, wd, use_ws=use_ws)
        torch.cuda.synchronize()
        res[tag] = [t.float().cpu().numpy().copy() for t in (layer.h_shared, layer.y_shared, layer.epd_h, layer.epd_y)]
    xs = wk.x.astype(np.float64)
    h_ref = np.zeros((T, S * f)); y_ref = np.zeros((T, d))
    for s_ in range(S):
        e = E + s_
        g = xs @ wk.w_gate[e].astype(np.float64).T
        u = xs @ wk.w_up[e].astype(np.float64).T
        h_ref[:, s_ * f:(s_ + 1) * f] = g / (1.0 + np.exp(-g)) * u
    for tag in ("plain", "scratch"):
        h, y = res[tag][0], res[tag][1]
        assert_one_rounding(h, h_ref, f"h_shared {tag}")
        # the down projection on the stored (rounded) h, as the kernel sees it
        y_st = np.zeros((T, d))
        for s_ in range(S):
            y_st += h[:, s_ * f:(s_ + 1) * f].astype(np.float64) @ wk.w_down[E + s_].astype(np.float64).T
        assert_one_rounding(y, y_st, f"y_shared {tag}")
    for other in ("scratch", "scratch again"):
        for a, b in zip(res["plain"], res[other]):
            assert np.array_equal(a, b)


def test_empty_batch_runs_every_call():
    """T = 0: every entry point returns without touching memory (the Gram matrix is still cleared)."""
    from paper_2505_13345_amd import binding as B
    dev = require_gpu()
    E, D, k, d, f, S = 16, 4, 4, 128, 64, 1
    layer = OccultLayer(0, d, f, E, S, k, D, "bf16")
    x = torch.zeros((0, d), dtype=torch.bfloat16, device=dev)
    wg = torch.zeros((E + S, f, d), dtype=torch.bfloat16, device=dev)
    wd = torch.zeros((E + S, d, f), dtype=torch.bfloat16, device=dev)
    y = layer.forward(torch.zeros((0, E), device=dev), x, wg, wg, wd)
    assert y.shape == (0, d)
    wr = torch.zeros((E, d), dtype=torch.bfloat16, device=dev)
    layer.route_from_hidden(x, wr, torch.zeros((0, E), device=dev))
    B.occult_dispatch_meta(layer.cfg, layer.plan, layer.ids, layer.w,
                           torch.zeros((1, k), dtype=torch.int32, device=dev), torch.zeros((1, k), device=dev))
    gram = torch.full((E, E), 5.0, dtype=torch.float64, device=dev)
    B.occult_similarity_gram(layer.cfg, torch.zeros((0, E), device=dev), gram, accumulate=False)
    C = torch.full((E, E), 5, dtype=torch.int32, device=dev)
    B.occult_coactivation(layer.cfg, layer.ids, C, False)
    torch.cuda.synchronize()
    assert float(gram.abs().max()) == 0.0 and int(C.abs().max()) == 0
    assert layer.stats().n_sfd == 0


def _packed_reference(wg, wu, wd):
    """The documented packed order written out with numpy (uint16 views of bf16 weights):
    all gate|up pairs, then all down matrices; units of 32 output columns; stages of 64 K elements;
    blocks of 1 KiB ordered (K step of 32, gate or up, column block of 16); piece l of a block = row
    l % 16 of the column block at K offset (l // 16) * 8."""
    n, f, d = wg.shape
    lanes = np.arange(64)
    rows, koff = lanes % 16, (lanes // 16) * 8

    def blocks(mats, N, K):          # mats: list of [N, K] arrays that alternate inside a stage
        out = []
        for cb in range(N // 32):
            for stage in range(K // 64):
                for ks in range(2):
                    for m in mats:
                        for nb in range(2):
                            r = cb * 32 + nb * 16 + rows
                            k0 = stage * 64 + ks * 32 + koff
                            out.append(np.stack([m[r[i], k0[i]:k0[i] + 8] for i in range(64)]).reshape(-1))
        return np.concatenate(out)

    part1 = [blocks([wg[e], wu[e]], f, d) for e in range(n)]
    part2 = [blocks([wd[e]], d, f) for e in range(n)]
    return np.concatenate(part1 + part2)


def test_pack_weights_layout_bit_exact():
    from paper_2505_13345_amd import binding as B
    dev = require_gpu()
    E, S, d, f = 3, 1, 128, 64
    rng = np.random.default_rng(4)
    layer = OccultLayer(8, d, f, E + 1, S, 2, 2, "bf16")          # E + 1 = 4 routed experts, one shared
    n = E + 1 + S
    as_u16 = lambda shape: rng.integers(0, 65536, size=shape, dtype=np.uint16)
    wg, wu, wd = as_u16((n, f, d)), as_u16((n, f, d)), as_u16((n, d, f))
    to_bf = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    packed = layer.pack_weights(to_bf(wg), to_bf(wu), to_bf(wd))
    torch.cuda.synchronize()
    assert packed.numel() * 2 == B.occult_pack_weights_bytes(layer.cfg) == n * 3 * d * f * 2
    got = packed.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, _packed_reference(wg, wu, wd))
    # a buffer that is too small is refused
    with pytest.raises(B.OccultError) as e:
        B.occult_pack_weights(layer.cfg, to_bf(wg), to_bf(wu), to_bf(wd), packed[:-8])
    assert e.value.code == -5


@pytest.mark.parametrize("name", ["decode_bf16", "few_rows"])
def test_packed_weights_give_bit_identical_ffn(name):
    say(f"packed weights {name}")
    dev = require_gpu()
    if name == "decode_bf16":
        shape = wl.CONFIGS[name]
    else:   # ragged: some experts empty, some over 32 rows (two row tiles), shared experts on the other kernels
        shape = wl.LayerShape(name, T=80, d=256, f=192, E=16, S=2, k=4, D=4, dtype="bf16", components=4)
    wk = wl.make_workload(shape, seed=17)
    layer, y_plain = _run_layer(shape, wk)
    epd_h, epd_y = layer.epd_h.clone(), layer.epd_y.clone()
    x = to_dev(wk.x, shape.dtype, dev)
    wg, wu, wd = (to_dev(a, shape.dtype, dev) for a in (wk.w_gate, wk.w_up, wk.w_down))
    layer.pack_weights(wg, wu, wd)
    layer.epd_h.zero_()
    layer.epd_y.zero_()
    y_packed = layer.forward(torch.from_numpy(wk.logits).to(dev), x, wg, wu, wd)
    torch.cuda.synchronize()
    assert torch.equal(layer.epd_h, epd_h) and torch.equal(layer.epd_y, epd_y)
    assert np.array_equal(y_packed.float().cpu().numpy(), y_plain)
