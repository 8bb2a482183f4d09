"""GPU parity for the backward pass of the expert computation and of the whole layer
(occult_transpose_weights, occult_expert_ffn_backward, and the chain occult_combine_backward ->
occult_expert_ffn_backward -> occult_dispatch_backward) against oracle/backward.py in float64.

Bars.  f32: max |g - o| / max(|o|, rms(o)) <= 2e-5 (a chain of four f32 products and the SwiGLU
derivative; the forward bar is 1e-5 for two products).
bf16: the chain stores eight tensors in bf16 on the way to dx (the forward's intermediate, the gate-scaled
output-gradient rows, the two pre-activations, the gradient of the intermediate, the pre-activation
gradients, the EPD gradient rows, the SFD payload, dx itself); one rounding moves a value by at most
2^-8 of itself.  Two comparisons:
 (A) against the oracle's chain with the same tensors rounded (storage=to_bf16).  The two sides then
     differ only where f32 accumulation (or the order of a sum) moves a value across a rounding boundary:
     such an element is off by one rounding step (2^-7 of the leading power of two of its value), and a
     later sum inherits the steps of its terms.  A stored value flips only if its f32 sum lands within the
     accumulation error (below 1e-5 of the value) of a boundary, and boundaries are 2^-8 .. 2^-7 of the value
     apart: under 0.3 % of the elements per stored tensor, compounding over the eight tensors and the sums
     over experts and devices to a few percent of the final elements, each off by one step.  Bar: no element
     further off than four steps at the scale of its row (|g - o| <= 2^-5 * max(|o|, rms of the row)), and
     mean |g - o| <= 2^-11 * rms (one element in sixteen off by a step).
 (B) against the exact gradient: mean |g - o| / rms within the quadrature sum of the roundings the tensor
     has passed (tests/helpers.py chain_mean_bar).
"""
import numpy as np
import pytest
import torch

from inputs import workloads as wl
from oracle import backward, routing
from paper_2505_13345_amd.layer import OccultLayer
from tests.helpers import cached_workload, chain_mean_bar, f32_rel_error, require_gpu, say, to_dev

pytestmark = pytest.mark.gpu


def _mean_rel(got, want):
    want = want.astype(np.float64)
    return float(np.abs(got.astype(np.float64) - want).mean() / np.sqrt(np.mean(want ** 2)))


def _row_rel_error(got, want):
    """max |g - o| / max(|o|, rms of o's row)."""
    want = want.astype(np.float64)
    row_rms = np.sqrt(np.mean(want ** 2, axis=-1, keepdims=True))
    den = np.maximum(np.maximum(np.abs(want), row_rms), 1e-30)
    return float((np.abs(got.astype(np.float64) - want) / den).max())


STEPS_MAX = 2.0 ** -5      # (A): four rounding steps of 2^-7 at the row's scale
STEPS_MEAN = 2.0 ** -11    # (A): one element in sixteen off by one step


def _check(name, got, exact, dtype, rounded=None, n_roundings=1, per_row=True):
    """f32: against the exact gradient.  bf16: (A) against the rounded chain if given, (B) against the exact
    gradient if given (see the module text)."""
    if dtype == "f32":
        mx = f32_rel_error(got, exact)
        say(f"  {name}: normalised max {mx:.3e}")
        assert mx <= 2e-5, name
        return
    if rounded is not None:
        mx = _row_rel_error(got, rounded) if per_row else f32_rel_error(got, rounded)
        mean = _mean_rel(got, rounded)
        say(f"  {name} vs rounded chain: max {mx:.3e} (bar {STEPS_MAX:.1e}), mean/rms {mean:.3e} (bar {STEPS_MEAN:.1e})")
        assert mx <= STEPS_MAX and mean <= STEPS_MEAN, name
    if exact is not None:
        mean = _mean_rel(got, exact)
        say(f"  {name} vs exact: mean/rms {mean:.3e} (bar {chain_mean_bar(n_roundings):.2e})")
        assert mean <= chain_mean_bar(n_roundings), name


def _check_weight_grads_on_stored_operands(layer, shape, x_np, dy_np, positions, x_dev=None, dy_dev=None):
    """The three products of occult_expert_ffn_backward_weights written out on the library's own
    stored operands (each of them compared with the oracle elsewhere in this file), in float64:
    pins the kernel's own arithmetic (f32 accumulation over an expert's rows) tightly.  Bar: 1e-5 of the
    matrix's scale up to 10^4 rows; beyond, the rounding of n sequential f32 additions grows like
    eps * sqrt(n) relative to the sum's own size, and the maximum over 10^7 elements sits ~5 deviations out:
    1e-7 * sqrt(rows)."""
    tabs = layer.tables()
    exp_off = tabs["exp_offset"].cpu().numpy()
    pos_expert = tabs["pos_expert"].cpu().numpy()
    src = tabs["epd_sfd_row"].long()
    f = shape.f
    for P in positions:
        q0, q1 = int(exp_off[P]), int(exp_off[P + 1])
        e = int(pos_expert[P])
        dyq = layer.epd_dy[q0:q1].double()
        gu = layer.epd_gu[q0:q1].double()
        xq = layer.sfd_x[src[q0:q1]].double()
        for name, want in (("dw_down", dyq.T @ layer.epd_h[q0:q1].double()), ("dw_gate", gu[:, :f].T @ xq),
                           ("dw_up", gu[:, f:].T @ xq)):
            got = getattr(layer, name)[e].cpu().numpy()
            if q1 == q0:
                assert not got.any(), (name, P)
            else:
                assert f32_rel_error(got, want.cpu().numpy()) <= max(1e-5, 1e-7 * np.sqrt(q1 - q0)), (name, P)
    if shape.S == 0:
        return
    xs = (torch.from_numpy(x_np).to(layer.device) if x_dev is None else x_dev).double()
    dys = (torch.from_numpy(dy_np).to(layer.device) if dy_dev is None else dy_dev).double()
    for sidx in range(shape.S):
        e = shape.E + sidx
        gu = layer.gu_shared[:, sidx * 2 * f:(sidx + 1) * 2 * f].double()
        want = dys.T @ layer.h_shared[:, sidx * f:(sidx + 1) * f].double()
        bar = max(1e-5, 1e-7 * np.sqrt(xs.shape[0]))
        assert f32_rel_error(layer.dw_down[e].cpu().numpy(), want.cpu().numpy()) <= bar
        assert f32_rel_error(layer.dw_gate[e].cpu().numpy(), (gu[:, :f].T @ xs).cpu().numpy()) <= bar
        assert f32_rel_error(layer.dw_up[e].cpu().numpy(), (gu[:, f:].T @ xs).cpu().numpy()) <= bar


def _check_per_matrix(name, got, exact, dtype, rounded=None):
    """Weight gradients (f32 sums over an expert's rows): every expert's matrix normalised by that matrix's own
    rms (experts differ widely in their number of rows, and so in the size of their gradients and errors).
    bf16: (A) against the rounded chain: the factors differ by a rounding step in about one row in a
    thousand, so the sums agree far inside one rounding: mean <= 2^-10 of the rms, no element beyond 2^-6
    of max(|o|, rms); (B) against the exact gradient: the mean within the quadrature sum of the five roundings
    a factor has passed.  The product itself is pinned to 1e-5 on its stored operands below."""
    worst_mx = worst_mean = worst_exact = 0.0
    for e in range(exact.shape[0]):
        if not exact[e].any():
            assert not got[e].any(), (name, e)
            continue
        if dtype == "f32":
            worst_mx = max(worst_mx, f32_rel_error(got[e], exact[e]))
            continue
        worst_mx = max(worst_mx, f32_rel_error(got[e], rounded[e]))
        worst_mean = max(worst_mean, _mean_rel(got[e], rounded[e]))
        worst_exact = max(worst_exact, _mean_rel(got[e], exact[e]))
    say(f"  {name}: worst expert: max {worst_mx:.3e}, mean/rms {worst_mean:.3e}; vs exact mean/rms {worst_exact:.3e}")
    if dtype == "f32":
        assert worst_mx <= 2e-5, name
    else:
        assert worst_mx <= 2.0 ** -6 and worst_mean <= 2.0 ** -10, name
        assert worst_exact <= chain_mean_bar(5), name


def _forward_backward(shape, wk, pos, dy):
    dev = require_gpu()
    layer = OccultLayer(shape.T, shape.d, shape.f, shape.E, shape.S, shape.k, shape.D, shape.dtype,
                        shape.n_d, shape.prune_mode, shape.renorm, pos)
    x = to_dev(wk.x, shape.dtype, dev)
    wg, wu, wd = (to_dev(a, shape.dtype, dev) for a in (wk.w_gate, wk.w_up, wk.w_down))
    layer.forward(torch.from_numpy(wk.logits).to(dev), x, wg, wu, wd)
    w_down_t, w_gu_t = layer.transpose_weights(wg, wu, wd)
    dy_d = to_dev(dy, shape.dtype, dev)
    dx, dw = layer.backward_input(x, wg, wu, dy_d)
    layer.expert_ffn_backward_weights(x, dy_d)
    torch.cuda.synchronize()
    # the transposed copies, bit for bit
    assert torch.equal(w_down_t, wd.transpose(1, 2).contiguous())
    assert torch.equal(w_gu_t, torch.cat([wg.transpose(1, 2), wu.transpose(1, 2)], dim=2))
    return layer, dx.float().cpu().numpy(), dw.cpu().numpy()


SMALL = [
    # name, T, d, f, E, S, k, D, dtype   (the forward test's shapes: every GEMM variant, ragged tails)
    ("f32_a", 300, 96, 80, 8, 0, 2, 4, "f32"),
    ("f32_shared", 130, 128, 256, 16, 2, 4, 4, "f32"),
    ("bf16_a", 700, 256, 192, 8, 0, 2, 4, "bf16"),
    ("bf16_shared", 333, 512, 320, 12, 2, 3, 3, "bf16"),
    ("bf16_one_row_experts", 9, 128, 64, 16, 1, 2, 8, "bf16"),
    ("bf16_big_expert", 1500, 192, 448, 4, 0, 1, 2, "bf16"),
    ("bf16_few_rows_ragged", 80, 256, 192, 16, 2, 4, 4, "bf16"),
    ("bf16_big_shared", 1100, 192, 128, 4, 3, 1, 4, "bf16"),
    # hidden rows of 14 KiB (two column chunks in combine), long K in the first product
    ("bf16_wide_rows", 200, 7168, 128, 32, 1, 4, 8, "bf16"),
    # outputs narrower than a wave tile of the 256-row kernel (d = 64 forward, f = 64 backward): the store
    # range must end inside the group's last row
    ("bf16_narrow_d", 900, 64, 128, 8, 0, 3, 2, "bf16"),
    ("bf16_narrow_f", 1100, 192, 64, 8, 0, 3, 1, "bf16"),
    # many experts with 160 rows or more and short hidden rows: the gathered weight-gradient product reads the
    # row indices of its fifth step while the loads issued before them are still in flight
    ("bf16_gather_steps", 2300, 576, 704, 64, 0, 4, 16, "bf16"),
    # two shared experts over 5000 rows with one output tile each: their weight-gradient products are cut into row
    # slices summed from scratch memory (the last slice ragged)
    ("bf16_shared_row_slices", 5000, 128, 128, 4, 2, 1, 2, "bf16"),
]


@pytest.mark.parametrize("name,T,d,f,E,S,k,D,dtype", SMALL)
def test_small_layers_backward_elementwise(name, T, d, f, E, S, k, D, dtype):
    say(f"small layer backward {name}")
    shape = wl.LayerShape(name, T=T, d=d, f=f, E=E, S=S, k=k, D=D, dtype=dtype,
                          components=4 if dtype == "bf16" else 0)
    wk = wl.make_workload(shape, seed=17)
    pos = wl.random_placement(E, D, seed=2)
    dy = np.random.default_rng(T).standard_normal((T, d)).astype(np.float32)
    if dtype == "bf16":
        dy = wl.round_to_bf16(dy)
    layer, dx, dw = _forward_backward(shape, wk, pos, dy)
    ids, w = layer.ids.cpu().numpy(), layer.w.cpu().numpy().astype(np.float64)
    ids_ref, _ = routing.route(wk.logits, k, D, pos)
    assert np.array_equal(ids, ids_ref)
    res = backward.layer_backward(wk.x, ids, w, pos, D, wk.w_gate, wk.w_up, wk.w_down, S, dy.astype(np.float64))
    rnd = None
    if dtype == "bf16":
        rnd = backward.layer_backward(wk.x, ids, w, pos, D, wk.w_gate, wk.w_up, wk.w_down, S, dy.astype(np.float64),
                                      storage=backward.to_bf16)
    n_sfd = res["trace"].n_sfd
    cat = lambda r, key: None if r is None else np.concatenate(r[key])
    get = lambda r, key: None if r is None else r[key]
    _check("epd_dy", layer.epd_dy.float().cpu().numpy(), cat(res, "g_epd_y"), dtype, cat(rnd, "g_epd_y"), 1)
    _check("epd_gu", layer.epd_gu.float().cpu().numpy(), cat(res, "g_epd_gu"), dtype, cat(rnd, "g_epd_gu"), 5)
    _check("epd_dx", layer.epd_dx.float().cpu().numpy(), cat(res, "g_epd_x"), dtype, cat(rnd, "g_epd_x"), 6)
    _check("sfd_dx", layer.sfd_dx[:n_sfd].float().cpu().numpy(), res["g_sfd_x"], dtype, get(rnd, "g_sfd_x"), 7)
    _check("dx", dx, res["g_x"], dtype, get(rnd, "g_x"), 8)
    _check("dw", dw, res["g_w"], dtype, get(rnd, "g_w"), 2, per_row=False)
    assert np.array_equal(layer.sfd_dy[:n_sfd].float().cpu().numpy(), res["g_sfd_y"])   # a copy of dy rows
    # weight gradients (f32 outputs; their inputs carry the roundings of the chain above)
    grads = {n: getattr(layer, n).cpu().numpy() for n in ("dw_gate", "dw_up", "dw_down")}
    for n, ref in (("dw_gate", "g_w_gate"), ("dw_up", "g_w_up"), ("dw_down", "g_w_down")):
        _check_per_matrix(n, grads[n], res[ref], dtype, get(rnd, ref))   # experts without rows: exact zeros
    _check_weight_grads_on_stored_operands(layer, shape, wk.x, dy, range(E))
    if name == "bf16_shared_row_slices":
        from paper_2505_13345_amd import binding as B
        assert B.occult_expert_ffn_backward_weights_ws_bytes(layer.cfg) == 2 * S * d * f * 4 and layer.wgrad_ws is not None
        # without the scratch the same products run unsplit: the same numbers up to the order of the f32 sums
        unsplit = [g.clone() for g in layer.expert_ffn_backward_weights(to_dev(wk.x, dtype, require_gpu()),
                                                                        to_dev(dy, dtype, require_gpu()), use_ws=False)]
        torch.cuda.synchronize()
        for n, u in zip(("dw_gate", "dw_up", "dw_down"), unsplit):
            assert np.array_equal(u[:E].cpu().numpy(), grads[n][:E])                 # routed experts: untouched by the split
            assert f32_rel_error(u[E:].cpu().numpy(), grads[n][E:]) <= 1e-5          # shared experts: other summation order
            assert not np.array_equal(u[E:].cpu().numpy(), grads[n][E:])
        layer.expert_ffn_backward_weights(to_dev(wk.x, dtype, require_gpu()), to_dev(dy, dtype, require_gpu()))
        torch.cuda.synchronize()
    # accumulate = 1 adds the same product again: exactly twice the first result
    layer.expert_ffn_backward_weights(to_dev(wk.x, dtype, require_gpu()), to_dev(dy, dtype, require_gpu()), accumulate=True)
    torch.cuda.synchronize()
    for n in grads:
        assert np.array_equal(getattr(layer, n).cpu().numpy(), 2 * grads[n]), n


_runs = {}


def _full_size_run(name):
    """Forward + backward of one configuration on the GPU, once per session: dx, dw on the host, the layer kept."""
    if name not in _runs:
        shape = wl.CONFIGS[name]
        wk = cached_workload(shape)
        dy = wl.round_to_bf16(np.random.default_rng(5).standard_normal((shape.T, shape.d), dtype=np.float32))
        say(f"{name}: forward + backward on GPU")
        layer, dx, dw = _forward_backward(shape, wk, None, dy)
        assert np.isfinite(dx).all() and np.isfinite(dw).all()
        _runs.clear()
        _runs[name] = (wk, dy, layer, dx, dw)
    return _runs[name]


def _backward_rows(name, lo, hi):
    """dx and dw of tokens [lo, hi) against the rounded chain of the oracle evaluated on those tokens alone
    (a token's gradients depend on its own row, its routing and the weights; the sums over its experts and
    devices keep their order whatever else is in the batch)."""
    shape = wl.CONFIGS[name]
    wk, dy, layer, dx, dw = _full_size_run(name)
    ids, w = layer.ids.cpu().numpy(), layer.w.cpu().numpy().astype(np.float64)
    say(f"{name}: oracle backward (rounded chain) on tokens [{lo}, {hi})")
    sl = slice(lo, hi)
    res = backward.layer_backward(wk.x[sl], ids[sl], w[sl], wl.contiguous_placement(shape.E, shape.D), shape.D, wk.w_gate,
                                  wk.w_up, wk.w_down, shape.S, dy[sl].astype(np.float64), storage=backward.to_bf16)
    _check(f"dx [{lo}, {hi})", dx[sl], None, "bf16", res["g_x"])
    _check(f"dw [{lo}, {hi})", dw[sl], None, "bf16", res["g_w"], per_row=False)


def test_decode_config_backward():
    shape = wl.CONFIGS["decode_bf16"]
    _backward_rows("decode_bf16", 0, shape.T)
    wk, dy, layer, dx, dw = _full_size_run("decode_bf16")
    _check_weight_grads_on_stored_operands(layer, shape, wk.x, dy, range(shape.E))


def test_prefill_config_backward_all_rows():
    shape = wl.CONFIGS["prefill_bf16"]
    _backward_rows("prefill_bf16", 0, shape.T)
    wk, dy, layer, dx, dw = _full_size_run("prefill_bf16")
    _check_weight_grads_on_stored_operands(layer, shape, wk.x, dy, sorted(set(range(0, shape.E, 8)) | {shape.E - 1}))


@pytest.mark.parametrize("part", range(4))
def test_large_config_backward_all_rows(part):
    shape = wl.CONFIGS["large_bf16"]
    n = shape.T // 4
    _backward_rows("large_bf16", part * n, (part + 1) * n)
    if part == 3:
        wk, dy, layer, dx, dw = _full_size_run("large_bf16")
        _check_weight_grads_on_stored_operands(layer, shape, wk.x, dy, [0, 21, 42, shape.E - 1])
        _runs.clear()


def test_ffn_backward_argument_checks():
    from paper_2505_13345_amd import binding as B
    dev = require_gpu()
    layer = OccultLayer(8, 64, 64, 4, 1, 2, 2, "bf16")
    z = torch.zeros((64, 64), dtype=torch.bfloat16, device=dev)
    with pytest.raises(B.OccultError) as e:   # shared experts need their buffers
        B.occult_expert_ffn_backward(layer.cfg, layer.plan, z, z, z, z, z, z, z, z, z, z, z, None, None, None)
    assert e.value.code == -4
    with pytest.raises(B.OccultError) as e:
        B.occult_transpose_weights(layer.cfg, z, z, z, None, z)
    assert e.value.code == -4
    empty = OccultLayer(0, 64, 64, 4, 0, 2, 2, "bf16")
    B.occult_expert_ffn_backward(empty.cfg, empty.plan, None, None, None, None, None, None, None, None, None, None, None)
    torch.cuda.synchronize()


KEEP_CASES = [
    ("bf16_a", 700, 256, 192, 8, 0, 2, 4, "bf16"),                  # 256-row tiles: stored by the first product itself
    ("bf16_big_shared", 1100, 192, 128, 4, 3, 1, 4, "bf16"),        # the same with shared experts as uniform groups
    ("bf16_few_rows_ragged", 80, 256, 192, 16, 2, 4, 4, "bf16"),    # other kernels: two more products
    ("f32_shared", 130, 128, 256, 16, 2, 4, 4, "f32"),
]


@pytest.mark.parametrize("name,T,d,f,E,S,k,D,dtype", KEEP_CASES)
def test_kept_preactivations_give_the_recomputed_gradients(name, T, d, f, E, S, k, D, dtype):
    """occult_expert_ffn_train + gu_saved = 1 against the recomputing backward (itself compared with the
    oracle above): same forward outputs, same gradients, bit for bit (the kept values are rounded from
    the same accumulators the recomputation produces)."""
    say(f"kept pre-activations {name}")
    dev = require_gpu()
    shape = wl.LayerShape(name, T=T, d=d, f=f, E=E, S=S, k=k, D=D, dtype=dtype, components=4 if dtype == "bf16" else 0)
    wk = wl.make_workload(shape, seed=17)
    pos = wl.random_placement(E, D, seed=2)
    dy = np.random.default_rng(T).standard_normal((T, d)).astype(np.float32)
    if dtype == "bf16":
        dy = wl.round_to_bf16(dy)
    x = to_dev(wk.x, dtype, dev)
    wg, wu, wd = (to_dev(a, dtype, dev) for a in (wk.w_gate, wk.w_up, wk.w_down))
    dy_d = to_dev(dy, dtype, dev)
    logits = torch.from_numpy(wk.logits).to(dev)
    results = []
    for train in (False, True):
        layer = OccultLayer(T, d, f, E, S, k, D, dtype, expert_pos=pos)
        y = layer.forward(logits, x, wg, wu, wd, train=train).clone()
        gu_fwd = layer.epd_gu.clone() if train else None
        layer.transpose_weights(wg, wu, wd)
        dx, dw = layer.backward_input(x, wg, wu, dy_d)
        grads = layer.expert_ffn_backward_weights(x, dy_d)
        torch.cuda.synchronize()
        assert getattr(layer, "gu_saved", False) is False
        results.append(dict(y=y, h=layer.epd_h.clone(), dx=dx.clone(), dw=dw.clone(), gu=layer.epd_gu.clone(),
                            epd_dx=layer.epd_dx.clone(), grads=[g.clone() for g in grads], gu_fwd=gu_fwd,
                            dx_sh=layer.dx_shared.clone() if S else None))
    a, b = results
    for key in ("y", "h", "dx", "dw", "gu", "epd_dx"):
        assert torch.equal(a[key], b[key]), key
    for ga, gb in zip(a["grads"], b["grads"]):
        assert torch.equal(ga, gb)
    if S:
        assert torch.equal(a["dx_sh"], b["dx_sh"])
    assert b["gu_fwd"].float().abs().max() > 0          # the kept values were really written by the forward call
