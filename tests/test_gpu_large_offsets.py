"""Buffers past 4 GiB: every row-indexed buffer of the hot path (SFD and EPD rows of 16 KiB each) is larger
than a 32-bit byte offset reaches, so an offset computed in 32 bits anywhere would address the wrong row.

Inputs are tiled from a small table of rows, row t = table[t mod P] with P prime (a period that no
power-of-two wrap-around maps onto itself), so the host holds only the table and the oracle runs on one
column: the data movement is linear per column, hence the oracle's result for a column of coefficients,
times the table row, is the exact expected row (small integers and power-of-two gates: every product and
partial sum is exactly representable)."""
import numpy as np
import pytest
import torch

from inputs import workloads as wl
from oracle import backward, moe_std, occult_ref, routing
from paper_2505_13345_amd.layer import OccultLayer
from tests.helpers import bf16_errors, check_plan_against_trace, expand_plan, f32_rel_error, require_gpu, say

pytestmark = pytest.mark.gpu

P = 4099


def _rows_equal(got, coef, table_d, tok, chunk=32768):
    """got[r] == coef[r] * table[tok[r] mod P] for every row, in chunks (the operands are exact in float32)."""
    dev = got.device
    coef_d = torch.from_numpy(np.asarray(coef, dtype=np.float32)).to(dev)
    tok_d = torch.from_numpy(np.asarray(tok, dtype=np.int64)).to(dev)
    for r0 in range(0, got.shape[0], chunk):
        r1 = min(r0 + chunk, got.shape[0])
        want = table_d[tok_d[r0:r1] % P] * coef_d[r0:r1, None]
        if not torch.equal(got[r0:r1].float(), want):
            return False
    return True


def _split_by_device(rows, trace):
    out, base = [], 0
    for b1 in trace.brim_1:
        n = int((b1 >= 0).sum())
        out.append(rows[base:base + n])
        base += n
    return out


def test_data_movement_past_4gib_forward_and_backward():
    dev = require_gpu()
    E, D, k, T, d = 8, 4, 4, 90001, 8192
    say(f"large offsets, data movement: T={T} d={d} k={k} D={D}: EPD buffers of {T * k * d * 2 / 2**30:.2f} GiB")
    lg = wl.random_logits(T, E, seed=77)
    pos_arr = wl.contiguous_placement(E, D)
    ids, _ = routing.route(lg, k, D, None)
    w = np.tile(np.array([.5, .25, .125, .125]), (T, 1)).astype(np.float32)
    w64 = w.astype(np.float64)
    scale = (np.arange(E) % 3 + 1).astype(np.float64)
    table = wl.integer_valued_rows(P, d, seed=3, lo=-3, hi=3)
    table_d = torch.from_numpy(table).to(dev)                       # float32, exact small integers
    tok = np.arange(T)
    x_d = table_d[torch.from_numpy(tok % P).to(dev)].to(torch.bfloat16)

    layer = OccultLayer(T, d, 64, E, 0, k, D, "bf16", with_ffn=False)
    ids_d = torch.from_numpy(ids).to(dev)
    layer.make_plan(ids_d, torch.from_numpy(w).to(dev))
    layer.dispatch(x_d)
    torch.cuda.synchronize()

    # oracle on single columns: the token index (which token each SFD row holds) and ones (coefficients)
    tr_tok = occult_ref.moe_forward(tok[:, None].astype(np.float64), ids, w64, pos_arr, D, bypass_scale=scale,
                                    acc=np.float64)
    tr_one = occult_ref.moe_forward(np.ones((T, 1)), ids, w64, pos_arr, D, bypass_scale=scale, acc=np.float64)
    n = tr_tok.n_sfd
    assert n * d * 2 > 2 ** 32, "the SFD rows in use must themselves pass 4 GiB"
    sfd_tok = tr_tok.x_sfd[:, 0].astype(np.int64)
    exp = expand_plan(layer.tables(), T, E, D, k)
    check_plan_against_trace(exp, tr_tok, ids, w, None, T, E, D, k)
    say("  dispatch")
    assert _rows_equal(layer.sfd_x[:n], np.ones(n), table_d, sfd_tok)

    # expert stand-in (test scaffolding): epd_y[q] = scale[expert of q] * sfd_x[source row of q]
    tabs = layer.tables()
    exp_off = tabs["exp_offset"].cpu().numpy()
    pos_expert = tabs["pos_expert"].cpu().numpy()
    row_scale = np.repeat(scale[pos_expert], np.diff(exp_off)).astype(np.float32)
    src = tabs["epd_sfd_row"].long()
    epd_y = torch.empty((T * k, d), dtype=torch.bfloat16, device=dev)
    rs_d = torch.from_numpy(row_scale).to(dev)
    for q0 in range(0, T * k, 65536):
        q1 = min(q0 + 65536, T * k)
        epd_y[q0:q1] = (layer.sfd_x[src[q0:q1]].float() * rs_d[q0:q1, None]).to(torch.bfloat16)
    say("  combine")
    layer.combine(epd_y)
    torch.cuda.synchronize()
    assert _rows_equal(layer.sfd_y[:n], tr_one.y_sfd[:, 0], table_d, sfd_tok)
    assert _rows_equal(layer.y, tr_one.y[:, 0], table_d, tok)

    # backward of combine with dy = x: copies of dy rows, gate-scaled EPD rows, gate gradients
    say("  combine backward")
    sfd_dy, epd_dy, dw = layer.combine_backward(x_d, ids_d, epd_y)
    torch.cuda.synchronize()
    L = occult_ref.placement_lists(pos_arr, D)
    scale_rows = _split_by_device(row_scale.astype(np.float64)[:, None], tr_one)
    args = (scale_rows, tr_one.brim_0, tr_one.brim_1, tr_one.brim_w, tr_one.dev_count)
    _, g_out_one, g_w_one = backward.combine_backward(np.ones((T, 1)), *args)
    _, g_out_tok, _ = backward.combine_backward(tok[:, None].astype(np.float64), *args)
    gate_q = np.concatenate(g_out_one)[:, 0]                      # gate of every EPD row
    epd_tok = np.rint(np.concatenate(g_out_tok)[:, 0] / gate_q).astype(np.int64)
    assert _rows_equal(sfd_dy[:n], np.ones(n), table_d, sfd_tok)
    assert _rows_equal(epd_dy, gate_q, table_d, epd_tok)
    # dw[t, j] = <dy[t], epd_y[q]> = scale_q |x_t|^2: below 2^24, exact in float32 in any order
    normsq = (table.astype(np.float64) ** 2).sum(axis=1)
    want_dw = backward.gate_grad_to_slots(g_w_one, ids, tr_one.brim_0, L, tr_one.dev_count) * normsq[tok % P][:, None]
    assert want_dw.max() < 2 ** 24
    assert np.array_equal(dw.cpu().numpy().astype(np.float64), want_dw)

    # backward of dispatch with epd_dx = epd_y (coefficient scale_q on the token's row)
    say("  dispatch backward")
    sfd_dx, dx = layer.dispatch_backward(epd_y)
    torch.cuda.synchronize()
    g_sfd_x, g_x = backward.dispatch_backward(scale_rows, tr_one.brim_0, tr_one.brim_1, tr_one.dev_count)
    assert _rows_equal(sfd_dx[:n], g_sfd_x[:, 0], table_d, sfd_tok)
    assert _rows_equal(dx, g_x[:, 0], table_d, tok)


def test_expert_ffn_past_4gib_forward_and_backward():
    """Hidden-row buffers of the experts past 4 GiB (gathered input rows, output rows, their gradients):
    sampled tokens against the oracles, weight gradients against the float64 product of the stored operands."""
    from tests.test_gpu_ffn_backward import _check_weight_grads_on_stored_operands
    dev = require_gpu()
    E, S, D, k, T, d, f = 8, 1, 4, 4, 70001, 8192, 1024
    say(f"large offsets, experts: T={T} d={d} f={f} k={k}: EPD rows of d take {T * k * d * 2 / 2**30:.2f} GiB")
    rng = np.random.default_rng(4242)
    lg = wl.random_logits(T, E, seed=78, scale=1.3)
    table = wl.round_to_bf16((rng.standard_normal((P, d)) * 0.7).astype(np.float32))
    P2 = 4093
    table_dy = wl.round_to_bf16(rng.standard_normal((P2, d)).astype(np.float32))
    wg = wl.round_to_bf16((rng.standard_normal((E + S, f, d)) / np.sqrt(d)).astype(np.float32))
    wu = wl.round_to_bf16((rng.standard_normal((E + S, f, d)) / np.sqrt(d)).astype(np.float32))
    wd = wl.round_to_bf16((rng.standard_normal((E + S, d, f)) * 0.25 / np.sqrt(f)).astype(np.float32))
    tok = np.arange(T)
    bf = torch.bfloat16
    x_d = torch.from_numpy(table).to(dev).to(bf)[torch.from_numpy(tok % P).to(dev)]
    dy_d = torch.from_numpy(table_dy).to(dev).to(bf)[torch.from_numpy(tok % P2).to(dev)]
    wg_d, wu_d, wd_d = (torch.from_numpy(a).to(dev).to(bf) for a in (wg, wu, wd))

    layer = OccultLayer(T, d, f, E, S, k, D, "bf16")
    assert layer.epd_y.numel() * 2 > 2 ** 32 and layer.sfd_x.numel() * 2 > 2 ** 32
    y = layer.forward(torch.from_numpy(lg).to(dev), x_d, wg_d, wu_d, wd_d, train=True)
    layer.transpose_weights(wg_d, wu_d, wd_d)
    dx, dw = layer.backward_input(x_d, wg_d, wu_d, dy_d)
    layer.expert_ffn_backward_weights(x_d, dy_d)
    torch.cuda.synchronize()
    ids, w = layer.ids.cpu().numpy(), layer.w.cpu().numpy().astype(np.float64)
    ids_ref, _ = routing.route(lg, k, D, None)
    assert np.array_equal(ids, ids_ref)

    tokens = np.sort(np.random.default_rng(9).choice(T, size=96, replace=False))
    tokens[0], tokens[-1] = 0, T - 1
    xs, dys = table[tokens % P], table_dy[tokens % P2]
    say("  oracle on 96 sampled tokens")
    y_ref = moe_std.moe_layer(xs, ids[tokens], w[tokens], wg, wu, wd, E, S)
    mx, mean = bf16_errors(y[tokens].float().cpu().numpy(), y_ref)
    say(f"  y max-abs {mx:.3e} mean-abs {mean:.3e}")
    assert mx <= 2e-2 and mean <= 2e-3
    g_x, g_w = backward.moe_layer_backward_tokens(xs, ids[tokens], w[tokens], wg, wu, wd, E, S, dys)
    for name, got, want in (("dx", dx[tokens].float().cpu().numpy(), g_x), ("dw", dw[tokens].cpu().numpy(), g_w)):
        mean_rel = float(np.abs(got - want).mean() / np.sqrt(np.mean(want ** 2)))
        say(f"  {name}: normalised max {f32_rel_error(got, want):.3e}, mean/rms {mean_rel:.3e}")
        assert f32_rel_error(got, want) <= 8e-2 and mean_rel <= 4e-3, name
    # every output row written and finite (rows are reached through offsets past 4 GiB on the way)
    assert bool(torch.isfinite(y).all()) and bool(torch.isfinite(dx).all())
    assert bool((y.float().abs().sum(dim=1) > 0).all()) and bool((dx.float().abs().sum(dim=1) > 0).all())

    class _Shape:
        pass
    shape = _Shape()
    shape.f, shape.S, shape.E = f, S, E
    say("  weight gradients on the stored operands")
    _check_weight_grads_on_stored_operands(layer, shape, None, None, [0, 3, E - 1], x_dev=x_d, dy_dev=dy_d)
