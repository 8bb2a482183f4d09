"""Seeded sweep over layer shapes (ragged tiles in every dimension, every kernel choice): the whole
forward and backward pass of each against the float64 oracles, at the bars of the fixed-shape tests."""
import numpy as np
import pytest
import torch

from inputs import workloads as wl
from oracle import backward, moe_std, routing
from paper_2505_13345_amd.layer import OccultLayer
from tests.helpers import bf16_errors, f32_rel_error, require_gpu, say, to_dev

pytestmark = pytest.mark.gpu


def _draw(seed):
    rng = np.random.default_rng(1000 + seed)
    E = int(rng.choice([4, 6, 8, 12, 16, 24, 48, 64]))
    D = int(rng.choice([j for j in (1, 2, 3, 4, 6, 8, 12, 16) if E % j == 0]))
    k = int(rng.integers(1, min(E, 8) + 1))
    T = int(rng.choice([1, 7, 33, 130, 257, 600, 1100, 2300, 4100]))
    d = int(rng.choice([64, 128, 192, 320, 576, 1024]))
    f = int(rng.choice([64, 128, 192, 448, 704]))
    S = int(rng.choice([0, 0, 1, 2, 3]))
    n_d = int(rng.choice([0, 0, min(D, 2)]))
    if n_d and n_d * (E // D) < k:
        n_d = 0
    return dict(T=T, d=d, f=f, E=E, S=S, k=k, D=D, n_d=n_d)


def _mean_rel(got, want):
    want = want.astype(np.float64)
    rms = np.sqrt(np.mean(want ** 2))
    return float(np.abs(got.astype(np.float64) - want).mean() / rms) if rms > 0 else float(np.abs(got).max())


@pytest.mark.parametrize("seed", range(40))
def test_random_layer_forward_and_backward(seed):
    p = _draw(seed)
    say(f"random layer {seed}: {p}")
    dev = require_gpu()
    dtype = "f32" if seed % 5 == 4 else "bf16"
    shape = wl.LayerShape(f"rand{seed}", dtype=dtype, components=4 if dtype == "bf16" else 0, prune_mode=1, **p)
    wk = wl.make_workload(shape, seed=seed)
    pos = wl.random_placement(p["E"], p["D"], seed=seed)
    T, d, E, S, k, D = p["T"], p["d"], p["E"], p["S"], p["k"], p["D"]
    layer = OccultLayer(T, d, p["f"], E, S, k, D, dtype, p["n_d"], 1, 1, pos)
    x = to_dev(wk.x, dtype, dev)
    wg, wu, wd = (to_dev(a, dtype, dev) for a in (wk.w_gate, wk.w_up, wk.w_down))
    train = seed % 2 == 0        # alternate kept and recomputed pre-activations
    y = layer.forward(torch.from_numpy(wk.logits).to(dev), x, wg, wu, wd, train=train).float().cpu().numpy()
    ids, w = layer.ids.cpu().numpy(), layer.w.cpu().numpy().astype(np.float64)
    ids_ref, _ = routing.route(wk.logits, k, D, pos, p["n_d"], 1, 1)
    assert np.array_equal(ids, ids_ref)
    y_ref = moe_std.moe_layer(wk.x, ids, w, wk.w_gate, wk.w_up, wk.w_down, E, S)
    if dtype == "bf16":
        mx, mean = bf16_errors(y, y_ref)
        assert mx <= 2e-2 and mean <= 2e-3, (mx, mean)
    else:
        assert f32_rel_error(y, y_ref) <= 1e-5
    if dtype == "bf16" and not train and layer.pack_weights(wg, wu, wd) is not None:
        # the repacked weights feed the same arithmetic: the same bits out, whichever kernel each product takes
        layer.expert_ffn(x, wg, wu, wd)
        layer.combine()
        assert np.array_equal(layer.y.float().cpu().numpy(), y)

    dy = np.random.default_rng(seed).standard_normal((T, d)).astype(np.float32)
    if dtype == "bf16":
        dy = wl.round_to_bf16(dy)
    dy_d = to_dev(dy, dtype, dev)
    layer.transpose_weights(wg, wu, wd)
    dx, dw = layer.backward_input(x, wg, wu, dy_d)
    grads = layer.expert_ffn_backward_weights(x, dy_d)
    torch.cuda.synchronize()
    res = backward.layer_backward(wk.x, ids, w, pos, D, wk.w_gate, wk.w_up, wk.w_down, S, dy.astype(np.float64))
    errs = {"dx": _mean_rel(dx.float().cpu().numpy(), res["g_x"]), "dw": _mean_rel(dw.cpu().numpy(), res["g_w"])}
    rows_of = np.bincount(ids.reshape(-1), minlength=E)
    for name, got, ref in zip(("dw_gate", "dw_up", "dw_down"), grads, ("g_w_gate", "g_w_up", "g_w_down")):
        got = got.cpu().numpy()
        errs[name] = _mean_rel(got, res[ref])           # all experts together: weighted by their rows
        for e in range(E + S):
            if not res[ref][e].any():
                assert not got[e].any(), (name, e)
            elif e >= E or rows_of[e] >= 32:            # one expert alone, once its sum averages over some rows
                errs[f"{name}[{e}]"] = _mean_rel(got[e], res[ref][e])
    say("  mean/rms " + " ".join(f"{n}={v:.1e}" for n, v in errs.items() if "[" not in n)
        + f" worst single expert {max([v for n, v in errs.items() if '[' in n] or [0.0]):.1e}")
    if dtype == "bf16":
        assert max(errs.values()) <= 5e-3, errs
        assert f32_rel_error(dx.float().cpu().numpy(), res["g_x"]) <= 1e-1
    else:
        assert max(errs.values()) <= 2e-6, errs
        assert f32_rel_error(dx.float().cpu().numpy(), res["g_x"]) <= 2e-5
    # accumulate = 1 adds the same products again: exactly twice the first result
    first = [g.clone() for g in grads]
    for got, one in zip(layer.expert_ffn_backward_weights(x, dy_d, accumulate=True), first):
        assert torch.equal(got, 2 * one)
