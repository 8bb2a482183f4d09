"""GPU parity for the backward pass of the data movement (occult_combine_backward,
occult_dispatch_backward) and of the routing weights (occult_route_backward) against
oracle/backward.py.  Copies are bit-exact; sums are bit-exact on inputs whose every partial sum is
exactly representable, and within the floating-point bars on random data."""
import numpy as np
import pytest
import torch

from inputs import workloads as wl
from oracle import backward, occult_ref, routing
from paper_2505_13345_amd.layer import OccultLayer
from tests.helpers import f32_rel_error, require_gpu, say, to_dev

pytestmark = pytest.mark.gpu

CASES = [
    # E, D, k, T, d, dtype, placement
    (16, 4, 4, 211, 128, "f32", "random"),
    (16, 4, 4, 256, 128, "bf16", "contig"),
    (60, 4, 4, 128, 2048, "bf16", "contig"),
    (64, 8, 8, 1500, 2048, "bf16", "random"),
    (64, 16, 6, 1027, 2048, "bf16", "random"),
    (64, 64, 8, 300, 512, "bf16", "contig"),
    (64, 2, 32, 40, 256, "bf16", "random"),      # k = 32: every lookup lane busy, long merge lists
    (8, 2, 2, 77, 8, "bf16", "contig"),          # 16-byte rows
    (8, 2, 2, 77, 4096, "bf16", "contig"),       # 8 KiB rows
    (8, 2, 2, 33, 1032, "f32", "random"),        # ragged vector count per lane
    (8, 2, 2, 40, 8192, "bf16", "contig"),       # 16 KiB rows: two column chunks per row
    (8, 4, 2, 21, 4104, "f32", "random"),        # 16.4 KiB rows: three chunks, the last ragged
    (8, 2, 2, 1, 64, "bf16", "contig"),          # one token
]

GATES = {2: [.5, .5], 4: [.5, .25, .125, .125], 6: [.25, .25, .125, .125, .125, .125], 8: [.125] * 8,
         32: [.03125] * 32}


def _split_by_device(rows, trace):
    """Global EPD rows (position-major) -> per-device blocks in the device's local EPD order."""
    out, base = [], 0
    for b1 in trace.brim_1:
        n = int((b1 >= 0).sum())
        out.append(rows[base:base + n])
        base += n
    return out


@pytest.mark.parametrize("E,D,k,T,d,dtype,placement", CASES)
def test_backward_data_movement_bit_exact_on_exact_inputs(E, D, k, T, d, dtype, placement):
    say(f"backward exact case E={E} D={D} k={k} T={T} d={d} {dtype} {placement}")
    dev = require_gpu()
    lg = wl.random_logits(T, E, seed=T + d)
    pos = None if placement == "contig" else wl.random_placement(E, D, seed=E)
    pos_arr = wl.contiguous_placement(E, D) if pos is None else pos
    ids, _ = routing.route(lg, k, D, pos)
    # power-of-two gates and small-integer rows: gate * row and every sum below are exact in bf16
    # and f32 (|dy| <= 3, |epd_y| <= 3: dot products stay below 2^24; |epd_dx| <= 2: sums <= 64)
    w = np.tile(np.array(GATES[k]), (T, 1)).astype(np.float32)
    dy = wl.integer_valued_rows(T, d, seed=5, lo=-3, hi=3)
    epd_y = wl.integer_valued_rows(T * k, d, seed=6, lo=-3, hi=3)
    epd_dx = wl.integer_valued_rows(T * k, d, seed=7, lo=-2, hi=2)
    dx_sh = wl.integer_valued_rows(T, d, seed=8, lo=-2, hi=2)

    layer = OccultLayer(T, d, 64, E, 0, k, D, dtype, expert_pos=pos, with_ffn=False)
    ids_d = torch.from_numpy(ids).to(dev)
    layer.make_plan(ids_d, torch.from_numpy(w).to(dev))
    sfd_dy, epd_dy, dw = layer.combine_backward(to_dev(dy, dtype, dev), ids_d, to_dev(epd_y, dtype, dev))
    sfd_dx, dx = layer.dispatch_backward(to_dev(epd_dx, dtype, dev), to_dev(dx_sh, dtype, dev))
    torch.cuda.synchronize()

    trace = occult_ref.moe_forward(np.zeros((T, 1)), ids, w.astype(np.float64), pos_arr, D)
    L = occult_ref.placement_lists(pos_arr, D)
    g_sfd, g_out, g_w = backward.combine_backward(dy.astype(np.float64), _split_by_device(epd_y, trace), trace.brim_0,
                                                  trace.brim_1, trace.brim_w, trace.dev_count)
    n = trace.n_sfd
    assert np.array_equal(sfd_dy[:n].float().cpu().numpy(), g_sfd)
    assert np.array_equal(epd_dy.float().cpu().numpy(), np.concatenate(g_out))
    assert np.array_equal(dw.cpu().numpy(), backward.gate_grad_to_slots(g_w, ids, trace.brim_0, L, trace.dev_count))
    g_sfd_x, g_x = backward.dispatch_backward(_split_by_device(epd_dx, trace), trace.brim_0, trace.brim_1,
                                              trace.dev_count)
    assert np.array_equal(sfd_dx[:n].float().cpu().numpy(), g_sfd_x)
    assert np.array_equal(dx.float().cpu().numpy(), g_x + dx_sh)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_backward_data_movement_random_values(dtype):
    say(f"backward random case {dtype}")
    dev = require_gpu()
    E, D, k, T, d = 32, 4, 6, 900, 1024
    rng = np.random.default_rng(11)
    lg = wl.random_logits(T, E, seed=9)
    pos = wl.random_placement(E, D, seed=1)
    ids, w = routing.route(lg, k, D, pos)
    w32 = w.astype(np.float32)
    dy = rng.standard_normal((T, d)).astype(np.float32)
    epd_y = rng.standard_normal((T * k, d)).astype(np.float32)
    epd_dx = rng.standard_normal((T * k, d)).astype(np.float32)
    if dtype == "bf16":
        dy, epd_y, epd_dx = wl.round_to_bf16(dy), wl.round_to_bf16(epd_y), wl.round_to_bf16(epd_dx)
    layer = OccultLayer(T, d, 64, E, 0, k, D, dtype, expert_pos=pos, with_ffn=False)
    ids_d = torch.from_numpy(ids).to(dev)
    layer.make_plan(ids_d, torch.from_numpy(w32).to(dev))
    # optional outputs: ask for the gate gradient alone first, then for everything
    none_sfd, none_epd, dw_only = layer.combine_backward(to_dev(dy, dtype, dev), ids_d, to_dev(epd_y, dtype, dev),
                                                         want_sfd=False, want_epd=False)
    torch.cuda.synchronize()
    assert none_sfd is None and none_epd is None
    dw_first = dw_only.clone()
    sfd_dy, epd_dy, dw = layer.combine_backward(to_dev(dy, dtype, dev), ids_d, to_dev(epd_y, dtype, dev))
    sfd_dx, dx = layer.dispatch_backward(to_dev(epd_dx, dtype, dev))
    torch.cuda.synchronize()
    assert torch.equal(dw_first, dw)

    trace = occult_ref.moe_forward(np.zeros((T, 1)), ids, w32.astype(np.float64), pos, D)
    L = occult_ref.placement_lists(pos, D)
    g_sfd, g_out, g_w = backward.combine_backward(dy.astype(np.float64), _split_by_device(epd_y, trace), trace.brim_0,
                                                  trace.brim_1, trace.brim_w, trace.dev_count)
    n = trace.n_sfd
    assert np.array_equal(sfd_dy[:n].float().cpu().numpy(), g_sfd)     # a copy
    want_dw = backward.gate_grad_to_slots(g_w, ids, trace.brim_0, L, trace.dev_count)
    assert f32_rel_error(dw.cpu().numpy(), want_dw) <= 1e-5           # f32 dot products of d = 1024 terms
    rnd = (lambda a: wl.round_to_bf16(a.astype(np.float32)).astype(np.float64)) if dtype == "bf16" else None
    g_sfd_x, g_x = backward.dispatch_backward(_split_by_device(epd_dx, trace), trace.brim_0, trace.brim_1,
                                              trace.dev_count, sfd_round=rnd)
    got_out, got_sfd_x, got_x = (t.float().cpu().numpy() for t in (epd_dy, sfd_dx[:n], dx))
    if dtype == "bf16":
        # relative to max(|value|, rms): one bf16 rounding is 2^-9 = 2e-3 of the value; dx adds the roundings of
        # up to D = 4 payload rows, each up to ~2.5x the rms, to its own
        assert f32_rel_error(got_out, np.concatenate(g_out)) <= 4e-3
        assert f32_rel_error(got_sfd_x, g_sfd_x) <= 4e-3
        assert f32_rel_error(got_x, g_x) <= 3e-2
    else:
        assert f32_rel_error(got_out, np.concatenate(g_out)) <= 1e-5
        assert f32_rel_error(got_sfd_x, g_sfd_x) <= 1e-5
        assert f32_rel_error(got_x, g_x) <= 1e-5


def test_backward_full_size_properties():
    """The benchmark's prefill shape: sampled rows against the definition, through the plan tables
    (which the planner tests pin to the oracle)."""
    shape = wl.CONFIGS["prefill_bf16"]
    say(f"backward full size T={shape.T} d={shape.d} E={shape.E} k={shape.k} D={shape.D}")
    dev = require_gpu()
    T, d, k = shape.T, shape.d, shape.k
    wk = wl.make_workload(shape, with_experts=False)
    layer = OccultLayer(T, d, shape.f, shape.E, 0, k, shape.D, "bf16", with_ffn=False)   # contiguous placement
    layer.route(torch.from_numpy(wk.logits).to(dev))
    layer.make_plan()
    g = torch.Generator(device=dev)
    g.manual_seed(3)
    dy = torch.randn((T, d), device=dev, generator=g).to(torch.bfloat16)
    epd_y = torch.randn((T * k, d), device=dev, generator=g).to(torch.bfloat16)
    sfd_dy, epd_dy, dw = layer.combine_backward(dy, epd_y=epd_y)
    sfd_dx, dx = layer.dispatch_backward(epd_y)
    torch.cuda.synchronize()
    tabs = layer.tables()
    n_sfd = int(tabs["dev_offset"][shape.D])
    sfd_token = tabs["sfd_token"][:n_sfd].long()
    assert torch.equal(sfd_dy[:n_sfd], dy[sfd_token])
    rng = np.random.default_rng(0)
    q = torch.from_numpy(rng.integers(0, T * k, 4096)).to(dev)
    tok = sfd_token[tabs["epd_sfd_row"].long()[q]]
    gate = tabs["epd_gate"][q]
    want = (gate[:, None] * dy[tok].float()).to(torch.bfloat16)
    assert torch.equal(epd_dy[q], want)
    # gate gradients: sum over a token's slots = <dy[t], sum of its k expert rows>; per slot via the expert's rows
    t_s = torch.from_numpy(rng.integers(0, T, 512)).to(dev)
    ids = layer.ids.long()
    pos = torch.arange(shape.E, device=dev)
    G = shape.E // shape.D
    exp_off = tabs["exp_offset"].long()
    for s in range(k):
        P = pos[ids[t_s, s]]
        r = tabs["tok_sfd_row"].long()[t_s, P // G]
        lists = tabs["sfd_epd_rows"].long()[r]                       # [n, M1]
        hit = (lists >= exp_off[P][:, None]) & (lists < exp_off[P + 1][:, None])
        assert bool((hit.sum(dim=1) == 1).all())
        qs = (lists * hit).sum(dim=1)
        want_dw = (dy[t_s].double() * epd_y[qs].double()).sum(dim=1)
        assert f32_rel_error(dw[t_s, s].cpu().numpy(), want_dw.cpu().numpy()) <= 1e-5
    # dispatch backward: a token's dx is the sum of its k rows (two roundings on the way)
    rows = []
    for s in range(k):
        P = pos[ids[t_s, s]]
        r = tabs["tok_sfd_row"].long()[t_s, P // G]
        lists = tabs["sfd_epd_rows"].long()[r]
        hit = (lists >= exp_off[P][:, None]) & (lists < exp_off[P + 1][:, None])
        rows.append((lists * hit).sum(dim=1))
    want_dx = sum(epd_y[qs].double() for qs in rows)
    # payload rows rounded to bf16, then their sum: a few 2^-9 relative roundings of values around the rms
    assert f32_rel_error(dx[t_s].float().cpu().numpy(), want_dx.cpu().numpy()) <= 3e-2


ROUTE_CASES = [
    # T, E, k, D, n_d, mode, renorm
    (300, 8, 2, 2, 0, 1, 1),
    (1000, 60, 4, 4, 0, 1, 1),
    (1000, 60, 4, 4, 2, 1, 0),
    (777, 64, 8, 8, 2, 2, 1),
    (129, 256, 32, 64, 0, 1, 1),
    (129, 200, 7, 8, 0, 1, 0),
    (1, 16, 16, 4, 0, 1, 1),     # every expert selected: renormalised weights are the softmax itself
]


@pytest.mark.parametrize("T,E,k,D,n_d,mode,renorm", ROUTE_CASES)
def test_route_backward_against_oracle(T, E, k, D, n_d, mode, renorm):
    say(f"route backward case T={T} E={E} k={k} D={D} n_d={n_d} mode={mode} renorm={renorm}")
    dev = require_gpu()
    lg = wl.random_logits(T, E, seed=T + E, scale=2.0)
    ids, _ = routing.route(lg, k, D, None, n_d=n_d, prune_mode=mode, renorm=renorm)
    dw = np.random.default_rng(T).standard_normal((T, k)).astype(np.float32)
    layer = OccultLayer(T, 64, 64, E, 0, k, D, "bf16", n_d=n_d, prune_mode=mode, renorm=renorm, with_ffn=False)
    dlogits = torch.full((T, E), 7.0, dtype=torch.float32, device=dev)
    layer.route_backward(torch.from_numpy(lg).to(dev), torch.from_numpy(dw).to(dev), dlogits,
                         ids=torch.from_numpy(ids).to(dev))
    torch.cuda.synchronize()
    want = backward.route_backward(lg, ids, dw.astype(np.float64), renorm)
    assert f32_rel_error(dlogits.cpu().numpy(), want) <= 1e-5


def test_backward_empty_batch_and_argument_checks():
    from paper_2505_13345_amd import binding as B
    dev = require_gpu()
    layer = OccultLayer(0, 64, 64, 8, 0, 2, 2, "bf16", with_ffn=False)
    layer.make_plan()
    B.occult_combine_backward(layer.cfg, layer.plan, None, None, None, None, None, None)
    B.occult_dispatch_backward(layer.cfg, layer.plan, None, None, None, None)
    B.occult_route_backward(layer.cfg, None, None, None, None)
    layer = OccultLayer(4, 64, 64, 8, 0, 2, 2, "bf16", with_ffn=False)
    dy = torch.zeros((4, 64), dtype=torch.bfloat16, device=dev)
    dw = torch.zeros((4, 2), dtype=torch.float32, device=dev)
    with pytest.raises(B.OccultError) as e:
        B.occult_combine_backward(layer.cfg, layer.plan, layer.ids, dy, None, None, None, dw)   # dw needs epd_y
    assert e.value.code == -4
    with pytest.raises(B.OccultError) as e:
        B.occult_dispatch_backward(layer.cfg, layer.plan, None, dy, None, dy)
    assert e.value.code == -4
    torch.cuda.synchronize()
