"""GPU parity of occult_router: the router projection (paper Eq. 1) fused with routing.

The scores are a float32 product summed in the kernel's own fixed order, so they equal the
float64 oracle only within float32 accumulation error, and a selection decided by scores closer
than that may differ from one made on other float32 scores.  What is exact and checked bit for
bit: routing the kernel's own scores with the oracle gives the kernel's ids; against the routing
of the workload's scores every differing token must have a deciding margin below the score error."""
import numpy as np
import pytest
import torch

from inputs import workloads as wl
from oracle import routing
from paper_2505_13345_amd.layer import OccultLayer
from tests.helpers import require_gpu, say

pytestmark = pytest.mark.gpu


def _run(x, wr, E, D, k, dtype, n_d=0, mode=1, renorm=1, pos=None):
    dev = require_gpu()
    T, d = x.shape
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    layer = OccultLayer(T, d, 64, E, 0, k, D, dtype, n_d, mode, renorm, pos, with_ffn=False)
    logits = torch.full((T, E), float("nan"), dtype=torch.float32, device=dev)
    layer.route_from_hidden(torch.from_numpy(x).to(dev).to(tdt), torch.from_numpy(wr).to(dev).to(tdt), logits)
    torch.cuda.synchronize()
    return logits.cpu().numpy(), layer.ids.cpu().numpy(), layer.w.cpu().numpy()


def _check(x, wr, E, D, k, dtype, n_d=0, mode=1, renorm=1, pos=None):
    lg, ids, w = _run(x, wr, E, D, k, dtype, n_d, mode, renorm, pos)
    ref = routing.router_scores(x, wr)                      # float64, from the stored inputs
    rms = np.sqrt(np.mean(ref ** 2))
    err = np.max(np.abs(lg - ref))
    assert err <= 1e-5 * max(rms, 1e-30), (err, rms)      # float32 accumulation over d terms
    # routing of the kernel's own scores: exact
    ids_ref, w_ref = routing.route(lg, k, D, pos, n_d=n_d, prune_mode=mode, renorm=renorm)
    assert np.array_equal(ids, ids_ref)
    assert np.max(np.abs(w - w_ref) / w_ref) <= 1e-5
    return lg, ids, ref, err


ROUTER_CASES = [
    # T, d, E, D, k, n_d, mode
    (1, 128, 16, 4, 4, 0, 1),
    (33, 128, 16, 4, 4, 0, 1),
    (257, 256, 60, 4, 4, 0, 1),
    (1000, 512, 64, 8, 8, 2, 1),
    (515, 384, 64, 8, 8, 2, 2),
    (300, 256, 128, 8, 8, 0, 1),
    (200, 128, 256, 16, 8, 4, 1),
    (100, 2048, 8, 8, 2, 0, 1),
]


@pytest.mark.parametrize("T,d,E,D,k,n_d,mode", ROUTER_CASES)
def test_router_bf16_cases(T, d, E, D, k, n_d, mode):
    say(f"router case T={T} d={d} E={E} D={D} k={k} n_d={n_d} mode={mode}")
    rng = np.random.default_rng(T * 31 + E)
    x = wl.round_to_bf16(rng.standard_normal((T, d)).astype(np.float32))
    wr = wl.round_to_bf16((rng.standard_normal((E, d)) / np.sqrt(d)).astype(np.float32))
    pos = wl.random_placement(E, D, seed=E + D) if n_d else None
    _check(x, wr, E, D, k, "bf16", n_d, mode, 1, pos)


def test_router_exact_on_integer_inputs():
    """Small integers: every product and partial sum is exact in float32, so the scores equal the
    oracle's bit for bit whatever the summation order, and so does everything downstream."""
    say("router exact integers")
    rng = np.random.default_rng(3)
    T, d, E, D, k = 333, 256, 64, 8, 8
    x = rng.integers(-4, 5, (T, d)).astype(np.float32)
    wr = rng.integers(-3, 4, (E, d)).astype(np.float32)
    lg, ids, _ = _run(x, wr, E, D, k, "bf16")
    ref = routing.router_scores(x, wr)
    assert np.array_equal(lg.astype(np.float64), ref)
    ids_ref, _ = routing.route(ref.astype(np.float32), k, D)
    assert np.array_equal(ids, ids_ref)


@pytest.mark.parametrize("name", ["tiny_f32", "decode_bf16", "prefill_bf16", "prefill_pruned_bf16", "large_bf16"])
def test_router_at_config_sizes(name):
    shape = wl.CONFIGS[name]
    say(f"router config {name}")
    wk = wl.make_workload(shape, with_experts=False)
    pos = wl.contiguous_placement(shape.E, shape.D)
    lg, ids, ref, err = _check(wk.x, wk.w_router, shape.E, shape.D, shape.k, shape.dtype, shape.n_d,
                               shape.prune_mode, shape.renorm, pos)
    # audit against the routing of the workload's own float32 scores: tokens may differ only where the
    # scores that decide the selection are closer than the two products can disagree
    ids_w, _ = routing.route(wk.logits, shape.k, shape.D, pos, n_d=shape.n_d, prune_mode=shape.prune_mode,
                             renorm=shape.renorm)
    differ = np.any(ids != ids_w, axis=1)
    gap = np.max(np.abs(lg.astype(np.float64) - wk.logits))
    say(f"  score error vs float64 {err:.3g}; vs workload scores {gap:.3g}; {int(differ.sum())} of {shape.T} tokens "
        f"route differently")
    if shape.n_d == 0:
        margin = routing.selection_margin(ref, shape.k)
        assert np.all(margin[differ] <= 2 * gap + 2 * err)
    assert differ.mean() <= 1e-3


@pytest.mark.parametrize("seed", range(24))
def test_router_random_shapes(seed):
    """Seeded draws over T, d (multiples of 128 for bf16), any E, D, k and pruning setting."""
    rng = np.random.default_rng(7000 + seed)
    dtype = "f32" if seed % 4 == 3 else "bf16"
    E = int(rng.choice([2, 3, 5, 8, 16, 24, 60, 64, 100, 128, 200, 256]))
    D = int(rng.choice([j for j in range(1, 65) if E % j == 0]))
    k = int(rng.integers(1, min(E, 8) + 1))
    T = int(rng.choice([1, 31, 32, 33, 100, 257, 1000, 3001]))
    d = int(rng.choice([128, 256, 384, 1152, 4096])) if dtype == "bf16" else int(rng.choice([4, 37, 128, 500]))
    mode = int(rng.integers(1, 3))
    n_d = int(rng.integers(0, D + 1))
    if n_d and n_d * (E // D) < k:
        n_d = 0
    say(f"router draw {seed}: T={T} d={d} E={E} D={D} k={k} n_d={n_d} mode={mode} {dtype}")
    x = rng.standard_normal((T, d)).astype(np.float32)
    wr = (rng.standard_normal((E, d)) / np.sqrt(d)).astype(np.float32)
    if dtype == "bf16":
        x, wr = wl.round_to_bf16(x), wl.round_to_bf16(wr)
    pos = wl.random_placement(E, D, seed=seed) if seed % 2 else None
    _check(x, wr, E, D, k, dtype, n_d, mode, int(rng.integers(0, 2)), pos)
