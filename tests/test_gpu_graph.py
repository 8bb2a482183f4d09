"""The hot path under HIP graph capture: every call is asynchronous on the caller's stream,
allocates nothing and never synchronises, so one step can be captured once and replayed.  Each
replay is checked bit for bit against the eager result on the same inputs, with eager work and
synchronisations between the replays and the inputs changed in place from one replay to the next."""
import numpy as np
import pytest
import torch

from inputs import workloads as wl
from paper_2505_13345_amd import binding as B
from paper_2505_13345_amd.layer import OccultLayer
from tests.helpers import require_gpu, say, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,T,d,f,E,S,k,D", [
    ("decode_like", 96, 256, 192, 16, 2, 4, 4),      # weight-streaming + small-tile kernels, split-K scratch
    ("prefill_like", 1300, 256, 128, 4, 0, 2, 2),    # persistent 256-row tiles
])
def test_step_replays_from_a_graph(name, T, d, f, E, S, k, D):
    say(f"graph capture {name}")
    dev = require_gpu()
    shape = wl.LayerShape(name, T=T, d=d, f=f, E=E, S=S, k=k, D=D, dtype="bf16", components=4)
    wks = [wl.make_workload(shape, seed=s) for s in (5, 6)]
    layer = OccultLayer(T, d, f, E, S, k, D, "bf16")
    logits = torch.zeros((T, E), dtype=torch.float32, device=dev)
    x = torch.zeros((T, d), dtype=torch.bfloat16, device=dev)
    wg, wu, wd = (to_dev(a, "bf16", dev) for a in (wks[0].w_gate, wks[0].w_up, wks[0].w_down))
    C = torch.zeros((E, E), dtype=torch.int32, device=dev)

    def step():
        layer.forward(logits, x, wg, wu, wd)
        B.occult_coactivation(layer.cfg, layer.ids, C, False)

    def load(wk):
        logits.copy_(torch.from_numpy(wk.logits))
        x.copy_(torch.from_numpy(wk.x).to(torch.bfloat16))

    load(wks[0])
    step()                                   # warm-up outside capture (first-use host queries)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for rep, wk in enumerate([wks[0], wks[1], wks[0], wks[1]]):
        load(wk)
        step()
        torch.cuda.synchronize()
        ref = (layer.y.clone(), layer.ids.clone(), layer.sfd_y.clone(), C.clone(), layer.stats().n_sfd)
        for t in (layer.y, layer.sfd_y, layer.sfd_x, layer.epd_y, layer.epd_h):
            t.fill_(3.0)                     # eager work between replays; stale outputs would show
        layer.ids.zero_()
        C.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        n = ref[4]
        assert layer.stats().n_sfd == n
        assert torch.equal(layer.ids, ref[1]), f"replay {rep}: ids differ"
        assert torch.equal(layer.y, ref[0]), f"replay {rep}: y differs"
        assert torch.equal(layer.sfd_y[:n], ref[2][:n]), f"replay {rep}: sfd_y differs"
        assert torch.equal(C, ref[3]), f"replay {rep}: co-activation counts differ"


def test_training_step_replays_from_a_graph():
    """Forward with kept pre-activations and the whole backward pass, captured once and replayed."""
    say("graph capture training step")
    dev = require_gpu()
    T, d, f, E, S, k, D = 700, 256, 192, 8, 1, 2, 4
    shape = wl.LayerShape("train_like", T=T, d=d, f=f, E=E, S=S, k=k, D=D, dtype="bf16", components=4)
    wks = [wl.make_workload(shape, seed=s) for s in (5, 6)]
    layer = OccultLayer(T, d, f, E, S, k, D, "bf16")
    logits = torch.zeros((T, E), dtype=torch.float32, device=dev)
    x = torch.zeros((T, d), dtype=torch.bfloat16, device=dev)
    dy = torch.zeros((T, d), dtype=torch.bfloat16, device=dev)
    dlogits = torch.zeros((T, E), dtype=torch.float32, device=dev)
    wg, wu, wd = (to_dev(a, "bf16", dev) for a in (wks[0].w_gate, wks[0].w_up, wks[0].w_down))
    out = {}

    def step():
        layer.forward(logits, x, wg, wu, wd, train=True)
        layer.transpose_weights(wg, wu, wd)
        out["dx"], out["dw"] = layer.backward_input(x, wg, wu, dy)
        out["grads"] = layer.expert_ffn_backward_weights(x, dy)
        layer.route_backward(logits, out["dw"], dlogits)

    def load(wk, seed):
        logits.copy_(torch.from_numpy(wk.logits))
        x.copy_(torch.from_numpy(wk.x).to(torch.bfloat16))
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        dy.copy_(torch.randn((T, d), device=dev, generator=g).to(torch.bfloat16))

    load(wks[0], 0)
    step()                                   # warm-up outside capture: allocates the layer's backward buffers
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for rep, (wk, seed) in enumerate([(wks[0], 0), (wks[1], 1), (wks[0], 2)]):
        load(wk, seed)
        step()
        torch.cuda.synchronize()
        watched = [layer.y, out["dx"], out["dw"], dlogits, *out["grads"]]
        ref = [t.clone() for t in watched]
        for t in watched + [layer.epd_gu, layer.epd_dx, layer.epd_dy]:
            t.fill_(3.0)                     # eager work between replays; stale outputs would show
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (t, r) in enumerate(zip(watched, ref)):
            assert torch.equal(t, r), f"replay {rep}: output {i} differs"
