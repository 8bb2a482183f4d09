"""occult_plan_static (the planner with its scratch in a device array of the library: for callers that cannot
allocate) against occult_plan, through the C ABI: every plan table bit for bit, on two calls in a row, the
second on a smaller batch with another expert and device count (the shared array then still holds the first
call's counts)."""
import numpy as np
import pytest
import torch

from inputs import workloads as wl
from oracle import routing
from paper_2505_13345_amd import binding as B
from tests.helpers import require_gpu, say

pytestmark = pytest.mark.gpu


def _plan_tables(cfg, plan_mem, T, E, D, k):
    """Copies of every table of the bound plan block, by name."""
    plan = B.occult_plan_bind(cfg, plan_mem)
    base = plan_mem.data_ptr()
    n_sfd_max, m1 = T * min(k, D), min(k, E // D)
    sizes = dict(tok_devmask=T * 8, dev_count=D * 4, dev_offset=(D + 1) * 4, tok_sfd_row=T * D * 4, sfd_token=n_sfd_max * 4,
                 exp_count=E * 4, exp_offset=(E + 1) * 4, pos_expert=E * 4, epd_sfd_row=T * k * 4, epd_gate=T * k * 4,
                 sfd_epd_rows=n_sfd_max * m1 * 4, counters=64)
    return plan, {n: (getattr(plan, n) - base, sz) for n, sz in sizes.items()}


def _run_both(T, E, D, k, seed, placement):
    dev = require_gpu()
    lg = wl.random_logits(T, E, seed=seed, scale=1.5)
    pos = None if placement == "contig" else wl.random_placement(E, D, seed=seed)
    ids, w = routing.route(lg, k, D, pos)
    ids_d = torch.from_numpy(ids).to(dev)
    w_d = torch.from_numpy(w.astype(np.float32)).to(dev)
    pos_d = None if pos is None else torch.from_numpy(pos).to(dev)
    cfg = B.make_cfg(T, 64, 64, E, 0, k, D, "bf16", expert_pos=pos_d)
    plan_bytes, ws_bytes = B.occult_plan_sizes(cfg)
    assert ws_bytes <= 4 << 20
    mem_a = torch.full((plan_bytes,), 0x5A, dtype=torch.uint8, device=dev)
    mem_b = torch.full((plan_bytes,), 0xA5, dtype=torch.uint8, device=dev)
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=dev)
    plan_a, spans = _plan_tables(cfg, mem_a, T, E, D, k)
    plan_b, _ = _plan_tables(cfg, mem_b, T, E, D, k)
    B.occult_plan(cfg, ids_d, w_d, plan_a, ws)
    B.occult_plan_static(cfg, ids_d, w_d, plan_b)
    torch.cuda.synchronize()
    n_sfd = int(mem_a[spans["dev_offset"][0]:spans["dev_offset"][0] + (D + 1) * 4].view(torch.int32)[D].item())
    assert n_sfd > 0
    for name, (off, sz) in spans.items():
        if name == "sfd_token":
            sz = n_sfd * 4                          # rows past N_sfd are not written by either call
        elif name == "sfd_epd_rows":
            sz = n_sfd * min(k, E // D) * 4
        assert torch.equal(mem_a[off:off + sz], mem_b[off:off + sz]), f"{name} differs (T={T} E={E} D={D} k={k})"
    return n_sfd


def test_plan_static_equals_plan_on_two_calls_in_a_row():
    say("occult_plan_static: first call, T=5000 E=64 D=8 k=8")
    n1 = _run_both(5000, 64, 8, 8, seed=1, placement="random")
    say("occult_plan_static: second call on a smaller batch, T=777 E=60 D=4 k=4")
    n2 = _run_both(777, 60, 4, 4, seed=2, placement="contig")
    say("occult_plan_static: third call, one partial block, T=19 E=16 D=16 k=3")
    n3 = _run_both(19, 16, 16, 3, seed=3, placement="random")
    assert n1 > n2 > n3


def test_plan_static_empty_batch_and_size_limit():
    dev = require_gpu()
    cfg = B.make_cfg(0, 64, 64, 16, 0, 4, 4, "bf16")
    plan_bytes, _ = B.occult_plan_sizes(cfg)
    mem = torch.full((plan_bytes,), 0x77, dtype=torch.uint8, device=dev)
    plan = B.occult_plan_bind(cfg, mem)
    B.occult_plan_static(cfg, None, None, plan)
    torch.cuda.synchronize()
    st = B.occult_plan_stats(cfg, plan)
    assert st.n_sfd == 0 and st.n_epd == 0
    # a layer whose scratch exceeds the built-in buffer is refused before anything is launched
    big = B.make_cfg(20_000_000, 64, 64, 256, 0, 1, 64, "bf16")
    with pytest.raises(B.OccultError) as e:
        B.occult_plan_static(big, None, None, plan)
    assert e.value.code == -5
