"""Test scaffolding shared by the GPU parity tests: move a seeded workload to the GPU, expand the
library's compact plan tables into the paper's dense re-index matrices, error metrics."""
from __future__ import annotations

import numpy as np
import torch


def require_gpu():
    assert torch.cuda.is_available(), "GPU tests need a HIP device"
    return torch.device("cuda:0")


def to_dev(a: np.ndarray, dtype: str, device):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(device)
    return t.to(torch.bfloat16) if dtype == "bf16" else t.to(torch.float32)


def say(msg: str) -> None:
    print(msg, flush=True)


def expand_plan(tabs: dict, T: int, E: int, D: int, k: int):
    """GPU tables (torch) -> numpy dict with BRIM_0 [D,T] and per-device BRIM_1 / brim_w."""
    G = E // D
    t = {n: v.cpu().numpy() for n, v in tabs.items()}
    n_sfd = int(t["dev_offset"][D])
    brim_0 = t["tok_sfd_row"].T.astype(np.int64)
    brim_1, brim_w = [], []
    epd_sfd = t["epd_sfd_row"]
    gate = t["epd_gate"]
    for j in range(D):
        lo, hi = int(t["dev_offset"][j]), int(t["dev_offset"][j + 1])
        b1 = np.full((G, hi - lo), -1, dtype=np.int64)
        bw = np.zeros((G, hi - lo), dtype=np.float64)
        base = int(t["exp_offset"][j * G])
        for s in range(G):
            q0, q1 = int(t["exp_offset"][j * G + s]), int(t["exp_offset"][j * G + s + 1])
            rows = epd_sfd[q0:q1].astype(np.int64)
            assert np.all((rows >= lo) & (rows < hi)), "EPD row points outside its device segment"
            b1[s, rows - lo] = np.arange(q0, q1) - base
            bw[s, rows - lo] = gate[q0:q1]
        brim_1.append(b1)
        brim_w.append(bw)
    return dict(t, n_sfd=n_sfd, brim_0=brim_0, brim_1=brim_1, brim_w=brim_w)


def check_plan_against_trace(exp: dict, trace, ids: np.ndarray, w: np.ndarray, expert_pos, T, E, D, k):
    """Bit-exact comparison of the expanded GPU plan with the oracle's BRIMs and counters."""
    G = E // D
    assert exp["n_sfd"] == trace.n_sfd
    assert np.array_equal(exp["dev_count"], trace.dev_count)
    assert np.array_equal(exp["dev_offset"], np.concatenate([[0], np.cumsum(trace.dev_count)]))
    assert np.array_equal(exp["brim_0"], trace.brim_0)
    for j in range(D):
        assert np.array_equal(exp["brim_1"][j], trace.brim_1[j]), f"BRIM_1 of device {j}"
        # gates: the oracle carries float64 gates, the plan copies the float32 ones it was given
        assert np.array_equal(exp["brim_w"][j].astype(np.float32), trace.brim_w[j].astype(np.float32))
    # sfd_token: token of every SFD row
    sfd_token = np.full(trace.n_sfd, -1, dtype=np.int64)
    for j in range(D):
        present = trace.brim_0[j] >= 0
        sfd_token[trace.brim_0[j][present]] = np.nonzero(present)[0]
    assert np.array_equal(exp["sfd_token"][:trace.n_sfd], sfd_token)
    # expert counts by placement position, pos_expert inverse, device masks
    pos = np.arange(E) if expert_pos is None else np.asarray(expert_pos)
    cnt = np.bincount(pos[ids.reshape(-1)], minlength=E)
    assert np.array_equal(exp["exp_count"], cnt)
    assert np.array_equal(exp["exp_offset"], np.concatenate([[0], np.cumsum(cnt)]))
    inv = np.empty(E, dtype=np.int64)
    inv[pos] = np.arange(E)
    assert np.array_equal(exp["pos_expert"], inv)
    mask = np.zeros(T, dtype=np.uint64)
    for s in range(k):
        mask |= np.uint64(1) << (pos[ids[:, s]] // G).astype(np.uint64)
    assert np.array_equal(exp["tok_devmask"].view(np.uint64), mask)
    # merge lists: EPD rows of each SFD row, slot-ascending, -1 padded
    m1 = min(k, G)
    want = np.full((trace.n_sfd, m1), -1, dtype=np.int64)
    fill = np.zeros(trace.n_sfd, dtype=np.int64)
    off = exp["dev_offset"]
    for j in range(D):
        base = int(exp["exp_offset"][j * G])
        b1 = trace.brim_1[j]
        for s in range(G):
            cols = np.nonzero(b1[s] >= 0)[0]
            rows = cols + int(off[j])
            want[rows, fill[rows]] = b1[s][cols] + base
            fill[rows] += 1
    assert np.array_equal(exp["sfd_epd_rows"][:trace.n_sfd], want)
    c = exp["counters"]
    assert c[0] == trace.n_sfd and c[1] == T * k and c[2] == T * k
    assert c[3] == (trace.dev_count.max() if D else 0) and c[4] == cnt.max()


def bf16_errors(got: np.ndarray, want: np.ndarray):
    diff = np.abs(got.astype(np.float64) - want.astype(np.float64))
    return float(diff.max()), float(diff.mean())


def f32_rel_error(got: np.ndarray, want: np.ndarray):
    """max |g - o| / max(|o|, rms(o)): element-wise relative error with the scale floored at the
    output's rms, so that entries near zero do not blow the ratio up."""
    want = want.astype(np.float64)
    rms = float(np.sqrt(np.mean(want ** 2)))
    den = np.maximum(np.abs(want), rms)
    return float((np.abs(got.astype(np.float64) - want) / den).max())


# ---- bars derived from the storage type ------------------------------------------------------------
# bfloat16 keeps 8 significant bits: rounding to nearest moves a value by at most half a step of 2^-7
# relative to its leading power of two, i.e. by at most 2^-8 of the value itself.
BF16_U = 2.0 ** -8


def chain_mean_bar(n_roundings: int) -> float:
    """Upper bound on (mean |error|) / rms of a result that passed through `n_roundings` stored bf16
    tensors: each rounding adds an independent relative error of at most BF16_U, uniform inside its
    step, hence of rms <= BF16_U / sqrt(3) of the value; independent errors add in quadrature, sums of
    such values keep the relative figure, and a mean absolute value never exceeds the rms."""
    return float(np.sqrt(n_roundings) * BF16_U / np.sqrt(3.0))


def assert_one_rounding(got: np.ndarray, want: np.ndarray, what: str) -> None:
    """`got` is `want` (float64, from the same stored operands) accumulated in f32 and rounded once to bf16:
    every element within one rounding (BF16_U of its value) plus the f32 accumulation and fast-math error
    (2e-5 of the tensor's rms: f32 sums of up to a few thousand products, hardware exp and reciprocal)."""
    want = want.astype(np.float64)
    rms = float(np.sqrt(np.mean(want ** 2)))
    excess = np.abs(got.astype(np.float64) - want) - (BF16_U * (1 + 2.0 ** -10) * np.abs(want) + 2e-5 * rms)
    worst = float(excess.max())
    assert worst <= 0.0, f"{what}: an element is {worst:.3e} beyond one bf16 rounding (rms {rms:.3e})"


_workloads = {}


def cached_workload(shape):
    """Workloads of the large configurations are drawn once per test session (the pruned prefill
    configuration reads the same tensors as the unpruned one: same seed, same draw order)."""
    from inputs import workloads as wl
    key = (shape.T, shape.d, shape.f, shape.E, shape.S, shape.dtype, shape.components)
    if key not in _workloads:
        say(f"{shape.name}: generating")
        _workloads.clear()            # one large workload at a time
        _workloads[key] = wl.make_workload(shape)
    return _workloads[key]
