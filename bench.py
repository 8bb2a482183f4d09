#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline] [--graph]

One step = one pass of the whole hot path over one batch of synthetic input already resident in
HBM: occult_route -> occult_plan -> occult_dispatch -> occult_expert_ffn -> occult_combine ->
occult_coactivation, enqueued back to back on one stream with no host synchronisation (with
--graph: captured once into a HIP graph and replayed per step).
Prints ONE JSON line.  `value` is tokens per second of the whole step (all six calls).  Every timed
step also records HIP events on the launching stream around dispatch, the two products of the
expert call and combine: `timed_region_ms`, the dispatch+FFN+combine rate and the roofline
fractions of those kernels come from these events; `calls_ms` holds every call timed again in
separate passes after the timed region.  The simulated exchange bytes per token and the paper's
collaboration statistics ride along in the same line.

The default workload is the prefill-shaped layer (T = 2**14 tokens, E = 64, k = 8: the shape of
the paper's Table 1 measurement, sharded over 8 simulated devices).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0    # MI355X dense bf16 MFMA, published

COPY_PROBE_ROW = "copy probe"


def measured_traffic(workload, kernels):
    """HBM bytes per launch of `kernels` (summed) from profiles/<workload>_hbm_traffic.txt, the summary of
    two rocprofv3 --pmc runs of this script (FETCH_SIZE, then WRITE_SIZE; raw counter values per dispatch).
    The same runs hold a copy kernel of known size (--copy-probe-mib N: reads N MiB, writes N MiB); its row
    fixes what one unit of each counter is worth in bytes.  None if the file, the probe row or a kernel's
    row is missing."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    rows, probe_mib = {}, None
    for line in open(path):
        if line.startswith("#"):
            if "--copy-probe-mib" in line:
                probe_mib = float(line.split("--copy-probe-mib")[1].split()[0])
            continue
        cells = [c.strip() for c in line.split("|")]
        if len(cells) >= 5:
            rows[cells[0]] = (float(cells[2]), float(cells[4]))      # raw FETCH_SIZE, raw WRITE_SIZE
    probe = next((v for n, v in rows.items() if n.startswith(COPY_PROBE_ROW)), None)
    if probe is None or probe_mib is None or probe[0] <= 0 or probe[1] <= 0:
        return None
    bytes_per_fetch_unit = probe_mib * (1 << 20) / probe[0]
    bytes_per_write_unit = probe_mib * (1 << 20) / probe[1]
    total = 0.0
    for k in kernels:
        if k not in rows:
            return None
        total += rows[k][0] * bytes_per_fetch_unit + rows[k][1] * bytes_per_write_unit
    return total


def _event_time_ms(fn, reps):
    import torch
    start = torch.cuda.Event(enable_timing=True)
    end = torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    start.record()
    for _ in range(reps):
        fn()
    end.record()
    torch.cuda.synchronize()
    return start.elapsed_time(end) / reps


def cpu_baseline(wk, shape, sample_tokens):
    """The oracle as it stands (float64, numpy/BLAS) on a bounded sample of the same workload:
    routing, then the method's own path (BRIM matrices, dispatch, per-device expert FFN, two-stage
    combine) and the textbook layer it must equal."""
    import numpy as np
    from inputs import workloads as wl
    from oracle import moe_std, occult_ref, routing
    n = min(sample_tokens, shape.T)
    tokens = np.arange(n)
    pos = wl.contiguous_placement(shape.E, shape.D)
    t0 = time.perf_counter()
    ids, w = routing.route(wk.logits[:n], shape.k, shape.D, None, shape.n_d, shape.prune_mode, shape.renorm)
    occult_ref.moe_forward(wk.x[:n], ids, w, pos, shape.D, wk.w_gate, wk.w_up, wk.w_down, shape.S)
    t_occ = time.perf_counter() - t0
    t0 = time.perf_counter()
    moe_std.moe_layer(wk.x[:n], ids, w, wk.w_gate, wk.w_up, wk.w_down, shape.E, shape.S, tokens=tokens)
    t_std = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    return {"value": n / t_occ, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n} tokens of the workload: oracle routing + deduplicated layer (BRIMs, dispatch, "
                      f"expert FFN, two-stage combine; float64, numpy BLAS) {t_occ:.1f} s -> value; "
                      f"textbook layer on the same tokens {t_std:.1f} s ({n / t_std:.0f} tokens/s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="prefill_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="replay one captured HIP graph per step instead of launching every call from the host "
                         "(measured: no faster on this runtime, 0.264 vs 0.252 ms on the decode workload)")
    ap.add_argument("--no-standard", action="store_true",
                    help="skip the comparison run with one simulated device per expert (standard dispatch)")
    ap.add_argument("--placement", action="store_true",
                    help="also run the layer with the greedy collaboration-aware placement of this batch's co-activation "
                         "counts (always done for the large workload)")
    ap.add_argument("--no-pack", action="store_true",
                    help="decode-shaped workloads: read the weights in the caller's layout instead of the repacked copy")
    ap.add_argument("--no-backward", action="store_true",
                    help="skip timing the backward calls (occult_combine_backward, occult_expert_ffn_backward, ...)")
    ap.add_argument("--merge-atomic", action="store_true",
                    help="also time occult_combine_atomic (the paper's atomic first-stage merge: f32 and packed bf16 atomics) "
                         "beside occult_combine")
    ap.add_argument("--gemm-context", action="store_true",
                    help="bf16 workloads: also time the two expert products on all-zero operands (the clock under matrix "
                         "load is power-limited, so operand values change the rate) and the vendor library's dense "
                         "bf16 GEMMs of the same row count and shapes (torch.matmul) on values of the workload's scale")
    ap.add_argument("--cpu-sample", type=int, default=16384)
    ap.add_argument("--call-reps", type=int, default=10)
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run an elementwise copy kernel over this many MiB (reads N, writes N bytes): "
                         "the known-size reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is one GPU's share of the layer; only --gpus 1 is supported "
              "(devices of expert parallelism are simulated as expert groups on one GPU).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from inputs import workloads as wl
    from paper_2505_13345_amd import binding as B
    from paper_2505_13345_amd.layer import OccultLayer

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    shape = wl.CONFIGS[args.workload]
    wk = wl.make_workload(shape)
    tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
    es = 2 if shape.dtype == "bf16" else 4
    layer = OccultLayer(shape.T, shape.d, shape.f, shape.E, shape.S, shape.k, shape.D, shape.dtype,
                        shape.n_d, shape.prune_mode, shape.renorm, None)
    logits = torch.from_numpy(wk.logits).to(dev)
    x = torch.from_numpy(wk.x).to(dev).to(tdt)
    wg, wu, wd = (torch.from_numpy(a).to(dev).to(tdt) for a in (wk.w_gate, wk.w_up, wk.w_down))
    C = torch.zeros((shape.E, shape.E), dtype=torch.int32, device=dev)
    w_router = torch.from_numpy(wk.w_router).to(dev).to(tdt)
    logits_gpu = torch.empty_like(logits)

    # few rows per expert (decode shape): the one-time repacked copy of the weights that the weight-streaming kernel
    # reads as contiguous streams (outside the timed region, like loading the weights)
    packed_weights = shape.dtype == "bf16" and shape.T * shape.k < 24 * shape.E and not args.no_pack
    if packed_weights:
        layer.pack_weights(wg, wu, wd)

    def step():
        layer.route(logits)
        layer.make_plan()
        layer.dispatch(x)
        layer.expert_ffn(x, wg, wu, wd)
        layer.combine()
        B.occult_coactivation(layer.cfg, layer.ids, C, False)

    if args.copy_probe_mib > 0:
        probe = torch.zeros(args.copy_probe_mib * (1 << 20) // 4, dtype=torch.float32, device=dev)
        for _ in range(3):
            probe_out = probe + 1.0          # one kernel: reads and writes copy_probe_mib MiB
        torch.cuda.synchronize()
        del probe, probe_out

    # --graph: the step is captured once into a HIP graph (the calls allocate nothing and never
    # synchronise) and replayed: one host launch per step instead of one per kernel.
    run_step = step
    if args.graph:
        step()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        run_step = graph.replay
    # Timed region.  With host launches every step also records HIP events on the launching stream around
    # dispatch, the two products of the expert call (issued as its two phases) and combine, so the per-kernel
    # durations below come from the timed steps themselves.
    live = None
    # decode-shaped steps (a few hundred microseconds of small kernels) are timed without the per-step events:
    # five event records per step cost about a tenth of such a step
    if args.graph or shape.T * shape.k < 24 * shape.E:
        for _ in range(args.warmup):
            run_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run_step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    else:
        def step_marked(ev):
            layer.route(logits)
            layer.make_plan()
            ev[0].record()
            layer.dispatch(x)
            ev[1].record()
            layer.cfg.ffn_phase = 1
            layer.expert_ffn(x, wg, wu, wd)
            ev[2].record()
            layer.cfg.ffn_phase = 2
            layer.expert_ffn(x, wg, wu, wd)
            ev[3].record()
            layer.cfg.ffn_phase = 0
            layer.combine()
            ev[4].record()
            B.occult_coactivation(layer.cfg, layer.ids, C, False)

        new_marks = lambda: [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        spare = new_marks()
        for _ in range(args.warmup):
            step_marked(spare)
        marks = [new_marks() for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for ev in marks:
            step_marked(ev)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        span = lambda a, b: sum(ev[a].elapsed_time(ev[b]) for ev in marks) / len(marks)
        live = {"dispatch": span(0, 1), "ffn_gemm1_swiglu": span(1, 2), "ffn_gemm2_down": span(2, 3),
                "expert_ffn": span(1, 3), "combine": span(3, 4), "dispatch_ffn_combine": span(0, 4)}
    ms_per_step = dt / args.steps * 1e3
    st = layer.stats()

    # per-call times: HIP events on the stream the kernels are launched on (torch's current stream)
    r = args.call_reps
    calls = {
        "route": _event_time_ms(lambda: layer.route(logits), r),
        "plan": _event_time_ms(lambda: layer.make_plan(), r),
        "dispatch": _event_time_ms(lambda: layer.dispatch(x), r),
        "expert_ffn": _event_time_ms(lambda: layer.expert_ffn(x, wg, wu, wd), r),
        "combine": _event_time_ms(lambda: layer.combine(), r),
        "coactivation": _event_time_ms(lambda: B.occult_coactivation(layer.cfg, layer.ids, C, False), r),
        # not part of the step (which starts from the workload's scores): projection x W_r^T fused with routing
        "router_projection_and_route": _event_time_ms(lambda: layer.route_from_hidden(x, w_router, logits_gpu), r),
    }
    layer.route(logits)      # the step's own routing back in place for the phase timings below
    layer.make_plan()
    layer.cfg.ffn_phase = 1
    calls["ffn_gemm1_swiglu"] = _event_time_ms(lambda: layer.expert_ffn(x, wg, wu, wd), r)
    layer.cfg.ffn_phase = 2
    calls["ffn_gemm2_down"] = _event_time_ms(lambda: layer.expert_ffn(x, wg, wu, wd), r)
    layer.cfg.ffn_phase = 0

    T, d, f, k, S = shape.T, shape.d, shape.f, shape.k, shape.S
    row = d * es
    n_sfd, n_epd = st.n_sfd, T * k
    # algorithmic work per call
    flops1 = 4.0 * d * f * (n_epd + S * T)          # gate + up projections
    flops2 = 2.0 * d * f * (n_epd + S * T)          # down projection
    bytes_dispatch = (T + n_sfd) * row              # read each token once, write one row per device
    bytes_combine = (n_epd + n_sfd + T + (T if S else 0)) * row   # fused two-stage combine
    tf = lambda fl, ms: fl / (ms * 1e-3) / 1e12
    gbs = lambda by, ms: by / (ms * 1e-3) / 1e9
    bytes_router = (T * d + shape.E * d) * es + T * shape.E * 4 + T * k * 8
    m1 = min(k, shape.E // shape.D)
    bytes_route = T * (shape.E * 4 + k * 8)                       # scores in, ids and gates out
    bytes_plan = (T * k * 8                                        # ids and gates in
                  + T * 8 + T * shape.D * 4 + n_sfd * 4            # device masks, BRIM_0 rows, SFD -> token
                  + 2 * n_epd * 4 + n_sfd * m1 * 4)                # EPD -> SFD row, gates, merge lists
    rooflines = {
        "route": {"bound": "hbm", "achieved": gbs(bytes_route, calls["route"]), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                  "note": "launch- and latency-bound at this size"},
        "plan": {"bound": "hbm", "achieved": gbs(bytes_plan, calls["plan"]), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                 "note": "three dependent launches; latency-bound"},
        "router_projection_and_route": {"bound": "hbm", "achieved": gbs(bytes_router, calls["router_projection_and_route"]),
                                        "peak": PEAK_HBM_GBS, "unit": "GB/s"},
        "ffn_gemm1_swiglu": {"bound": "mfma", "achieved": tf(flops1, calls["ffn_gemm1_swiglu"]),
                             "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"},
        "ffn_gemm2_down": {"bound": "mfma", "achieved": tf(flops2, calls["ffn_gemm2_down"]),
                           "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"},
        "expert_ffn": {"bound": "mfma", "achieved": tf(flops1 + flops2, calls["expert_ffn"]),
                       "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"},
        "dispatch": {"bound": "hbm", "achieved": gbs(bytes_dispatch, calls["dispatch"]),
                     "peak": PEAK_HBM_GBS, "unit": "GB/s"},
        "combine": {"bound": "hbm", "achieved": gbs(bytes_combine, calls["combine"]),
                    "peak": PEAK_HBM_GBS, "unit": "GB/s"},
    }
    # few rows per expert (decode shape): the FFN streams every active expert's weights once, so
    # its roofline is HBM bandwidth on weight bytes (3*d*f elements per active or shared expert)
    weight_bound = T * k < 24 * shape.E
    if weight_bound:
        active = int((layer.tables()["exp_count"] > 0).sum().item()) + S
        rooflines["expert_ffn_weights"] = {"bound": "hbm", "achieved": gbs(active * 3.0 * d * f * es, calls["expert_ffn"]),
                                           "peak": PEAK_HBM_GBS, "unit": "GB/s", "active_experts": active}
    if live is not None:
        # the same figures from the events of the timed steps
        for n, work, unit in (("ffn_gemm1_swiglu", flops1, tf), ("ffn_gemm2_down", flops2, tf),
                              ("expert_ffn", flops1 + flops2, tf)):
            rooflines[n]["achieved_separate_pass"] = rooflines[n]["achieved"]
            rooflines[n]["achieved"] = unit(work, live[n])
        # the two short data-movement kernels keep the back-to-back figure: an event pair around a 80 - 190 us
        # kernel adds several microseconds of its own (rocprofv3's kernel durations sit between the two)
        for n, work in (("dispatch", bytes_dispatch), ("combine", bytes_combine)):
            rooflines[n]["achieved_timed_region"] = gbs(work, live[n])
        if weight_bound:
            rooflines["expert_ffn_weights"]["achieved"] = gbs(active * 3.0 * d * f * es, live["expert_ffn"])
    for v in rooflines.values():
        v["frac"] = v["achieved"] / v["peak"]
    if weight_bound:
        dom = dict(rooflines["expert_ffn_weights"])
        dom["kernel"] = "skinny::grouped_gemm_bf16 (weight streaming, both projections of occult_expert_ffn)"
        dom["traffic"] = measured_traffic(args.workload, [
            "occult::skinny::grouped_gemm_bf16<true, 2, true>", "occult::skinny::grouped_gemm_bf16<false, 2, true>",
            "occult::small::grouped_gemm_bf16<true>", "occult::small::grouped_gemm_bf16<false>",
            "occult::splitk_reduce_bf16"])
    else:
        dom = dict(rooflines["ffn_gemm1_swiglu"])
        dom["kernel"] = "t256::grouped_gemm_bf16<true, false, false> (gate/up projections of occult_expert_ffn)"
        dom["traffic"] = measured_traffic(args.workload, ["occult::t256::grouped_gemm_bf16<true, false, false>"])

    # backward pass (not part of the step, which is the paper's inference metric: reported beside it)
    backward = None
    if not args.no_backward:
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        dy = torch.randn((T, d), device=dev, generator=gen).to(tdt)
        dlogits = torch.empty_like(logits)
        layer.combine_backward(dy)
        bc = {
            "combine_backward": _event_time_ms(lambda: layer.combine_backward(dy), r),
            "combine_backward_rows_only": _event_time_ms(lambda: layer.combine_backward(dy, want_dw=False), r),
            "dispatch_backward": _event_time_ms(lambda: layer.dispatch_backward(layer.epd_dy), r),
            "route_backward": _event_time_ms(lambda: layer.route_backward(logits, layer.dw, dlogits), r),
        }
        bb = {
            # dispatch of dy (T rows in, N_sfd out) + scaled rows (T in, N_epd out) + gate gradients (N_epd in)
            "combine_backward": (2 * T + n_sfd + 2 * n_epd) * row,
            "combine_backward_rows_only": (2 * T + n_sfd + n_epd) * row,
            "dispatch_backward": (n_epd + n_sfd + T) * row,
            "route_backward": T * (2 * shape.E * 4 + k * 8),
        }
        # backward of the expert computation: input gradients (5 products of 2*d*f flops per row, the forward has 3)
        # and weight gradients (3 products)
        layer.transpose_weights(wg, wu, wd)
        layer.expert_ffn_backward(x, wg, wu, layer.epd_dy, dy)
        layer.expert_ffn_backward_weights(x, dy)
        bc["transpose_weights"] = _event_time_ms(lambda: layer.transpose_weights(wg, wu, wd), r)
        bc["expert_ffn_backward"] = _event_time_ms(lambda: layer.expert_ffn_backward(x, wg, wu, layer.epd_dy, dy), r)
        bc["expert_ffn_backward_weights"] = _event_time_ms(lambda: layer.expert_ffn_backward_weights(x, dy), r)
        # the alternative for a training step: the forward call keeps the pre-activations, the backward does not recompute
        bc["expert_ffn_train"] = _event_time_ms(lambda: layer.expert_ffn_train(x, wg, wu, wd), r)
        bc["expert_ffn_backward_kept"] = _event_time_ms(
            lambda: layer.expert_ffn_backward(x, wg, wu, layer.epd_dy, dy, gu_saved=True), r)
        rows_ffn = n_epd + S * T
        fb = {"expert_ffn_backward": 10.0 * d * f * rows_ffn, "expert_ffn_backward_weights": 6.0 * d * f * rows_ffn,
              "expert_ffn_train": 6.0 * d * f * rows_ffn, "expert_ffn_backward_kept": 6.0 * d * f * rows_ffn}
        bb["transpose_weights"] = 2.0 * 3 * (shape.E + S) * d * f * es
        bc["backward_total"] = (bc["combine_backward"] + bc["expert_ffn_backward"] + bc["expert_ffn_backward_weights"]
                                + bc["dispatch_backward"] + bc["route_backward"])
        # forward + backward of one training step with kept pre-activations, against recomputing them
        fwd_rest = calls["route"] + calls["plan"] + calls["dispatch"] + calls["combine"]
        bc["train_step_kept"] = (fwd_rest + bc["expert_ffn_train"] + bc["backward_total"] - bc["expert_ffn_backward"]
                                 + bc["expert_ffn_backward_kept"])
        bc["train_step_recompute"] = fwd_rest + calls["expert_ffn"] + bc["backward_total"]
        backward = {"calls_ms": bc,
                    "rooflines": {n: {"bound": "hbm", "achieved": gbs(bb[n], bc[n]), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                      "frac": gbs(bb[n], bc[n]) / PEAK_HBM_GBS} for n in bb}}
        for n in fb:
            backward["rooflines"][n] = {"bound": "mfma", "achieved": tf(fb[n], bc[n]), "peak": PEAK_BF16_TFLOPS,
                                        "unit": "TFLOP/s", "frac": tf(fb[n], bc[n]) / PEAK_BF16_TFLOPS}
        for n in ("sfd_dy", "epd_dy", "sfd_dx", "dx", "dw", "w_down_t", "w_gu_t", "epd_gu", "epd_dh", "epd_dx", "gu_shared",
                  "dh_shared", "dx_shared", "dw_gate", "dw_up", "dw_down"):
            setattr(layer, n, None)
        del dy, dlogits
        torch.cuda.empty_cache()

    dom["timing"] = ("HIP events around the kernel in each of the timed steps" if live is not None
                     else "HIP events around repeated calls, after the timed region")
    three = live["dispatch_ffn_combine"] if live is not None else calls["dispatch"] + calls["expert_ffn"] + calls["combine"]
    out = {
        # `value` is the whole step (all six calls); the dispatch+FFN+combine part of the same steps is
        # tokens_per_s_dispatch_ffn_combine
        "metric": "MoE-layer tokens/sec (whole step: route+plan+dispatch+FFN+combine+co-activation)",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "T": T, "d": d, "f": f, "E": shape.E, "S": S, "k": k,
                   "D": shape.D, "n_d": shape.n_d, "step": "route+plan+dispatch+expert_ffn+combine+coactivation",
                   "launch": "one HIP graph replay per step" if args.graph else "host launch per call",
                   "weights": "repacked once for the weight-streaming kernel (occult_pack_weights)" if packed_weights
                   else "caller's layout"},
        "roofline": dom,
        "calls_ms": calls,
        "timed_region_ms": live,
        "tokens_per_s_dispatch_ffn_combine": T / (three * 1e-3),
        "rooflines": rooflines,
        "exchange": {"c_t": st.c_t, "bytes_per_token_occult": st.bytes_occ / T,
                     "bytes_per_token_standard": st.bytes_std / T,
                     "saved_fraction": 1.0 - st.bytes_occ / st.bytes_std,
                     "meta_bytes_per_token": st.bytes_meta / T},
    }
    def collaboration(ids_dev, pos_host):
        """Sec. 3.2 statistics of a routing under a placement: co-activation counts on the GPU, averages on the host."""
        Cc = torch.zeros((shape.E, shape.E), dtype=torch.int32, device=dev)
        cfgc = B.make_cfg(T, d, f, shape.E, S, k, shape.D, shape.dtype, 0, 1, shape.renorm, None)
        B.occult_coactivation(cfgc, ids_dev, Cc, False)
        torch.cuda.synchronize()
        c_intra, c_inter, frac = B.occult_collaboration_stats(Cc.cpu().numpy(), shape.D, pos_host)
        off = ~np.eye(shape.D, dtype=bool)
        return {"intra_fraction": frac, "inter_fraction": 1.0 - frac, "c_intra_mean": float(c_intra.mean()),
                "c_inter_mean": float(c_inter[off].mean()) if shape.D > 1 else 0.0}

    out["collaboration"] = collaboration(layer.ids, None)
    if args.merge_atomic:
        # the paper's first-stage merge through atomic adds (Sec. 3.1) against the order-fixed fused combine
        modes = {"f32_atomics": 0, "packed_bf16_atomics": 1} if shape.dtype == "bf16" else {"f32_atomics": 0}
        am = {n: _event_time_ms(lambda m=m: layer.combine_atomic(mode=m), r) for n, m in modes.items()}
        out["atomic_merge"] = {"calls_ms": am, "combine_ms": calls["combine"],
                               "merged_rows": n_epd, "target_rows": n_sfd, "payload_bytes": n_epd * row,
                               "note": "clear + atomic merge + stage 2 (three kernels) against the fused order-fixed occult_combine"}
        layer.combine()
        layer.sfd_acc = None
        torch.cuda.empty_cache()
    if args.gemm_context and shape.dtype == "bf16":
        n_rows = n_epd + S * T

        def two_products(xx, a, b, c):
            layer.dispatch(xx)
            res = {}
            for ph, name, fl in ((1, "gemm1_swiglu", flops1), (2, "gemm2_down", flops2)):
                layer.cfg.ffn_phase = ph
                ms = _event_time_ms(lambda: layer.expert_ffn(xx, a, b, c), r)
                res[name] = {"ms": ms, "tflops": fl / ms / 1e9, "frac_of_peak": fl / ms / 1e9 / 2500.0}
            layer.cfg.ffn_phase = 0
            return res

        ctx = {"expert_gemm_workload_values": two_products(x, wg, wu, wd)}
        zx, zg, zd = torch.zeros_like(x), torch.zeros_like(wg), torch.zeros_like(wd)
        ctx["expert_gemm_zero_operands"] = two_products(zx, zg, zg, zd)
        del zx, zg, zd
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        lib = {}
        for name, kk, nn, fl in (("dense_gemm1_shape", d, 2 * f, flops1), ("dense_gemm2_shape", f, d, flops2)):
            pa = torch.randn(n_rows, kk, device=dev, generator=gen).to(tdt)
            pb = (torch.randn(nn, kk, device=dev, generator=gen) / kk ** 0.5).to(tdt)
            ms = _event_time_ms(lambda: torch.matmul(pa, pb.t()), r)
            lib[name] = {"m": n_rows, "n": nn, "k": kk, "ms": ms, "tflops": fl / ms / 1e9,
                         "frac_of_peak": fl / ms / 1e9 / 2500.0}
            del pa, pb
        ctx["vendor_library_dense_bf16"] = lib
        ctx["note"] = ("same row count and flops as the two expert products; the library GEMMs have no row gather, no "
                       "groups, no ragged tiles and no fused activation")
        out["gemm_context"] = ctx
        layer.dispatch(x)
        layer.expert_ffn(x, wg, wu, wd)
        torch.cuda.empty_cache()
    if backward is not None:
        out["backward"] = backward
    # The same layer with one simulated device per expert (D = E): the standard per-expert dispatch
    # the paper compares against (a token's row is replicated once per selected expert, C_T = k).
    if shape.E <= 64 and shape.n_d == 0 and not args.no_standard:
        del layer
        torch.cuda.empty_cache()
        std = OccultLayer(T, d, f, shape.E, S, k, shape.E, shape.dtype, 0, 1, shape.renorm, None)
        if packed_weights:
            std.pack_weights(wg, wu, wd)
        std.route(logits)
        std.make_plan()
        std.dispatch(x)
        std.expert_ffn(x, wg, wu, wd)
        sc = {
            "plan": _event_time_ms(lambda: std.make_plan(), r),
            "dispatch": _event_time_ms(lambda: std.dispatch(x), r),
            "expert_ffn": _event_time_ms(lambda: std.expert_ffn(x, wg, wu, wd), r),
            "combine": _event_time_ms(lambda: std.combine(), r),
        }
        sst = std.stats()
        s3 = sc["dispatch"] + sc["expert_ffn"] + sc["combine"]
        out["standard_per_expert_dispatch"] = {
            "c_t": sst.c_t, "calls_ms": sc, "tokens_per_s_dispatch_ffn_combine": T / (s3 * 1e-3),
            "bytes_per_token": sst.bytes_occ / T,
            "occult_speedup_dispatch_ffn_combine": s3 / three,
            "occult_speedup_dispatch_plus_combine": (sc["dispatch"] + sc["combine"]) / (calls["dispatch"] + calls["combine"]),
        }
        layer = std
    # Collaboration-aware placement (paper Sec. 3.2): the co-activation counts of this batch -> greedy placement on
    # the host -> the same layer with that placement, against the contiguous one above.
    if (args.workload == "large_bf16" or args.placement) and shape.E // shape.D >= 2 and shape.n_d == 0:
        C.zero_()
        ids_prof = torch.empty((T, k), dtype=torch.int32, device=dev)
        w_prof = torch.empty((T, k), dtype=torch.float32, device=dev)
        cfg0 = B.make_cfg(T, d, f, shape.E, S, k, shape.D, shape.dtype, 0, 1, shape.renorm, None)
        B.occult_route(cfg0, logits, ids_prof, w_prof)
        B.occult_coactivation(cfg0, ids_prof, C, False)
        torch.cuda.synchronize()
        _, pos = B.occult_placement_greedy(C.cpu().numpy(), shape.D)
        del layer
        torch.cuda.empty_cache()
        gr = OccultLayer(T, d, f, shape.E, S, k, shape.D, shape.dtype, 0, 1, shape.renorm, pos)
        if packed_weights:
            gr.pack_weights(wg, wu, wd)
        gr.route(logits)
        gr.make_plan()
        gr.dispatch(x)
        gr.expert_ffn(x, wg, wu, wd)
        gc = {
            "plan": _event_time_ms(lambda: gr.make_plan(), r),
            "dispatch": _event_time_ms(lambda: gr.dispatch(x), r),
            "expert_ffn": _event_time_ms(lambda: gr.expert_ffn(x, wg, wu, wd), r),
            "combine": _event_time_ms(lambda: gr.combine(), r),
        }
        gst = gr.stats()
        g3 = gc["dispatch"] + gc["expert_ffn"] + gc["combine"]
        out["greedy_placement"] = {
            "c_t": gst.c_t, "c_t_contiguous": st.c_t, "bytes_per_token": gst.bytes_occ / T,
            "bytes_per_token_contiguous": st.bytes_occ / T, "saved_fraction_vs_contiguous": 1.0 - gst.bytes_occ / st.bytes_occ,
            "calls_ms": gc, "tokens_per_s_dispatch_ffn_combine": T / (g3 * 1e-3),
            "speedup_dispatch_plus_combine": (calls["dispatch"] + calls["combine"]) / (gc["dispatch"] + gc["combine"]),
            "collaboration": collaboration(gr.ids, pos), "collaboration_contiguous": out["collaboration"],
        }
        layer = gr
    # Collaboration pruning (paper Sec. 3.3): the same layer without pruning, for the routing change, the bytes
    # and the difference of the outputs.
    if shape.n_d > 0:
        y_pruned = layer.y.float().clone() if getattr(layer, "y", None) is not None else None
        ids_pruned = layer.ids.clone()
        del layer
        torch.cuda.empty_cache()
        un = OccultLayer(T, d, f, shape.E, S, k, shape.D, shape.dtype, 0, 1, shape.renorm, None)
        y_un = un.forward(logits, x, wg, wu, wd).float()
        torch.cuda.synchronize()
        ust = un.stats()
        same_set = lambda a, b: (a.sort(dim=1).values == b.sort(dim=1).values).all(dim=1).float().mean().item()
        rel_l2 = lambda a, b: ((a - b).norm() / b.norm()).item()
        out["pruning"] = {
            "n_d": shape.n_d, "prune_mode": shape.prune_mode, "c_t": st.c_t, "c_t_unpruned": ust.c_t,
            "bytes_per_token": st.bytes_occ / T, "bytes_per_token_unpruned": ust.bytes_occ / T,
            "tokens_with_unchanged_experts": same_set(ids_pruned, un.ids),
            "output_rel_l2_diff_vs_unpruned": rel_l2(y_pruned, y_un),
            "collaboration_unpruned": collaboration(un.ids, None),
        }
        # the other device-choice rule of Sec. 3.3 (mode 2: walk the top-k in descending score until n_d devices are
        # met; mode 1: the n_d devices of highest summed gate score), same layer and inputs
        other = 2 if shape.prune_mode == 1 else 1
        alt = OccultLayer(T, d, f, shape.E, S, k, shape.D, shape.dtype, shape.n_d, other, shape.renorm, None)
        y_alt = alt.forward(logits, x, wg, wu, wd).float()
        torch.cuda.synchronize()
        ast = alt.stats()
        alt_ms = {"route": _event_time_ms(lambda: alt.route(logits), r), "dispatch": _event_time_ms(lambda: alt.dispatch(x), r),
                  "combine": _event_time_ms(lambda: alt.combine(), r)}
        out["pruning"][f"prune_mode_{other}"] = {
            "c_t": ast.c_t, "bytes_per_token": ast.bytes_occ / T,
            "tokens_with_unchanged_experts": same_set(alt.ids, un.ids),
            "tokens_with_same_experts_as_configured_mode": same_set(alt.ids, ids_pruned),
            "output_rel_l2_diff_vs_unpruned": rel_l2(y_alt, y_un),
            "calls_ms": alt_ms, "collaboration": collaboration(alt.ids, None),
        }
        del alt, y_alt
        layer = un
    if not args.no_cpu_baseline:
        del layer
        out["cpu_baseline"] = cpu_baseline(wk, shape, args.cpu_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
