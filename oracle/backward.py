"""CPU oracle: backward pass of the layer: its data movement (dispatch, row replication, two-stage
merge, combine), its SwiGLU experts and its routing weights.

TEST INFRASTRUCTURE ONLY (see oracle/routing.py for who may import this).

The paper trains through the layer (Introduction: its sparse matrix multiplication serves the
forward and the backward pass; Section 4, Training) but prints no backward algorithm.  Every step
of the forward data movement is linear in the hidden rows, so its backward is the transposed map
on the same re-index matrices (paper Section 3.1, Appendix A.2), written here as the forward's
loops with source and destination exchanged:

  forward "Combine"            x_ori[t] += x_sfd[BRIM_0[d, t]]       ->  g_sfd[BRIM_0[d, t]] = g_ori[t]
  forward merge into SFD rows  x_sfd[t] += w * out[BRIM_1[e, t]]     ->  g_out[BRIM_1[e, t]] = w * g_sfd[t]
                                                                          g_w[e, t] = <g_sfd[t], out[BRIM_1[e, t]]>
  forward SFD -> EPD gather    in[BRIM_1[e, t]] = x_sfd[t]           ->  g_sfd[t] += g_in[BRIM_1[e, t]]
  forward "Dispatch"           x_sfd[BRIM_0[d, t]] = x_ori[t]        ->  g_ori[t] += g_sfd[BRIM_0[d, t]]

so the gradient of combine is a dispatch of the output gradient, the gradient of dispatch is a
two-stage combine with unit weights, and both exchanges again carry one row per (token, device).
Readings (the paper is silent on all of them): the routing weight multiplies the expert's output
row (for a linear down projection the same as multiplying the intermediate, which is where the
forward oracle applies it); roundings of the forward pass are not differentiated; sums run over
local experts in slot order, then over devices in ascending order, as in the forward pass.

`expert_ffn_backward` is the chain rule through one SwiGLU expert (input and weight gradients);
`layer_backward` strings the pieces together for the whole layer, shared experts included.

`route_backward` is the gradient of the gate values of Eq. 1 with respect to the router scores:
Softmax over all E experts, the values at the k selected experts, optionally divided by their sum.
The selection itself is piecewise constant and contributes nothing.
Float arithmetic is float64.

Storage rounding (``storage=`` of `layer_backward`, `expert_ffn_backward`, `combine_backward`): the
paper keeps parameters and activations in bfloat16 (Section 4, Experimental Setup), so a bfloat16
implementation of this chain stores every tensor that travels between two products in that type.
Given ``storage`` (e.g. `to_bf16`), the same float64 chain is evaluated with each such tensor passed
through it, at the points listed in `layer_backward`; with ``storage=None`` nothing is rounded (the
exact gradient, pinned by central differences in tests/test_oracle_backward.py).  The rounded chain
is what a bfloat16 implementation is compared with at a tight bar: the two then differ only by
accumulation order and by values that sit on a rounding boundary.
"""
from __future__ import annotations

import numpy as np


def to_bf16(a):
    """Nearest bfloat16 (8 significant bits, ties to even) of float32(a), as float64: the upper 16 bits of
    the float32 pattern after adding half a step (0x7FFF, plus the lowest kept bit so that ties go to the
    even mantissa).  Finite values below the overflow threshold only."""
    u = np.asarray(a, dtype=np.float32).view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(np.float64)


def to_bf16_by_mantissa(a):
    """The same rounding from its definition, for float64 input: scale the mantissa to 8 bits, round to
    nearest even, scale back (slow; the twin that pins `to_bf16`)."""
    m, e = np.frexp(np.asarray(a, dtype=np.float64))      # a = m * 2**e with 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def _keep(a):
    return a


def combine_backward(g_y, out_epd, brim_0, brim_1, brim_w, dev_count, storage=None):
    """Transposes of "Combine" and of the weighted merge.

    g_y [T, d] gradient of the layer output; out_epd: per device, the experts' output rows
    [n_epd_dev, d] in the device's local EPD order; brim_0 [D, T]; brim_1 / brim_w per device.
    Returns g_sfd [N_sfd, d], per device g_out [n_epd_dev, d] and g_w [G, n_sfd_dev] (gradient of
    brim_w; zero where BRIM_1 is -1).  ``storage`` rounds the rows of g_out (they are stored and read
    again by the experts' backward).
    """
    rnd = storage or _keep
    D, T = brim_0.shape
    n_sfd = int(np.sum(dev_count))
    g_sfd = np.zeros((n_sfd, g_y.shape[1]), dtype=np.float64)
    for d in range(D):
        v = brim_0[d]
        present = v >= 0
        g_sfd[v[present]] = g_y[present]
    offs = np.concatenate([[0], np.cumsum(dev_count)])
    g_out_all, g_w_all = [], []
    for d in range(D):
        seg = g_sfd[int(offs[d]):int(offs[d + 1])]
        b1, bw = brim_1[d], brim_w[d]
        g_out = np.zeros((int((b1 >= 0).sum()), g_y.shape[1]), dtype=np.float64)
        g_w = np.zeros(b1.shape, dtype=np.float64)
        for e in range(b1.shape[0]):
            v = b1[e]
            present = v >= 0
            g_out[v[present]] = rnd(bw[e, present][:, None] * seg[present])
            g_w[e, present] = np.einsum("rc,rc->r", seg[present], out_epd[d][v[present]].astype(np.float64))
        g_out_all.append(g_out)
        g_w_all.append(g_w)
    return g_sfd, g_out_all, g_w_all


def dispatch_backward(g_in_epd, brim_0, brim_1, dev_count, sfd_round=None):
    """Transposes of the SFD -> EPD row gather and of "Dispatch".

    g_in_epd: per device, the gradient of every expert input row [n_epd_dev, d] (local EPD order).
    Returns g_sfd [N_sfd, d] (the payload of the backward return trip; passed through
    ``sfd_round`` if given, as the forward merge rounds its payload to the storage type) and
    g_x [T, d].
    """
    D, T = brim_0.shape
    d_model = g_in_epd[0].shape[1]
    n_sfd = int(np.sum(dev_count))
    offs = np.concatenate([[0], np.cumsum(dev_count)])
    g_sfd = np.zeros((n_sfd, d_model), dtype=np.float64)
    for d in range(D):
        seg = g_sfd[int(offs[d]):int(offs[d + 1])]   # a view: written in place
        b1 = brim_1[d]
        for e in range(b1.shape[0]):                  # local experts in slot order
            v = b1[e]
            present = v >= 0
            seg[present] += g_in_epd[d][v[present]].astype(np.float64)
    if sfd_round is not None:
        g_sfd = sfd_round(g_sfd)
    g_x = np.zeros((T, d_model), dtype=np.float64)
    for d in range(D):                                # devices in ascending order
        v = brim_0[d]
        present = v >= 0
        g_x[present] += g_sfd[v[present]]
    return g_sfd, g_x


def gate_grad_to_slots(g_w_all, ids, brim_0, L, dev_count):
    """Per-device gradients of brim_w -> gradient of w [T, k]: slot s of token t belongs to
    expert ids[t, s], which is local expert e of device d; its entry is g_w[d][e, SFD row of t
    inside the device's segment]."""
    T, k = ids.shape
    where = {}
    for d, experts in enumerate(L):
        for e, expert in enumerate(experts):
            where[int(expert)] = (d, e)
    offs = np.concatenate([[0], np.cumsum(dev_count)])
    g = np.zeros((T, k), dtype=np.float64)
    for t in range(T):
        for s in range(k):
            d, e = where[int(ids[t, s])]
            g[t, s] = g_w_all[d][e, int(brim_0[d, t] - offs[d])]
    return g


def route_backward(logits, ids, g_w, renorm):
    """Gradient of the gate values with respect to the router scores, [T, E].

    p = Softmax(logits); w_s = p[ids_s], divided by Z = sum_s p[ids_s] if renorm.
    """
    T, E = logits.shape
    l64 = logits.astype(np.float64)
    z = np.exp(l64 - l64.max(axis=1, keepdims=True))
    p = z / z.sum(axis=1, keepdims=True)
    g_p = np.zeros((T, E), dtype=np.float64)        # gradient with respect to p
    rows = np.arange(T)[:, None]
    sel = p[rows, ids]
    if renorm:
        Z = sel.sum(axis=1, keepdims=True)
        w = sel / Z
        # w_s = sel_s / Z  ->  d w_s / d sel_r = (delta_sr - w_s) / Z
        g_sel = (g_w - (g_w * w).sum(axis=1, keepdims=True)) / Z
    else:
        g_sel = g_w.astype(np.float64)
    np.add.at(g_p, (np.broadcast_to(rows, ids.shape), ids), g_sel)
    # softmax: d p_i / d l_j = p_i (delta_ij - p_j)
    return p * (g_p - (g_p * p).sum(axis=1, keepdims=True))


def expert_ffn_backward(v, g_out, w_gate, w_up, w_down, with_pre=False, storage=None, store_g_v=True):
    """Backward of one SwiGLU expert E(v) = W_down (silu(W_gate v) * (W_up v)) for rows v [n, d] and
    output gradients g_out [n, d] (the forward is the expert of the baseline configuration; the
    chain rule through it, nothing else).  Returns g_v [n, d] and the weight gradients
    (g_w_gate [f, d], g_w_up [f, d], g_w_down [d, f]) summed over the rows; ``with_pre`` appends the
    gradients of the two pre-activations, [g_gate | g_up] as rows of 2f.
    ``storage`` rounds the tensors kept between the products: the pre-activations as the derivative
    reads them, the intermediate h the forward pass kept (rounded from the unrounded
    pre-activations, as the forward pass computes it), the gradient of h, the gradients of the
    pre-activations and (unless ``store_g_v`` is False: the caller sums several experts first) the rows
    of g_v; the weight gradients are sums in full precision of the rounded factors."""
    rnd = storage or _keep
    v = v.astype(np.float64)
    g_out = g_out.astype(np.float64)
    wg, wu, wd = (a.astype(np.float64) for a in (w_gate, w_up, w_down))
    g = v @ wg.T
    u = v @ wu.T
    h = rnd(g / (1.0 + np.exp(-g)) * u)                # what the forward pass stored
    g, u = rnd(g), rnd(u)
    sig = 1.0 / (1.0 + np.exp(-g))
    g_h = rnd(g_out @ wd)                              # [n, f]
    g_g = rnd(g_h * u * sig * (1.0 + g * (1.0 - sig)))  # d silu(g) / d g = sig * (1 + g * (1 - sig))
    g_u = rnd(g_h * g * sig)
    g_v = g_g @ wg + g_u @ wu
    if store_g_v:
        g_v = rnd(g_v)
    if with_pre:
        return g_v, (g_g.T @ v, g_u.T @ v, g_out.T @ h), np.concatenate([g_g, g_u], axis=1)
    return g_v, (g_g.T @ v, g_u.T @ v, g_out.T @ h)


def layer_backward(x, ids, w, expert_pos, D, w_gate, w_up, w_down, S, g_y, storage=None):
    """Backward of the whole deduplicated layer, the forward pipeline walked in reverse on the same
    re-index matrices: transposed Combine and merge, the experts' own backward per device and local
    expert, transposed row gather and Dispatch; shared experts see every token with weight 1.
    Returns a dict: g_x [T, d], g_w [T, k], g_w_gate / g_w_up / g_w_down like the weights, and the
    intermediate payloads g_sfd_y, g_sfd_x and per-device EPD rows g_epd_y, g_epd_gu ([g_gate | g_up]), g_epd_x.
    ``storage`` (see the module text) rounds: the forward's kept tensors (the intermediate h and the
    experts' output rows, which the gate gradient reads), the gate-scaled output-gradient rows, every
    tensor `expert_ffn_backward` lists, the SFD payload of the return trip, the shared experts' summed
    input gradient, and g_x itself."""
    from . import occult_ref
    rnd = storage or _keep
    T, d = x.shape
    E = len(expert_pos)
    tr = occult_ref.moe_forward(x, ids, w, expert_pos, D)
    L = occult_ref.placement_lists(expert_pos, D)
    offs = np.concatenate([[0], np.cumsum(tr.dev_count)])
    # forward pieces that the backward needs: every expert's output rows, per device in local EPD order
    out_epd = []
    for j in range(D):
        seg = tr.x_sfd[int(offs[j]):int(offs[j + 1])].astype(np.float64)
        rows = np.zeros((int((tr.brim_1[j] >= 0).sum()), d))
        for e, expert in enumerate(L[j]):
            v = tr.brim_1[j][e]
            present = v >= 0
            if present.any():
                g = seg[present] @ w_gate[expert].astype(np.float64).T
                u = seg[present] @ w_up[expert].astype(np.float64).T
                rows[v[present]] = rnd(rnd(g / (1.0 + np.exp(-g)) * u) @ w_down[expert].astype(np.float64).T)
        out_epd.append(rows)
    g_sfd_y, g_out, g_bw = combine_backward(g_y, out_epd, tr.brim_0, tr.brim_1, tr.brim_w, tr.dev_count, storage)
    g_wg = np.zeros(w_gate.shape)
    g_wu = np.zeros(w_up.shape)
    g_wd = np.zeros(w_down.shape)
    g_in, g_pre = [], []
    for j in range(D):
        seg = tr.x_sfd[int(offs[j]):int(offs[j + 1])]
        rows = np.zeros_like(g_out[j])
        pre = np.zeros((g_out[j].shape[0], 2 * w_gate.shape[1]))
        for e, expert in enumerate(L[j]):
            v = tr.brim_1[j][e]
            present = v >= 0
            if present.any():
                g_v, (a, b, c), gu = expert_ffn_backward(seg[present], g_out[j][v[present]], w_gate[expert],
                                                         w_up[expert], w_down[expert], with_pre=True,
                                                         storage=storage)
                rows[v[present]] = g_v
                pre[v[present]] = gu
                g_wg[expert] += a
                g_wu[expert] += b
                g_wd[expert] += c
        g_in.append(rows)
        g_pre.append(pre)
    g_sfd_x, g_x = dispatch_backward(g_in, tr.brim_0, tr.brim_1, tr.dev_count, sfd_round=storage)
    g_shared = np.zeros_like(g_x)
    for s in range(S):
        # the shared experts' input gradients are summed before they are stored: one rounding
        g_v, (a, b, c) = expert_ffn_backward(x, g_y, w_gate[E + s], w_up[E + s], w_down[E + s],
                                             storage=storage, store_g_v=False)
        g_shared += g_v
        g_wg[E + s] += a
        g_wu[E + s] += b
        g_wd[E + s] += c
    g_x = rnd(g_x + rnd(g_shared)) if S else rnd(g_x)
    return {"g_x": g_x, "g_w": gate_grad_to_slots(g_bw, ids, tr.brim_0, L, tr.dev_count),
            "g_w_gate": g_wg, "g_w_up": g_wu, "g_w_down": g_wd, "g_sfd_y": g_sfd_y, "g_sfd_x": g_sfd_x,
            "g_epd_x": g_in, "g_epd_y": g_out, "g_epd_gu": g_pre, "trace": tr}


def moe_layer_backward_tokens(x, ids, w, w_gate, w_up, w_down, E, S, g_y, tokens=None):
    """Input and gate gradients of the textbook layer y[t] = sum_s w[t,s] E_{ids[t,s]}(x[t]) + shared,
    for a subset of tokens (sampled parity at full size): a token's gradients depend on its own row
    only.  Returns g_x [n, d] and g_w [n, k] for the n tokens, grouped by expert so that BLAS does
    the products."""
    if tokens is None:
        tokens = np.arange(x.shape[0])
    tokens = np.asarray(tokens)
    xs = x[tokens].astype(np.float64)
    gs = g_y[tokens].astype(np.float64)
    ids_s = ids[tokens]
    w_s = w[tokens].astype(np.float64)
    g_x = np.zeros_like(xs)
    g_w = np.zeros(ids_s.shape, dtype=np.float64)
    for e in range(E):
        rows, slots = np.nonzero(ids_s == e)
        if rows.size == 0:
            continue
        v = xs[rows]
        g_v, _ = expert_ffn_backward(v, w_s[rows, slots][:, None] * gs[rows], w_gate[e], w_up[e], w_down[e])
        g_x[rows] += g_v
        a = v @ w_gate[e].astype(np.float64).T
        u = v @ w_up[e].astype(np.float64).T
        out = (a / (1.0 + np.exp(-a)) * u) @ w_down[e].astype(np.float64).T
        g_w[rows, slots] = np.einsum("rc,rc->r", gs[rows], out)
    for s in range(S):
        g_v, _ = expert_ffn_backward(xs, gs, w_gate[E + s], w_up[E + s], w_down[E + s])
        g_x += g_v
    return g_x, g_w
