"""CPU oracle: backward pass of the layer's data movement (dispatch, row replication, two-stage
merge, combine) and of the routing weights.

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

`route_backward` is the gradient of the gate values of Eq. 1 with respect to the router scores:
Softmax over all E experts, the values at the k selected experts, optionally divided by their sum.
The selection itself is piecewise constant and contributes nothing.
Float arithmetic is float64.
"""
from __future__ import annotations

import numpy as np


def combine_backward(g_y, out_epd, brim_0, brim_1, brim_w, dev_count):
    """Transposes of "Combine" and of the weighted merge.

    g_y [T, d] gradient of the layer output; out_epd: per device, the experts' output rows
    [n_epd_dev, d] in the device's local EPD order; brim_0 [D, T]; brim_1 / brim_w per device.
    Returns g_sfd [N_sfd, d], per device g_out [n_epd_dev, d] and g_w [G, n_sfd_dev] (gradient of
    brim_w; zero where BRIM_1 is -1).
    """
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
            g_out[v[present]] = bw[e, present][:, None] * seg[present]
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
