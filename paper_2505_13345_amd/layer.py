"""Device buffers for one layer and the call sequence of its hot path (forward, and the backward
pass of the data movement).

Memory plumbing only: torch allocates the worst-case-sized buffers once (N_sfd <= T*min(k, D),
N_epd = T*k), every step is one call into the C library on the current stream, and nothing here
synchronises or computes.  Table views onto the plan block are for tests and reports.
"""
from __future__ import annotations

import torch

from . import binding as B


class OccultLayer:
    def __init__(self, T, d, f, E, S, k, D, dtype="bf16", n_d=0, prune_mode=1, renorm=1,
                 expert_pos=None, device="cuda:0", with_ffn=True, sim_table=None):
        B.load_library()          # fail early and loudly if the HIP library is missing
        self.device = torch.device(device)
        self.shape = dict(T=T, d=d, f=f, E=E, S=S, k=k, D=D)
        self.dtype_name = dtype
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        dev = self.device
        self.expert_pos = None
        if expert_pos is not None:
            self.expert_pos = torch.as_tensor(expert_pos, dtype=torch.int32).to(dev).contiguous()
        self.sim_table = None
        if sim_table is not None:
            self.sim_table = torch.as_tensor(sim_table, dtype=torch.int32).to(dev).contiguous()
        self.cfg = B.make_cfg(T, d, f, E, S, k, D, dtype, n_d, prune_mode, renorm, self.expert_pos, self.sim_table)
        plan_bytes, ws_bytes = B.occult_plan_sizes(self.cfg)
        self.plan_mem = torch.zeros(plan_bytes, dtype=torch.uint8, device=dev)
        self.ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=dev)
        self.plan = B.occult_plan_bind(self.cfg, self.plan_mem)
        n_sfd_max = T * min(k, D)
        self.n_sfd_max = n_sfd_max
        self.ids = torch.zeros((T, k), dtype=torch.int32, device=dev)
        self.w = torch.zeros((T, k), dtype=torch.float32, device=dev)
        self.sfd_x = torch.zeros((n_sfd_max, d), dtype=self.tdtype, device=dev)
        self.sfd_y = torch.zeros((n_sfd_max, d), dtype=self.tdtype, device=dev)
        self.y = torch.zeros((T, d), dtype=self.tdtype, device=dev)
        self.epd_h = self.epd_y = self.h_shared = self.y_shared = self.ffn_ws = None
        if with_ffn:
            ws_bytes = B.occult_expert_ffn_ws_bytes(self.cfg)
            if ws_bytes:
                self.ffn_ws = torch.empty(ws_bytes // 4, dtype=torch.float32, device=dev)
            self.epd_h = torch.zeros((T * k, f), dtype=self.tdtype, device=dev)
            self.epd_y = torch.zeros((T * k, d), dtype=self.tdtype, device=dev)
            if S > 0:
                self.h_shared = torch.zeros((T, S * f), dtype=self.tdtype, device=dev)
                self.y_shared = torch.zeros((T, d), dtype=self.tdtype, device=dev)

    # ---- element type and size of the caller's tensors (the library sees raw pointers) --------
    def _hidden(self, t, name, rows=None):
        s = self.shape
        return B.expect(t, name, self.tdtype, (s["T"] if rows is None else rows) * s["d"])

    def _weights(self, w_gate, w_up, w_down):
        s = self.shape
        n = (s["E"] + s["S"]) * s["d"] * s["f"]
        for t, name in ((w_gate, "w_gate"), (w_up, "w_up"), (w_down, "w_down")):
            B.expect(t, name, self.tdtype, n)

    def _routing(self, ids, w):
        s = self.shape
        B.expect(ids, "ids", torch.int32, s["T"] * s["k"])
        B.expect(w, "w", torch.float32, s["T"] * s["k"])

    # ---- steps (each = one library call on the current stream) -------------------------------
    def route(self, logits):
        B.expect(logits, "logits", torch.float32, self.shape["T"] * self.shape["E"])
        B.occult_route(self.cfg, logits, self.ids, self.w)

    def route_from_hidden(self, x, w_router, logits_out):
        """Router projection x w_router^T -> logits_out [T, E] f32, then routing, in one call."""
        s = self.shape
        self._hidden(x, "x")
        B.expect(w_router, "w_router", self.tdtype, s["E"] * s["d"])
        B.expect(logits_out, "logits_out", torch.float32, s["T"] * s["E"])
        B.occult_router(self.cfg, x, w_router, logits_out, self.ids, self.w)

    def make_plan(self, ids=None, w=None):
        self._routing(ids, w)
        B.occult_plan(self.cfg, self.ids if ids is None else ids, self.w if w is None else w,
                      self.plan, self.ws)

    def dispatch(self, x):
        self._hidden(x, "x")
        B.occult_dispatch(self.cfg, self.plan, x, self.sfd_x)

    def pack_weights(self, w_gate, w_up, w_down):
        """One-time repacking of the weights for decode-shaped batches (again after a weight update);
        expert_ffn() then reads the packed copy wherever the weight-streaming kernel runs."""
        n = B.occult_pack_weights_bytes(self.cfg)
        if n == 0:
            return None
        if getattr(self, "packed", None) is None:
            self.packed = torch.empty(n // 2, dtype=torch.bfloat16, device=self.device)
        B.occult_pack_weights(self.cfg, w_gate, w_up, w_down, self.packed)
        return self.packed

    def expert_ffn(self, x, w_gate, w_up, w_down, use_ws=True):
        self._hidden(x, "x")
        self._weights(w_gate, w_up, w_down)
        if getattr(self, "packed", None) is not None:
            B.occult_expert_ffn_packed(self.cfg, self.plan, self.sfd_x, x, w_gate, w_up, w_down, self.packed, self.epd_h,
                                       self.epd_y, self.h_shared, self.y_shared, self.ffn_ws if use_ws else None)
            return
        if use_ws and self.ffn_ws is not None:
            B.occult_expert_ffn_ws(self.cfg, self.plan, self.sfd_x, x, w_gate, w_up, w_down, self.epd_h,
                                   self.epd_y, self.h_shared, self.y_shared, self.ffn_ws)
        else:
            B.occult_expert_ffn(self.cfg, self.plan, self.sfd_x, x, w_gate, w_up, w_down, self.epd_h,
                                self.epd_y, self.h_shared, self.y_shared)

    def expert_ffn_train(self, x, w_gate, w_up, w_down):
        """expert_ffn() that also keeps the pre-activations [g | u] for expert_ffn_backward(gu_saved=True)."""
        s = self.shape
        T, k, f, S = s["T"], s["k"], s["f"], s["S"]
        self._hidden(x, "x")
        self._weights(w_gate, w_up, w_down)
        epd_gu = self._buf("epd_gu", (T * k, 2 * f), self.tdtype)
        gu_sh = self._buf("gu_shared", (T, S * 2 * f), self.tdtype) if S > 0 else None
        B.occult_expert_ffn_train(self.cfg, self.plan, self.sfd_x, x, w_gate, w_up, w_down, self.epd_h, self.epd_y,
                                  self.h_shared, self.y_shared, epd_gu, gu_sh, self.ffn_ws)
        self.gu_saved = True

    def combine(self, epd_y=None):
        self._hidden(epd_y, "epd_y", self.shape["T"] * self.shape["k"])
        B.occult_combine(self.cfg, self.plan, self.epd_y if epd_y is None else epd_y, self.sfd_y,
                         self.y_shared, self.y)

    def combine_atomic(self, epd_y=None, mode=0):
        """combine() with the paper's atomic merge as its first stage (mode 0: float32 atomics into a scratch
        tensor allocated on first use; mode 1: packed bf16 atomics into sfd_y)."""
        s = self.shape
        self._hidden(epd_y, "epd_y", s["T"] * s["k"])
        acc = self._buf("sfd_acc", (self.n_sfd_max, s["d"]), torch.float32) if mode == 0 else None
        B.occult_combine_atomic(self.cfg, self.plan, self.epd_y if epd_y is None else epd_y, acc, self.sfd_y,
                                self.y_shared, self.y, mode)

    def forward(self, logits, x, w_gate, w_up, w_down, train=False):
        self.route(logits)
        self.make_plan()
        self.dispatch(x)
        if train:
            self.expert_ffn_train(x, w_gate, w_up, w_down)
        else:
            self.expert_ffn(x, w_gate, w_up, w_down)
        self.combine()
        return self.y

    # ---- backward of the data movement (buffers allocated on first use) -----------------------
    def _buf(self, name, shape, dtype):
        if getattr(self, name, None) is None:
            setattr(self, name, torch.zeros(shape, dtype=dtype, device=self.device))
        return getattr(self, name)

    def combine_backward(self, dy, ids=None, epd_y=None, want_sfd=True, want_epd=True, want_dw=True):
        """dy [T, d] -> sfd_dy, epd_dy, dw (each None if not asked for)."""
        s = self.shape
        sfd_dy = self._buf("sfd_dy", (self.n_sfd_max, s["d"]), self.tdtype) if want_sfd else None
        epd_dy = self._buf("epd_dy", (s["T"] * s["k"], s["d"]), self.tdtype) if want_epd else None
        dw = self._buf("dw", (s["T"], s["k"]), torch.float32) if want_dw else None
        self._hidden(dy, "dy")
        self._hidden(epd_y, "epd_y", s["T"] * s["k"])
        B.expect(ids, "ids", torch.int32, s["T"] * s["k"])
        B.occult_combine_backward(self.cfg, self.plan, self.ids if ids is None else ids, dy,
                                  self.epd_y if epd_y is None else epd_y, sfd_dy, epd_dy, dw)
        return sfd_dy, epd_dy, dw

    def dispatch_backward(self, epd_dx, dx_shared=None):
        """epd_dx [T*k, d] -> sfd_dx, dx."""
        s = self.shape
        sfd_dx = self._buf("sfd_dx", (self.n_sfd_max, s["d"]), self.tdtype)
        dx = self._buf("dx", (s["T"], s["d"]), self.tdtype)
        self._hidden(epd_dx, "epd_dx", s["T"] * s["k"])
        self._hidden(dx_shared, "dx_shared")
        B.occult_dispatch_backward(self.cfg, self.plan, epd_dx, sfd_dx, dx_shared, dx)
        return sfd_dx, dx

    def transpose_weights(self, w_gate, w_up, w_down):
        """Transposed weight copies for the backward products (again after every weight update)."""
        s = self.shape
        n = s["E"] + s["S"]
        w_down_t = self._buf("w_down_t", (n, s["f"], s["d"]), self.tdtype)
        w_gu_t = self._buf("w_gu_t", (n, s["d"], 2 * s["f"]), self.tdtype)
        self._weights(w_gate, w_up, w_down)
        B.occult_transpose_weights(self.cfg, w_gate, w_up, w_down, w_down_t, w_gu_t)
        return w_down_t, w_gu_t

    def expert_ffn_backward(self, x, w_gate, w_up, epd_dy, dy, gu_saved=None):
        """epd_dy [T*k, d] (and dy [T, d] for shared experts) -> epd_dx, dx_shared (None if S == 0);
        needs transpose_weights() first and the forward's sfd_x."""
        s = self.shape
        T, k, d, f, S = s["T"], s["k"], s["d"], s["f"], s["S"]
        epd_gu = self._buf("epd_gu", (T * k, 2 * f), self.tdtype)
        epd_dh = self._buf("epd_dh", (T * k, f), self.tdtype)
        epd_dx = self._buf("epd_dx", (T * k, d), self.tdtype)
        gu_sh = dh_sh = dx_sh = None
        if S > 0:
            gu_sh = self._buf("gu_shared", (T, S * 2 * f), self.tdtype)
            dh_sh = self._buf("dh_shared", (T, S * f), self.tdtype)
            dx_sh = self._buf("dx_shared", (T, d), self.tdtype)
        self._hidden(x, "x")
        self._hidden(dy, "dy")
        self._hidden(epd_dy, "epd_dy", T * k)
        self._weights(w_gate, w_up, None)
        if gu_saved is None:   # pre-activations kept by expert_ffn_train() since the last backward
            gu_saved = getattr(self, "gu_saved", False)
        B.occult_expert_ffn_backward(self.cfg, self.plan, self.sfd_x, x, w_gate, w_up, self.w_down_t, self.w_gu_t,
                                     epd_dy, dy, epd_gu, epd_dh, epd_dx, gu_sh, dh_sh, dx_sh, gu_saved)
        self.gu_saved = False      # overwritten with [dg | du]
        return epd_dx, dx_sh

    def expert_ffn_backward_weights(self, x, dy, accumulate=False, use_ws=True):
        """f32 weight gradients dw_gate, dw_up [E+S, f, d], dw_down [E+S, d, f]; after expert_ffn_backward()."""
        s = self.shape
        n = s["E"] + s["S"]
        dw_gate = self._buf("dw_gate", (n, s["f"], s["d"]), torch.float32)
        dw_up = self._buf("dw_up", (n, s["f"], s["d"]), torch.float32)
        dw_down = self._buf("dw_down", (n, s["d"], s["f"]), torch.float32)
        self._hidden(x, "x")
        self._hidden(dy, "dy")
        ws = None
        if use_ws:   # scratch for the row slices of the shared experts' products (large T, few shared experts)
            n = B.occult_expert_ffn_backward_weights_ws_bytes(self.cfg)
            if n:
                ws = self._buf("wgrad_ws", (n // 4,), torch.float32)
        B.occult_expert_ffn_backward_weights_ws(self.cfg, self.plan, self.sfd_x, x, self.epd_h, self.h_shared, self.epd_dy,
                                                dy, self.epd_gu, getattr(self, "gu_shared", None), dw_gate, dw_up, dw_down,
                                                ws, accumulate)
        return dw_gate, dw_up, dw_down

    def backward_input(self, x, w_gate, w_up, dy):
        """dy [T, d] -> dx [T, d], dw [T, k]: the three backward calls in order (after forward())."""
        _, epd_dy, dw = self.combine_backward(dy, want_sfd=True)
        epd_dx, dx_sh = self.expert_ffn_backward(x, w_gate, w_up, epd_dy, dy)
        _, dx = self.dispatch_backward(epd_dx, dx_sh)
        return dx, dw

    def route_backward(self, logits, dw, dlogits, ids=None):
        s = self.shape
        B.expect(logits, "logits", torch.float32, s["T"] * s["E"])
        B.expect(dlogits, "dlogits", torch.float32, s["T"] * s["E"])
        self._routing(ids, dw)
        B.occult_route_backward(self.cfg, logits, self.ids if ids is None else ids, dw, dlogits)

    def stats(self):
        return B.occult_plan_stats(self.cfg, self.plan)

    # ---- views onto the plan block ------------------------------------------------------------
    def _view(self, field, count, dtype):
        base = self.plan_mem.data_ptr()
        off = getattr(self.plan, field) - base
        nbytes = count * torch.empty((), dtype=dtype).element_size()
        return self.plan_mem[off:off + nbytes].view(dtype)

    def tables(self):
        s = self.shape
        T, E, D, k = s["T"], s["E"], s["D"], s["k"]
        m1 = min(k, E // D)
        i32 = torch.int32
        return {
            "tok_devmask": self._view("tok_devmask", T, torch.int64),
            "dev_count": self._view("dev_count", D, i32),
            "dev_offset": self._view("dev_offset", D + 1, i32),
            "tok_sfd_row": self._view("tok_sfd_row", T * D, i32).view(T, D),
            "sfd_token": self._view("sfd_token", self.n_sfd_max, i32),
            "exp_count": self._view("exp_count", E, i32),
            "exp_offset": self._view("exp_offset", E + 1, i32),
            "pos_expert": self._view("pos_expert", E, i32),
            "epd_sfd_row": self._view("epd_sfd_row", T * k, i32),
            "epd_gate": self._view("epd_gate", T * k, torch.float32),
            "sfd_epd_rows": self._view("sfd_epd_rows", self.n_sfd_max * m1, i32).view(self.n_sfd_max, m1),
            "counters": self._view("counters", 8, torch.int64),
        }
