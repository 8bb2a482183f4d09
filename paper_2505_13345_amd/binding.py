"""ctypes binding of liboccult.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/occult.h) and does
nothing but turn torch tensors into device pointers, pass the current HIP stream and raise
``OccultError`` on a non-zero return code.  All arithmetic of the layer runs in the library's
HIP kernels; torch supplies device memory and streams.  There is no CPU fallback: if the shared
library is missing or was not built, importing a symbol raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_double, c_float, c_int, c_int32, c_size_t, c_uint64, c_void_p
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liboccult.so")

OCCULT_F32, OCCULT_BF16 = 0, 1

EXPORTS = [
    "occult_version", "occult_last_error", "occult_plan_sizes", "occult_plan_bind", "occult_route",
    "occult_plan", "occult_dispatch", "occult_expert_ffn", "occult_combine", "occult_coactivation",
    "occult_placement_greedy", "occult_plan_stats", "occult_router", "occult_dispatch_meta",
    "occult_similarity_gram", "occult_similarity_table", "occult_expert_ffn_ws_bytes", "occult_expert_ffn_ws",
    "occult_combine_backward", "occult_dispatch_backward", "occult_route_backward",
    "occult_transpose_weights", "occult_expert_ffn_backward", "occult_expert_ffn_backward_weights",
    "occult_pack_weights_bytes", "occult_pack_weights", "occult_expert_ffn_packed", "occult_expert_ffn_train",
    "occult_collaboration_stats", "occult_plan_static", "occult_combine_atomic",
    "occult_expert_ffn_backward_weights_ws_bytes", "occult_expert_ffn_backward_weights_ws",
]


class OccultError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"occult error {code}: {msg}")
        self.code = code


class occult_cfg_t(Structure):
    _fields_ = [("T", c_int32), ("d", c_int32), ("f", c_int32), ("E", c_int32), ("S", c_int32),
                ("k", c_int32), ("D", c_int32), ("n_d", c_int32), ("prune_mode", c_int32),
                ("renorm", c_int32), ("dtype", c_int32), ("ffn_phase", c_int32),
                ("expert_pos", c_void_p), ("sim_table", c_void_p)]


class occult_plan_t(Structure):
    _fields_ = [("tok_devmask", c_void_p), ("dev_count", c_void_p), ("dev_offset", c_void_p),
                ("tok_sfd_row", c_void_p), ("sfd_token", c_void_p), ("exp_count", c_void_p),
                ("exp_offset", c_void_p), ("pos_expert", c_void_p), ("epd_sfd_row", c_void_p),
                ("epd_gate", c_void_p), ("sfd_epd_rows", c_void_p), ("counters", c_void_p)]


class occult_weights_t(Structure):
    _fields_ = [("w_gate", c_void_p), ("w_up", c_void_p), ("w_down", c_void_p)]


class occult_stats_t(Structure):
    _fields_ = [("n_sfd", c_uint64), ("n_epd", c_uint64), ("rows_std", c_uint64),
                ("max_dev_count", c_uint64), ("max_exp_count", c_uint64), ("bytes_occ", c_uint64),
                ("bytes_std", c_uint64), ("bytes_meta", c_uint64), ("c_t", c_double)]


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load liboccult.so (built in-tree by paper_2505_13345_amd.build).  Fails loudly."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise ImportError(f"{p} not found: build it with `python -m paper_2505_13345_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(p)
    cfgp, planp = POINTER(occult_cfg_t), POINTER(occult_plan_t)
    lib.occult_version.restype = c_int
    lib.occult_version.argtypes = []
    lib.occult_last_error.restype = c_char_p
    lib.occult_last_error.argtypes = []
    lib.occult_plan_sizes.argtypes = [cfgp, POINTER(c_size_t), POINTER(c_size_t)]
    lib.occult_plan_bind.argtypes = [cfgp, c_void_p, c_size_t, planp]
    lib.occult_route.argtypes = [cfgp, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.occult_similarity_gram.argtypes = [cfgp, c_void_p, c_void_p, c_int, c_void_p]
    lib.occult_similarity_table.argtypes = [c_void_p, c_int32, c_void_p]
    lib.occult_router.argtypes = [cfgp, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.occult_plan.argtypes = [cfgp, c_void_p, c_void_p, planp, c_void_p, c_size_t, c_void_p]
    lib.occult_plan_static.argtypes = [cfgp, c_void_p, c_void_p, planp, c_void_p]
    lib.occult_dispatch.argtypes = [cfgp, planp, c_void_p, c_void_p, c_void_p]
    lib.occult_dispatch_meta.argtypes = [cfgp, planp, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.occult_expert_ffn.argtypes = [cfgp, planp, c_void_p, c_void_p, POINTER(occult_weights_t),
                                      c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.occult_expert_ffn_ws_bytes.argtypes = [cfgp, POINTER(c_size_t)]
    lib.occult_expert_ffn_ws.argtypes = [cfgp, planp, c_void_p, c_void_p, POINTER(occult_weights_t),
                                         c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.occult_pack_weights_bytes.argtypes = [cfgp, POINTER(c_size_t)]
    lib.occult_pack_weights.argtypes = [cfgp, POINTER(occult_weights_t), c_void_p, c_size_t, c_void_p]
    lib.occult_expert_ffn_packed.argtypes = [cfgp, planp, c_void_p, c_void_p, POINTER(occult_weights_t), c_void_p,
                                             c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.occult_combine.argtypes = [cfgp, planp, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.occult_combine_atomic.argtypes = [cfgp, planp, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p]
    lib.occult_combine_backward.argtypes = [cfgp, planp, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                            c_void_p]
    lib.occult_dispatch_backward.argtypes = [cfgp, planp, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.occult_route_backward.argtypes = [cfgp, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.occult_transpose_weights.argtypes = [cfgp, POINTER(occult_weights_t), c_void_p, c_void_p, c_void_p]
    lib.occult_expert_ffn_backward.argtypes = ([cfgp, planp, c_void_p, c_void_p, POINTER(occult_weights_t)] + [c_void_p] * 10
                                              + [c_int, c_void_p])
    lib.occult_expert_ffn_train.argtypes = [cfgp, planp, c_void_p, c_void_p, POINTER(occult_weights_t)] + [c_void_p] * 7 + [
        c_size_t, c_void_p]
    lib.occult_expert_ffn_backward_weights.argtypes = [cfgp, planp] + [c_void_p] * 11 + [c_int, c_void_p]
    lib.occult_expert_ffn_backward_weights_ws_bytes.argtypes = [cfgp, POINTER(c_size_t)]
    lib.occult_expert_ffn_backward_weights_ws.argtypes = [cfgp, planp] + [c_void_p] * 11 + [c_int, c_void_p, c_size_t, c_void_p]
    lib.occult_coactivation.argtypes = [cfgp, c_void_p, c_void_p, c_int, c_void_p]
    lib.occult_placement_greedy.argtypes = [c_void_p, c_int32, c_int32, c_void_p, c_void_p]
    lib.occult_collaboration_stats.argtypes = [c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.occult_plan_stats.argtypes = [cfgp, planp, POINTER(occult_stats_t), c_void_p]
    for name in EXPORTS:
        if name not in ("occult_version", "occult_last_error"):
            getattr(lib, name).restype = c_int
    if path is None:
        _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise OccultError(rc, load_library().occult_last_error().decode())


def _ptr(t) -> Optional[int]:
    """Device address of a tensor.  The library reads raw memory, so the tensor must be a dense
    (contiguous) block in GPU memory: anything else would hand it a pointer it misreads."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("occult: tensor is not in GPU memory")
    if not t.is_contiguous():
        raise ValueError(f"occult: tensor of shape {tuple(t.shape)} is not contiguous")
    return t.data_ptr()


def expect(t, name: str, dtype, numel: int):
    """Marshalling check for a caller's tensor: element type and element count the call will read or
    write (None passes through).  Returns t."""
    if t is None:
        return t
    if t.dtype != dtype:
        raise ValueError(f"occult: {name} has dtype {t.dtype}, the call needs {dtype}")
    if t.numel() < numel:
        raise ValueError(f"occult: {name} has {t.numel()} elements, the call needs {numel}")
    return t


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def make_cfg(T, d, f, E, S, k, D, dtype, n_d=0, prune_mode=1, renorm=1, expert_pos=None,
             sim_table=None) -> occult_cfg_t:
    """expert_pos: int32 device tensor [E] or None; sim_table: int32 device tensor [E, E-1] or None;
    the caller keeps both alive."""
    code = {"bf16": OCCULT_BF16, "f32": OCCULT_F32}[dtype] if isinstance(dtype, str) else int(dtype)
    return occult_cfg_t(T, d, f, E, S, k, D, n_d, prune_mode, renorm, code, 0, _ptr(expert_pos), _ptr(sim_table))


def occult_version() -> int:
    return load_library().occult_version()


def occult_last_error() -> str:
    return load_library().occult_last_error().decode()


def occult_plan_sizes(cfg: occult_cfg_t):
    pb, wb = c_size_t(0), c_size_t(0)
    _check(load_library().occult_plan_sizes(ctypes.byref(cfg), ctypes.byref(pb), ctypes.byref(wb)))
    return pb.value, wb.value


def occult_plan_bind(cfg: occult_cfg_t, plan_mem) -> occult_plan_t:
    """plan_mem: uint8 device tensor of at least plan_bytes; the caller keeps it alive."""
    plan = occult_plan_t()
    _check(load_library().occult_plan_bind(ctypes.byref(cfg), _ptr(plan_mem), plan_mem.numel(),
                                           ctypes.byref(plan)))
    return plan


def occult_route(cfg, logits, ids, w, stream=None) -> None:
    _check(load_library().occult_route(ctypes.byref(cfg), _ptr(logits), _ptr(ids), _ptr(w), _stream(stream)))


def occult_similarity_gram(cfg, logits, gram, accumulate=False, stream=None) -> None:
    _check(load_library().occult_similarity_gram(ctypes.byref(cfg), _ptr(logits), _ptr(gram), int(bool(accumulate)),
                                                 _stream(stream)))


def occult_similarity_table(gram_host):
    """Host: Gram matrix (numpy float64 [E, E]) -> similarity table (numpy int32 [E, E-1])."""
    import numpy as np
    g = np.ascontiguousarray(gram_host, dtype=np.float64)
    E = g.shape[0]
    out = np.empty((E, max(E - 1, 0)), dtype=np.int32)
    _check(load_library().occult_similarity_table(g.ctypes.data_as(ctypes.c_void_p), E,
                                                  out.ctypes.data_as(ctypes.c_void_p)))
    return out


def occult_router(cfg, x, w_router, logits, ids, w, stream=None) -> None:
    _check(load_library().occult_router(ctypes.byref(cfg), _ptr(x), _ptr(w_router), _ptr(logits), _ptr(ids), _ptr(w),
                                        _stream(stream)))


def occult_plan(cfg, ids, w, plan: occult_plan_t, ws, stream=None) -> None:
    _check(load_library().occult_plan(ctypes.byref(cfg), _ptr(ids), _ptr(w), ctypes.byref(plan), _ptr(ws),
                                      ws.numel() * ws.element_size(), _stream(stream)))


def occult_plan_static(cfg, ids, w, plan: occult_plan_t, stream=None) -> None:
    _check(load_library().occult_plan_static(ctypes.byref(cfg), _ptr(ids), _ptr(w), ctypes.byref(plan), _stream(stream)))


def occult_dispatch(cfg, plan, x, sfd_x, stream=None) -> None:
    _check(load_library().occult_dispatch(ctypes.byref(cfg), ctypes.byref(plan), _ptr(x), _ptr(sfd_x),
                                          _stream(stream)))


def occult_dispatch_meta(cfg, plan, ids, w, sfd_ids, sfd_w, stream=None) -> None:
    _check(load_library().occult_dispatch_meta(ctypes.byref(cfg), ctypes.byref(plan), _ptr(ids), _ptr(w),
                                               _ptr(sfd_ids), _ptr(sfd_w), _stream(stream)))


def occult_expert_ffn(cfg, plan, sfd_x, x, w_gate, w_up, w_down, epd_h, epd_y, h_shared=None,
                      y_shared=None, stream=None) -> None:
    wts = occult_weights_t(_ptr(w_gate), _ptr(w_up), _ptr(w_down))
    _check(load_library().occult_expert_ffn(ctypes.byref(cfg), ctypes.byref(plan), _ptr(sfd_x), _ptr(x),
                                            ctypes.byref(wts), _ptr(epd_h), _ptr(epd_y), _ptr(h_shared),
                                            _ptr(y_shared), _stream(stream)))


def occult_expert_ffn_ws_bytes(cfg) -> int:
    n = c_size_t(0)
    _check(load_library().occult_expert_ffn_ws_bytes(ctypes.byref(cfg), ctypes.byref(n)))
    return int(n.value)


def occult_expert_ffn_ws(cfg, plan, sfd_x, x, w_gate, w_up, w_down, epd_h, epd_y, h_shared, y_shared, ws,
                         stream=None) -> None:
    wts = occult_weights_t(_ptr(w_gate), _ptr(w_up), _ptr(w_down))
    nbytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().occult_expert_ffn_ws(ctypes.byref(cfg), ctypes.byref(plan), _ptr(sfd_x), _ptr(x),
                                               ctypes.byref(wts), _ptr(epd_h), _ptr(epd_y), _ptr(h_shared),
                                               _ptr(y_shared), _ptr(ws), nbytes, _stream(stream)))


def occult_pack_weights_bytes(cfg) -> int:
    n = c_size_t(0)
    _check(load_library().occult_pack_weights_bytes(ctypes.byref(cfg), ctypes.byref(n)))
    return int(n.value)


def occult_pack_weights(cfg, w_gate, w_up, w_down, packed, stream=None) -> None:
    wts = occult_weights_t(_ptr(w_gate), _ptr(w_up), _ptr(w_down))
    _check(load_library().occult_pack_weights(ctypes.byref(cfg), ctypes.byref(wts), _ptr(packed),
                                              packed.numel() * packed.element_size(), _stream(stream)))


def occult_expert_ffn_packed(cfg, plan, sfd_x, x, w_gate, w_up, w_down, packed, epd_h, epd_y, h_shared, y_shared, ws,
                             stream=None) -> None:
    wts = occult_weights_t(_ptr(w_gate), _ptr(w_up), _ptr(w_down))
    nbytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().occult_expert_ffn_packed(ctypes.byref(cfg), ctypes.byref(plan), _ptr(sfd_x), _ptr(x),
                                                   ctypes.byref(wts), _ptr(packed), _ptr(epd_h), _ptr(epd_y),
                                                   _ptr(h_shared), _ptr(y_shared), _ptr(ws), nbytes, _stream(stream)))


def occult_combine(cfg, plan, epd_y, sfd_y, y_shared, y, stream=None) -> None:
    _check(load_library().occult_combine(ctypes.byref(cfg), ctypes.byref(plan), _ptr(epd_y), _ptr(sfd_y),
                                         _ptr(y_shared), _ptr(y), _stream(stream)))


def occult_combine_atomic(cfg, plan, epd_y, sfd_acc, sfd_y, y_shared, y, mode=0, stream=None) -> None:
    _check(load_library().occult_combine_atomic(ctypes.byref(cfg), ctypes.byref(plan), _ptr(epd_y), _ptr(sfd_acc), _ptr(sfd_y),
                                                _ptr(y_shared), _ptr(y), int(mode), _stream(stream)))


def occult_combine_backward(cfg, plan, ids, dy, epd_y, sfd_dy, epd_dy, dw, stream=None) -> None:
    _check(load_library().occult_combine_backward(ctypes.byref(cfg), ctypes.byref(plan), _ptr(ids), _ptr(dy),
                                                  _ptr(epd_y), _ptr(sfd_dy), _ptr(epd_dy), _ptr(dw), _stream(stream)))


def occult_dispatch_backward(cfg, plan, epd_dx, sfd_dx, dx_shared, dx, stream=None) -> None:
    _check(load_library().occult_dispatch_backward(ctypes.byref(cfg), ctypes.byref(plan), _ptr(epd_dx), _ptr(sfd_dx),
                                                   _ptr(dx_shared), _ptr(dx), _stream(stream)))


def occult_route_backward(cfg, logits, ids, dw, dlogits, stream=None) -> None:
    _check(load_library().occult_route_backward(ctypes.byref(cfg), _ptr(logits), _ptr(ids), _ptr(dw), _ptr(dlogits),
                                                _stream(stream)))


def occult_transpose_weights(cfg, w_gate, w_up, w_down, w_down_t, w_gu_t, stream=None) -> None:
    wts = occult_weights_t(_ptr(w_gate), _ptr(w_up), _ptr(w_down))
    _check(load_library().occult_transpose_weights(ctypes.byref(cfg), ctypes.byref(wts), _ptr(w_down_t), _ptr(w_gu_t),
                                                   _stream(stream)))


def occult_expert_ffn_train(cfg, plan, sfd_x, x, w_gate, w_up, w_down, epd_h, epd_y, h_shared, y_shared, epd_gu, gu_shared,
                            ws=None, stream=None) -> None:
    wts = occult_weights_t(_ptr(w_gate), _ptr(w_up), _ptr(w_down))
    nbytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().occult_expert_ffn_train(ctypes.byref(cfg), ctypes.byref(plan), _ptr(sfd_x), _ptr(x),
                                                  ctypes.byref(wts), _ptr(epd_h), _ptr(epd_y), _ptr(h_shared),
                                                  _ptr(y_shared), _ptr(epd_gu), _ptr(gu_shared), _ptr(ws), nbytes,
                                                  _stream(stream)))


def occult_expert_ffn_backward(cfg, plan, sfd_x, x, w_gate, w_up, w_down_t, w_gu_t, epd_dy, dy, epd_gu, epd_dh, epd_dx,
                               gu_shared=None, dh_shared=None, dx_shared=None, gu_saved=False, stream=None) -> None:
    wts = occult_weights_t(_ptr(w_gate), _ptr(w_up), None)
    _check(load_library().occult_expert_ffn_backward(ctypes.byref(cfg), ctypes.byref(plan), _ptr(sfd_x), _ptr(x),
                                                     ctypes.byref(wts), _ptr(w_down_t), _ptr(w_gu_t), _ptr(epd_dy),
                                                     _ptr(dy), _ptr(epd_gu), _ptr(epd_dh), _ptr(epd_dx), _ptr(gu_shared),
                                                     _ptr(dh_shared), _ptr(dx_shared), int(bool(gu_saved)),
                                                     _stream(stream)))


def occult_expert_ffn_backward_weights(cfg, plan, sfd_x, x, epd_h, h_shared, epd_dy, dy, epd_gu, gu_shared, dw_gate,
                                       dw_up, dw_down, accumulate=False, stream=None) -> None:
    _check(load_library().occult_expert_ffn_backward_weights(
        ctypes.byref(cfg), ctypes.byref(plan), _ptr(sfd_x), _ptr(x), _ptr(epd_h), _ptr(h_shared), _ptr(epd_dy), _ptr(dy),
        _ptr(epd_gu), _ptr(gu_shared), _ptr(dw_gate), _ptr(dw_up), _ptr(dw_down), int(bool(accumulate)), _stream(stream)))


def occult_expert_ffn_backward_weights_ws_bytes(cfg) -> int:
    n = c_size_t(0)
    _check(load_library().occult_expert_ffn_backward_weights_ws_bytes(ctypes.byref(cfg), ctypes.byref(n)))
    return int(n.value)


def occult_expert_ffn_backward_weights_ws(cfg, plan, sfd_x, x, epd_h, h_shared, epd_dy, dy, epd_gu, gu_shared, dw_gate,
                                          dw_up, dw_down, ws, accumulate=False, stream=None) -> None:
    nbytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().occult_expert_ffn_backward_weights_ws(
        ctypes.byref(cfg), ctypes.byref(plan), _ptr(sfd_x), _ptr(x), _ptr(epd_h), _ptr(h_shared), _ptr(epd_dy), _ptr(dy),
        _ptr(epd_gu), _ptr(gu_shared), _ptr(dw_gate), _ptr(dw_up), _ptr(dw_down), int(bool(accumulate)), _ptr(ws), nbytes,
        _stream(stream)))


def occult_coactivation(cfg, ids, C, accumulate: bool = False, stream=None) -> None:
    _check(load_library().occult_coactivation(ctypes.byref(cfg), _ptr(ids), _ptr(C), int(accumulate),
                                              _stream(stream)))


def occult_placement_greedy(C_host, D: int):
    """C_host: numpy int32 [E, E] (host).  Returns (L [D, G] int32, expert_pos [E] int32)."""
    import numpy as np
    C_host = np.ascontiguousarray(C_host, dtype=np.int32)
    E = C_host.shape[0]
    if D <= 0 or E % D:
        L = np.zeros((max(D, 1), 1), dtype=np.int32)
    else:
        L = np.zeros((D, E // D), dtype=np.int32)
    pos = np.zeros(E, dtype=np.int32)
    _check(load_library().occult_placement_greedy(C_host.ctypes.data, E, D, L.ctypes.data, pos.ctypes.data))
    return L, pos


def occult_collaboration_stats(C_host, D: int, expert_pos_host=None):
    """C_host: numpy int32 [E, E]; expert_pos_host: numpy int32 [E] or None (contiguous).
    Returns (c_intra [D], c_inter [D, D], intra_fraction) as computed by the library on the host."""
    import numpy as np
    C_host = np.ascontiguousarray(C_host, dtype=np.int32)
    E = C_host.shape[0]
    pos = None if expert_pos_host is None else np.ascontiguousarray(expert_pos_host, dtype=np.int32)
    c_intra = np.zeros(max(D, 1), dtype=np.float64)
    c_inter = np.zeros((max(D, 1), max(D, 1)), dtype=np.float64)
    frac = c_double(0.0)
    _check(load_library().occult_collaboration_stats(C_host.ctypes.data, E, D, None if pos is None else pos.ctypes.data,
                                                     c_intra.ctypes.data, c_inter.ctypes.data,
                                                     ctypes.addressof(frac)))
    return c_intra, c_inter, float(frac.value)


def occult_plan_stats(cfg, plan, stream=None) -> occult_stats_t:
    st = occult_stats_t()
    _check(load_library().occult_plan_stats(ctypes.byref(cfg), ctypes.byref(plan), ctypes.byref(st),
                                            _stream(stream)))
    return st
