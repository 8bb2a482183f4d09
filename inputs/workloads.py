"""Seeded synthetic MoE-layer workloads (inputs only).

This module draws random numbers and shapes them; it holds none of the layer's
routing, planning, dispatch, expert or combine arithmetic.  Both the CPU oracle
(through the tests) and the GPU path (through the tests and the benchmark)
read their inputs from here, so the two sides see identical bits.

The shapes follow the MoE-LLMs the paper evaluates (its Table 2: top-k and
expert counts of Qwen1.5-MoE 4/60, DeepSeek-MoE 6/64, OLMoE 8/64) and the
2**14-token prefill of its Table 1.  None of the paper's datasets or model
weights is used: hidden states are a Gaussian mixture, so that expert loads
and co-activation are skewed the way trained routers skew them, and weights
are Gaussian.

Draw order for one workload (one ``numpy.random.default_rng(seed)`` stream):
mixture means [components, d] -> component id per token [T] -> noise [T, d]
-> router weight W_r [E, d] -> for e in 0..E+S-1: W_gate[e] [f, d],
W_up[e] [f, d], W_down[e] [d, f].

Router scores ("logits") are produced here once, as the float32 product of the
stored hidden states and W_r, and handed to both sides as an input: the
boundary's routing call starts from router scores (the paper treats the router
as a black box that returns ids and weights).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np

SEED = 13345


@dataclasses.dataclass(frozen=True)
class LayerShape:
    name: str
    T: int          # tokens
    d: int          # hidden size
    f: int          # expert intermediate size
    E: int          # routed experts
    S: int          # shared experts (always active)
    k: int          # top-k
    D: int          # simulated devices
    dtype: str      # "f32" or "bf16" storage of x / weights / activations
    components: int  # Gaussian-mixture components (0 = plain N(0, 1/d) tokens)
    n_d: int = 0    # collaboration pruning: 0 = off, else max devices per token
    prune_mode: int = 1
    renorm: int = 1

    @property
    def G(self) -> int:
        return self.E // self.D


# The five benchmark configurations.
CONFIGS = {
    "tiny_f32": LayerShape("tiny_f32", T=256, d=128, f=256, E=16, S=0, k=4, D=4,
                           dtype="f32", components=0),
    "decode_bf16": LayerShape("decode_bf16", T=128, d=2048, f=1408, E=60, S=4, k=4, D=4,
                              dtype="bf16", components=16),
    "prefill_bf16": LayerShape("prefill_bf16", T=16384, d=2048, f=1024, E=64, S=0, k=8, D=8,
                               dtype="bf16", components=32),
    "prefill_pruned_bf16": LayerShape("prefill_pruned_bf16", T=16384, d=2048, f=1024, E=64, S=0,
                                      k=8, D=8, dtype="bf16", components=32, n_d=2),
    "large_bf16": LayerShape("large_bf16", T=65536, d=2048, f=1408, E=64, S=2, k=6, D=16,
                             dtype="bf16", components=64),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


@dataclasses.dataclass
class Workload:
    shape: LayerShape
    x: np.ndarray                   # [T, d] float32 (bf16-representable when dtype == "bf16")
    w_router: np.ndarray            # [E, d] float32
    logits: np.ndarray              # [T, E] float32 router scores
    w_gate: Optional[np.ndarray]    # [E+S, f, d] float32
    w_up: Optional[np.ndarray]      # [E+S, f, d]
    w_down: Optional[np.ndarray]    # [E+S, d, f]


def make_workload(shape: LayerShape, seed: int = SEED, with_experts: bool = True,
                  w_down_gain: Optional[float] = None) -> Workload:
    """Draw one layer's inputs.  ``with_experts=False`` skips the expert weights
    (routing / planning / dispatch tests do not need them)."""
    rng = np.random.default_rng(seed)
    T, d, f, E, S = shape.T, shape.d, shape.f, shape.E, shape.S
    inv_sqrt_d = np.float32(1.0 / math.sqrt(d))
    if shape.components > 0:
        means = rng.standard_normal((shape.components, d), dtype=np.float32)
        comp = rng.integers(0, shape.components, size=T)
        noise = rng.standard_normal((T, d), dtype=np.float32)
        x = means[comp] + np.float32(0.5) * noise
        del noise
    else:
        x = rng.standard_normal((T, d), dtype=np.float32) * inv_sqrt_d
    w_router = rng.standard_normal((E, d), dtype=np.float32) * inv_sqrt_d
    bf16 = shape.dtype == "bf16"
    if bf16:
        x = round_to_bf16(x)
        w_router = round_to_bf16(w_router)
    logits = (x @ w_router.T).astype(np.float32)

    w_gate = w_up = w_down = None
    if with_experts:
        n = E + S
        if w_down_gain is None:
            # tiny f32 layer: every weight N(0, 1/d); bf16 layers: a quarter of fan-in scaling
            # so that outputs stay O(1) and bf16 output quantisation sits well inside tolerance
            down_std = inv_sqrt_d if not bf16 else np.float32(0.25 / math.sqrt(f))
        else:
            down_std = np.float32(w_down_gain / math.sqrt(f))
        w_gate = np.empty((n, f, d), dtype=np.float32)
        w_up = np.empty((n, f, d), dtype=np.float32)
        w_down = np.empty((n, d, f), dtype=np.float32)
        for e in range(n):
            w_gate[e] = rng.standard_normal((f, d), dtype=np.float32) * inv_sqrt_d
            w_up[e] = rng.standard_normal((f, d), dtype=np.float32) * inv_sqrt_d
            w_down[e] = rng.standard_normal((d, f), dtype=np.float32) * down_std
        if bf16:
            for e in range(n):
                w_gate[e] = round_to_bf16(w_gate[e])
                w_up[e] = round_to_bf16(w_up[e])
                w_down[e] = round_to_bf16(w_down[e])
    return Workload(shape, x, w_router, logits, w_gate, w_up, w_down)


def contiguous_placement(E: int, D: int) -> np.ndarray:
    """expert_pos[e] = e: expert e sits on device e // (E/D) in slot e % (E/D)."""
    return np.arange(E, dtype=np.int32)


def random_placement(E: int, D: int, seed: int) -> np.ndarray:
    """A seeded random permutation of placement positions (device = pos // G, slot = pos % G)."""
    return np.random.default_rng(seed).permutation(E).astype(np.int32)


def random_logits(T: int, E: int, seed: int, scale: float = 1.0, ties: bool = False) -> np.ndarray:
    """Plain Gaussian router scores; ``ties=True`` quantises them coarsely so that equal
    scores occur and the tie rule is exercised."""
    rng = np.random.default_rng(seed)
    lg = (rng.standard_normal((T, E), dtype=np.float32) * np.float32(scale)).astype(np.float32)
    if ties:
        lg = (np.round(lg * 2.0) / 2.0).astype(np.float32)
    return lg


def integer_valued_rows(T: int, d: int, seed: int, lo: int = -4, hi: int = 4) -> np.ndarray:
    """Small-integer hidden states: every sum of a few of them is exact in bf16 and f32."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=(T, d)).astype(np.float32)
