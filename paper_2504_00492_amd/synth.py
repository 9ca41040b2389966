"""Seeded synthetic workloads shaped like the multi-head [L, R, d] drivers of the low-rank delta
rule (ParallelFlow, arXiv 2504.00492, Section 3.1).

This module only draws and rounds numbers.  It holds none of the method's arithmetic and is the
one module both the GPU tests/bench and the CPU oracle's callers take their inputs from.

Recipe per head (counter-based Philox stream keyed by (workload seed, head index), draws in
this fixed order): q ~ N(0,1)/sqrt(d_k); k ~ N(0,1), each key L2-normalised in fp32;
v ~ N(0,1)/sqrt(d_v); beta = sigmoid(N(0,1)); optional S0 ~ N(0, s0_std^2); optional
"near-reflection" tokens: Bernoulli(reflect_frac) per token, on which all R betas are redrawn
from U(1.5, 2.0).  For a bf16 workload q, k, v, beta are then rounded once to bf16
(round-to-nearest-even); the rounded values are what both sides see.  S0 stays fp32.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str          # "f32" or "bf16": element type of Q, K, V, beta, O
    B: int
    H: int
    L: int
    d_k: int
    d_v: int
    r: int
    chunk: int
    seed: int
    s0_std: float = 0.0        # 0 => S0 = 0 (passed as None)
    reflect_frac: float = 0.0  # fraction of tokens whose betas are drawn from U(1.5, 2)

    @property
    def heads(self) -> int:
        return self.B * self.H

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    "cfg0": Workload("cfg0", "f32", 1, 1, 64, 16, 16, 1, 16, seed=0),
    "cfg1": Workload("cfg1", "bf16", 4, 8, 2048, 64, 64, 1, 64, seed=1),
    "cfg2": Workload("cfg2", "bf16", 4, 16, 4096, 128, 128, 2, 64, seed=2),
    "cfg3a": Workload("cfg3a", "bf16", 2, 16, 8192, 128, 128, 4, 64, seed=3, s0_std=0.1),
    "cfg3b": Workload("cfg3b", "bf16", 2, 16, 8192, 128, 128, 4, 128, seed=3, s0_std=0.1),
    "cfg4": Workload("cfg4", "bf16", 1, 32, 65536, 128, 128, 2, 128, seed=4, reflect_frac=0.1),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bf16 (ties to even), returned as fp32 values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) & np.uint32(0xFFFF0000)).view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 values that are exactly bf16-representable -> their 16-bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def head_inputs(w: Workload, head: int):
    """Inputs of one head as fp32 arrays: q [L,dk], k [L,r,dk], v [L,r,dv], beta [L,r],
    s0 [dv,dk] or None.  Deterministic in (w.seed, head) alone."""
    g = np.random.Generator(np.random.Philox(key=[np.uint64(w.seed), np.uint64(head)]))
    L, r, dk, dv = w.L, w.r, w.d_k, w.d_v
    q = g.standard_normal((L, dk), dtype=np.float32) * np.float32(1.0 / np.sqrt(dk))
    k = g.standard_normal((L, r, dk), dtype=np.float32)
    k /= np.sqrt(np.sum(k * k, axis=-1, keepdims=True, dtype=np.float32))
    v = g.standard_normal((L, r, dv), dtype=np.float32) * np.float32(1.0 / np.sqrt(dv))
    z = g.standard_normal((L, r), dtype=np.float32)
    beta = (np.float32(1.0) / (np.float32(1.0) + np.exp(-z))).astype(np.float32)
    s0 = None
    if w.s0_std > 0.0:
        s0 = g.standard_normal((dv, dk), dtype=np.float32) * np.float32(w.s0_std)
    if w.reflect_frac > 0.0:
        pick = g.random(L, dtype=np.float32) < np.float32(w.reflect_frac)
        u = np.float32(1.5) + np.float32(0.5) * g.random((L, r), dtype=np.float32)
        beta = np.where(pick[:, None], u, beta).astype(np.float32)
    if w.dtype == "bf16":
        q, k, v, beta = (round_to_bf16(a) for a in (q, k, v, beta))
    return q, k, v, beta, s0


def make_inputs(w: Workload, heads=None):
    """Stack head_inputs over `heads` (default: all B*H heads, in (b, h) order).

    Returns dict of fp32 arrays with a leading head axis N: Q [N,L,dk], K [N,L,r,dk],
    V [N,L,r,dv], beta [N,L,r], S0 [N,dv,dk] or None."""
    ids = list(range(w.heads)) if heads is None else list(heads)
    N = len(ids)
    Q = np.empty((N, w.L, w.d_k), np.float32)
    K = np.empty((N, w.L, w.r, w.d_k), np.float32)
    V = np.empty((N, w.L, w.r, w.d_v), np.float32)
    beta = np.empty((N, w.L, w.r), np.float32)
    S0 = np.empty((N, w.d_v, w.d_k), np.float32) if w.s0_std > 0.0 else None
    for i, h in enumerate(ids):
        q, k, v, b, s0 = head_inputs(w, h)
        Q[i], K[i], V[i], beta[i] = q, k, v, b
        if S0 is not None:
            S0[i] = s0
    return {"Q": Q, "K": K, "V": V, "beta": beta, "S0": S0}
