"""Seeded synthetic inputs for the Blossom attention path.

This module only draws random numbers and rounds them to the storage type; it
contains none of the method's arithmetic (no pooling, scoring, masking, softmax
or gating).  It is the one module shared by the CPU oracle's tests and the HIP
path's tests/bench, so both sides read exactly the same bits.

The five workloads stand in for the paper's recommender histories (Sec. 4.1,
App. E: max length 200, hidden 64, a handful of selected blocks, window 8-16)
and extend its efficiency-study axis (Sec. 4.3, App. B: long sequences, one
layer) to L = 1024 and L = 8192.  Values are i.i.d. Gaussian, which spreads the
block scores almost uniformly, i.e. the selected blocks are scattered over the
whole past: the worst case for K/V locality.

Draw order per workload (numpy ``default_rng(seed)``, PCG64):
Q, K, V, valid_len, gate_w, dO.  ``gate_b`` is zero.  Pad positions hold
ordinary random values: the method must ignore them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    L: int
    d: int
    block: int          # b: query-block size == key-block size
    topk: int           # k: selected blocks per query block, diagonal included
    window: int         # w: query i sees keys j with 0 <= i-j < w
    dtype: str          # "fp32" | "bf16" (storage type of Q,K,V,O,dO)
    len_lo: int         # valid_len ~ U{len_lo..len_hi}
    len_hi: int
    qkv_scaled: bool    # True: Q,K,V ~ N(0,1)/sqrt(d); False: N(0,1)
    seed: int
    backward: bool = False
    stis_block: int = 0  # 0: the short-term mask is the causal window; >= 1: all of Eq. 15 with this mask block size
    bidir: bool = False  # True: bidirectional form (Eq. 15 as printed, no causal mask in either branch)

    @property
    def NB(self) -> int:
        return -(-self.L // self.block)


WORKLOADS = {
    "cfg1": Workload("cfg1", 4, 2, 50, 32, 8, 2, 8, "fp32", 10, 50, False, 1001),
    "cfg2": Workload("cfg2", 256, 2, 200, 32, 16, 4, 16, "fp32", 20, 200, False, 1002),
    "cfg3": Workload("cfg3", 128, 4, 1024, 64, 32, 8, 64, "bf16", 100, 1024, True, 1003),
    "cfg4": Workload("cfg4", 16, 8, 8192, 64, 64, 16, 128, "bf16", 8192, 8192, True, 1004),
    "cfg5": Workload("cfg5", 128, 4, 1024, 64, 32, 8, 64, "bf16", 100, 1024, True, 1005,
                     backward=True),
}


def with_shape(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (reduced parity cases)."""
    return replace(w, **kw)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).copy()
    u += np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    u &= np.uint32(0xFFFF0000)
    return u.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of bf16-representable fp32 values, as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns widened exactly to fp32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Inputs:
    w: Workload
    Q: np.ndarray          # [B,H,L,d] fp32 (bf16-representable when w.dtype == "bf16")
    K: np.ndarray
    V: np.ndarray
    valid_len: np.ndarray  # [B] int32, left padding: valid positions are L-n .. L-1
    gate_w: np.ndarray     # [H,2d] fp32
    gate_b: np.ndarray     # [H] fp32
    dO: np.ndarray         # [B,H,L,d] fp32 (bf16-representable when bf16), or None


def make_inputs(w: Workload, input_set: int = 0, want_dO: bool | None = None) -> Inputs:
    """Draw one input set.  ``input_set`` s uses seed + 100*s (bench rotation)."""
    rng = np.random.default_rng(w.seed + 100 * input_set)
    shape = (w.B, w.H, w.L, w.d)
    div = np.float32(np.sqrt(np.float32(w.d))) if w.qkv_scaled else np.float32(1.0)

    def tensor():
        x = rng.standard_normal(shape, dtype=np.float32)
        if w.qkv_scaled:
            x /= div
        return round_to_bf16(x) if w.dtype == "bf16" else x

    Q = tensor()
    K = tensor()
    V = tensor()
    valid_len = rng.integers(w.len_lo, w.len_hi + 1, size=w.B).astype(np.int32)
    gate_w = (rng.standard_normal((w.H, 2 * w.d), dtype=np.float32) * np.float32(0.02))
    gate_b = np.zeros(w.H, dtype=np.float32)
    if want_dO is None:
        want_dO = w.backward
    dO = None
    if want_dO:
        dO = rng.standard_normal(shape, dtype=np.float32)
        if w.dtype == "bf16":
            dO = round_to_bf16(dO)
    return Inputs(w, Q, K, V, valid_len, gate_w, gate_b, dO)


def rope_tables(L: int, d: int, base: float = 10000.0):
    """cos/sin tables [L, d/2] float32 of the rotary position embedding (Sec. 3.3): entry [m][i] holds the
    angle m * base**(-2i/d), evaluated in float64 and rounded once.  An input of both the oracle and
    the HIP path, like the gate weights; the rotation itself is theirs."""
    m = np.arange(L, dtype=np.float64)[:, None]
    inv = base ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)[None, :]
    ang = m * inv
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
