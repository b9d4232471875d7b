"""Seeded synthetic inputs for the additive-attention layer.

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: it only draws random tensors of the shapes
and value distributions of the five workloads and rounds them to the storage
type.  It imports neither the binding nor the oracle.

The workloads stand in for the attention layer of the LSTM translation model
of the paper (Section 2, attention steps 1-2; Section 5.1 gives the usual
sequence length of 50-100 and Section 6.2 the batch size of 128); the paper's
corpora and trained weights are not used: cost and numerics of the layer
depend only on shapes, storage type and the key lengths.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict

import numpy as np

SEED_BASE = 18050889900


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Tq: int
    Tk: int
    H: int
    Dv: int
    in_dtype: str          # "f32" or "bf16": storage type of Qp, Kp, V, v
    scale: float           # std of Qp, Kp, V
    key_lo: int            # key_len ~ U{key_lo..key_hi}, both ends included
    key_hi: int
    v_normal: bool = False  # v ~ scale*N(0,1) instead of U(-1/sqrt(H), 1/sqrt(H))

    @property
    def n4(self) -> int:
        """Elements of the 4-D tanh feature map B x Tq x Tk x H."""
        return self.B * self.Tq * self.Tk * self.H


WORKLOADS = (
    Workload("cfg0_tiny_f32", 4, 6, 7, 16, 16, "f32", 0.5, 1, 7),
    Workload("cfg1_nmt_f32_B64_T50_H512", 64, 50, 50, 512, 512, "f32", 0.5, 10, 50),
    Workload("cfg2_large_batch_f32_B128_T100_H512", 128, 100, 100, 512, 512, "f32", 0.5, 20, 100),
    Workload("cfg3_long_f32_B32_T300_H1024", 32, 300, 300, 1024, 1024, "f32", 0.3, 150, 300),
    Workload("cfg4_bf16_B128_T50_H1024", 128, 50, 50, 1024, 1024, "bf16", 0.5, 5, 50, True),
)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns the
    16-bit patterns as uint16.  NaN/inf do not occur in the generated data."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_inputs(wl: Workload, seed: int | None = None, *, B: int | None = None) -> Dict[str, np.ndarray]:
    """Draw one batch for `wl`.

    Draw order is fixed: Qp, Kp, V, v, key_len, dContext.  Returned arrays:
      Qp [B,Tq,H], Kp [B,Tk,H], V [B,Tk,Dv], v [H]  float32 holding the values
          the layer consumes (for "bf16" workloads already rounded to bf16);
      Qp_bits, Kp_bits, V_bits, v_bits  uint16 bf16 patterns ("bf16" only);
      key_len [B] int32;  dContext [B,Tq,Dv] float32.
    `B` overrides the batch size (same stream prefix is NOT guaranteed).
    """
    idx = WORKLOADS.index(wl) if wl in WORKLOADS else 99
    rng = np.random.default_rng(SEED_BASE + idx if seed is None else seed)
    nb = wl.B if B is None else B
    f32 = np.float32
    Qp = (rng.standard_normal((nb, wl.Tq, wl.H)) * wl.scale).astype(f32)
    Kp = (rng.standard_normal((nb, wl.Tk, wl.H)) * wl.scale).astype(f32)
    V = (rng.standard_normal((nb, wl.Tk, wl.Dv)) * wl.scale).astype(f32)
    if wl.v_normal:
        v = (rng.standard_normal(wl.H) * wl.scale).astype(f32)
    else:
        a = 1.0 / np.sqrt(wl.H)
        v = rng.uniform(-a, a, wl.H).astype(f32)
    key_len = rng.integers(wl.key_lo, wl.key_hi + 1, nb).astype(np.int32)
    dC = rng.standard_normal((nb, wl.Tq, wl.Dv)).astype(f32)
    out = {"Qp": Qp, "Kp": Kp, "V": V, "v": v, "key_len": key_len, "dContext": dC}
    if wl.in_dtype == "bf16":
        for k in ("Qp", "Kp", "V", "v"):
            bits = round_to_bf16(out[k])
            out[k + "_bits"] = bits
            out[k] = bf16_bits_to_f32(bits)
    return out


def make_lstm_inputs(B: int, H: int, seed: int, scale: float = 1.0) -> Dict[str, np.ndarray]:
    """One LSTM cell's worth of inputs (Section 2: two fully-connected outputs of four times the hidden size,
    the previous cell state) and the two upstream gradients.  Draw order: Gx, Gh, c_prev, dh, dc; float32.
    The translation model of the paper runs its cells at batch size 128 (Section 6.2); the pre-activations of a
    trained cell are of order one, which `scale` = 1 stands in for."""
    rng = np.random.default_rng(SEED_BASE + 1000 + seed)
    f32 = np.float32
    return {
        "Gx": (rng.standard_normal((B, 4 * H)) * scale).astype(f32),
        "Gh": (rng.standard_normal((B, 4 * H)) * scale).astype(f32),
        "c_prev": rng.standard_normal((B, H)).astype(f32),
        "dh": rng.standard_normal((B, H)).astype(f32),
        "dc": rng.standard_normal((B, H)).astype(f32),
    }
