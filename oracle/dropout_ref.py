"""Dropout whose feature map is one bit per element.

TEST INFRASTRUCTURE.  Plain NumPy, shares no code with the HIP path.

What is computed (Section 5.2 of the paper: the feature maps of dropout layers are encoded to 1 bit in the
forward pass and decoded back to 32 bits in the backward pass; the paper takes the encoding from Gist and
prints no formula, so the definition of inverted dropout is used):

  keep_i = (u_i >= p)                              u_i uniform in [0, 1)
  y_i    = keep_i ? x_i / (1 - p) : 0              forward output
  bits   : bit (i mod 32) of 32-bit word (i div 32) = keep_i     -- all that is kept for the backward pass
  dx_i   = keep_i ? dy_i / (1 - p) : 0             backward, from the bits alone

The random numbers come from a counter-based generator so that both sides can draw the same ones without
exchanging them: Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
SC 2011).  Element i uses output word (i mod 4) of the block with counter (i div 4 as 64 bits, offset as 64
bits) and key = seed; u = (word >> 8) * 2^-24, compared with p in float32 (the decision is taken in the same
precision on both sides).

Pins (tests/test_oracle_dropout.py): the generator against the known-answer vectors of its authors, the bit
order against a per-element loop, the kept fraction against 1 - p, p = 0 as the identity, bwd as the adjoint
of fwd.
"""
from __future__ import annotations

import numpy as np

M0, M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)      # round multipliers
W0, W1 = np.uint32(0x9E3779B9), np.uint32(0xBB67AE85)      # key increments (golden ratio, sqrt(3) - 1)
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(counter: np.ndarray, key: np.ndarray) -> np.ndarray:
    """counter [..., 4] uint32, key [..., 2] uint32 (broadcastable) -> [..., 4] uint32."""
    c = [np.asarray(counter[..., k], dtype=np.uint32) for k in range(4)]
    k0 = np.asarray(key[..., 0], dtype=np.uint32)
    k1 = np.asarray(key[..., 1], dtype=np.uint32)
    with np.errstate(over="ignore"):
        for rnd in range(10):
            if rnd > 0:
                k0 = (k0 + W0).astype(np.uint32)
                k1 = (k1 + W1).astype(np.uint32)
            p0 = M0 * c[0].astype(np.uint64)
            p1 = M1 * c[2].astype(np.uint64)
            hi0, lo0 = (p0 >> np.uint64(32)).astype(np.uint32), (p0 & _MASK32).astype(np.uint32)
            hi1, lo1 = (p1 >> np.uint64(32)).astype(np.uint32), (p1 & _MASK32).astype(np.uint32)
            c = [hi1 ^ c[1] ^ k0, lo1, hi0 ^ c[3] ^ k1, lo0]
    return np.stack(c, axis=-1)


def uniforms(n: int, seed: int, offset: int) -> np.ndarray:
    """u_0 .. u_{n-1} as float32 in [0, 1)."""
    nblk = (n + 3) // 4
    idx = np.arange(nblk, dtype=np.uint64)
    ctr = np.empty((nblk, 4), dtype=np.uint32)
    ctr[:, 0] = (idx & _MASK32).astype(np.uint32)
    ctr[:, 1] = (idx >> np.uint64(32)).astype(np.uint32)
    ctr[:, 2] = np.uint32(offset & 0xFFFFFFFF)
    ctr[:, 3] = np.uint32((offset >> 32) & 0xFFFFFFFF)
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint32)
    words = philox4x32_10(ctr, key).reshape(-1)[:n]
    return ((words >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)).astype(np.float32)


def keep_flags(n: int, p: float, seed: int, offset: int) -> np.ndarray:
    return uniforms(n, seed, offset) >= np.float32(p)


def pack_bits(keep: np.ndarray) -> np.ndarray:
    """bit (i mod 32) of word (i div 32) = keep_i; the last word is zero-padded."""
    n = keep.shape[0]
    padded = np.zeros((n + 31) // 32 * 32, dtype=np.uint8)
    padded[:n] = keep
    return np.packbits(padded.reshape(-1, 32), axis=1, bitorder="little").view(np.uint32).reshape(-1)


def unpack_bits(bits: np.ndarray, n: int) -> np.ndarray:
    b = np.unpackbits(np.ascontiguousarray(bits, dtype=np.uint32).view(np.uint8).reshape(-1, 4), axis=1,
                      bitorder="little")
    return b.reshape(-1)[:n].astype(bool)


def forward(x: np.ndarray, p: float, seed: int, offset: int):
    """Returns (y float64 [n], bits uint32 [ceil(n/32)])."""
    x = np.asarray(x, dtype=np.float64).reshape(-1)
    keep = keep_flags(x.shape[0], p, seed, offset)
    y = np.where(keep, x / (1.0 - float(np.float32(p))), 0.0)
    return y, pack_bits(keep)


def backward(dy: np.ndarray, bits: np.ndarray, p: float):
    """dx float64 [n] from the one-bit feature map."""
    dy = np.asarray(dy, dtype=np.float64).reshape(-1)
    keep = unpack_bits(bits, dy.shape[0])
    return np.where(keep, dy / (1.0 - float(np.float32(p))), 0.0)
