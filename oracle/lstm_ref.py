"""The non-linear block of one LSTM cell, forward and backward.

TEST INFRASTRUCTURE.  Plain NumPy in float64, shares no code with the HIP path.

What is computed (Section 2 of the paper, the LSTM cell: the two fully-connected outputs, each four times the
hidden size, enter a block of slicing and element-wise operations together with the previous cell state and
leave it as the new hidden and cell state; the paper prints no formula for the block, so the textbook cell of
Hochreiter and Schmidhuber with a forget gate is used, gates sliced in the order input, forget, candidate,
output):

  a        = Gx + Gh                                 [B, 4H]  summed pre-activations
  i, f, o  = sigmoid(a[:, 0:H]), sigmoid(a[:, H:2H]), sigmoid(a[:, 3H:4H])
  g        = tanh(a[:, 2H:3H])
  c        = f * c_prev + i * g                      new cell state
  h        = o * tanh(c)                             new hidden state

The backward pass starts from dh, dc (the gradient that reaches c from the next time step) and returns the
gradient with respect to a (equal to the gradient of Gx and of Gh, the add passes it through) and c_prev:

  tc = tanh(c);  do = dh * tc;  dct = dc + dh * o * (1 - tc^2)
  di = dct * g;  dg = dct * i;  df = dct * c_prev;  dc_prev = dct * f
  da = [di * i (1 - i),  df * f (1 - f),  dg * (1 - g^2),  do * o (1 - o)]

Only a and c_prev are needed for that: every activation is a function of them (Section 4.1: keep the single
sum rather than the two addends).  `backward` therefore re-evaluates the forward pass from a and c_prev.

Pins (tests/test_oracle_lstm.py): central finite differences on every input, a per-element loop that uses
math.exp and math.tanh only, PyTorch's own LSTM cell in float64 (a library routine this block reduces to when
the weights are identities), closed forms at a = 0 and at saturated gates, no NaN at |a| = 1000.
"""
from __future__ import annotations

import numpy as np


def sigmoid(x: np.ndarray) -> np.ndarray:
    """1 / (1 + exp(-x)) without overflow for large |x|."""
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(-np.abs(x))
    return np.where(x >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


def activations(a: np.ndarray, c_prev: np.ndarray):
    """a [B, 4H], c_prev [B, H] -> i, f, g, o, c, tanh(c), each [B, H]."""
    a = np.asarray(a, dtype=np.float64)
    c_prev = np.asarray(c_prev, dtype=np.float64)
    H = c_prev.shape[-1]
    assert a.shape[-1] == 4 * H
    i = sigmoid(a[..., 0:H])
    f = sigmoid(a[..., H:2 * H])
    g = np.tanh(a[..., 2 * H:3 * H])
    o = sigmoid(a[..., 3 * H:4 * H])
    c = f * c_prev + i * g
    return i, f, g, o, c, np.tanh(c)


def forward(Gx: np.ndarray, Gh: np.ndarray, c_prev: np.ndarray):
    """-> h [B, H], c [B, H], a [B, 4H] (the tensor kept for the backward pass)."""
    a = np.asarray(Gx, dtype=np.float64) + np.asarray(Gh, dtype=np.float64)
    i, f, g, o, c, tc = activations(a, c_prev)
    return o * tc, c, a


def backward(dh: np.ndarray, dc: np.ndarray, a: np.ndarray, c_prev: np.ndarray):
    """-> da [B, 4H], dc_prev [B, H]; the activations are re-evaluated from a and c_prev."""
    dh = np.asarray(dh, dtype=np.float64)
    dc = np.asarray(dc, dtype=np.float64)
    c_prev = np.asarray(c_prev, dtype=np.float64)
    i, f, g, o, c, tc = activations(a, c_prev)
    do = dh * tc
    dct = dc + dh * o * (1.0 - tc * tc)
    di, dg, df = dct * g, dct * i, dct * c_prev
    da = np.concatenate([di * i * (1.0 - i), df * f * (1.0 - f), dg * (1.0 - g * g), do * o * (1.0 - o)], axis=-1)
    return da, dct * f


def kept_elements(B: int, H: int, recompute: bool) -> int:
    """Elements one cell keeps between its forward and backward pass, the previous cell state included:
    a and c_prev when the activations are recomputed; the four activations, tanh(c) and c_prev otherwise."""
    return (4 + 1) * B * H if recompute else (4 + 1 + 1) * B * H
