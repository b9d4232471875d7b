"""Plain float64 definition of additive (MLP) attention, forward and backward.

TEST INFRASTRUCTURE.  Slow, obviously-correct NumPy; one sample of the batch at
a time so that the largest live array is one sample's Tq x Tk x H map.  Shares
no code with the HIP path.

What is computed (the recompute-in-backward of the paper changes what is kept
in memory, not any value -- Section 7, Related Work, "Algorithm Changes"):

  scoring       a broadcast add of every query row with every key row followed
                by tanh (Section 4.1, the figure with T tensors of shape [N]
                added to one [T x N] tensor; Section 2, attention step 1),
                then a projection onto the vector v (a fully-connected layer
                with one output, Eq. 1 without bias);
  weights       softmax over the keys of one sample that are inside its key
                length (Section 2, the weights alpha_ts of step 1);
  context       weights-weighted average of the value rows (Section 2, step 2).

Backward rules used: tanh' = 1 - tanh^2 (Section 3.2, feature maps), the
fully-connected / batched-dot gradients that need only the layer inputs
(Eq. 2, Section 5.2), and the softmax Jacobian.

Pins (tests/test_oracle*.py): central finite differences, an independent
per-element loop, closed forms (v = 0, one valid key, the linear regime of
tanh), softmax and conservation invariants, permutation equivariance, and a
PyTorch float64 autograd cross-check.  The paper prints no worked numeric
example of this layer, so no value here is pinned by the paper itself.
"""
from __future__ import annotations

import numpy as np


def _valid_len(key_len_b, Tk: int) -> int:
    """Number of keys that take part: key_len clamped to [0, Tk]."""
    return int(min(max(int(key_len_b), 0), Tk))


def tanh_map(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """T4[i, j, h] = tanh(q[i, h] + k[j, h]) for one sample (the feature map
    that the baseline stashes and the recompute path never stores)."""
    return np.tanh(q[:, None, :] + k[None, :, :])


def sample_forward(q, k, val, v, L):
    """One sample.  q [Tq,H], k [Tk,H], val [Tk,Dv], v [H], L valid keys.
    Returns (context [Tq,Dv], P [Tq,Tk], S [Tq,L])."""
    Tq, Tk = q.shape[0], k.shape[0]
    P = np.zeros((Tq, Tk), dtype=np.float64)
    C = np.zeros((Tq, val.shape[1]), dtype=np.float64)
    if L == 0:
        return C, P, np.zeros((Tq, 0), dtype=np.float64)
    T4 = tanh_map(q, k[:L])                    # [Tq, L, H]
    S = T4 @ v                                 # [Tq, L]
    m = S.max(axis=1, keepdims=True)
    e = np.exp(S - m)
    P[:, :L] = e / e.sum(axis=1, keepdims=True)
    C[:] = P[:, :L] @ val[:L]
    return C, P, S


def sample_backward(dC, P, q, k, val, v, L):
    """One sample.  Returns (dq [Tq,H], dk [Tk,H], dval [Tk,Dv], dv [H])."""
    dq = np.zeros_like(q, dtype=np.float64)
    dk = np.zeros_like(k, dtype=np.float64)
    dval = np.zeros_like(val, dtype=np.float64)
    dv = np.zeros(v.shape[0], dtype=np.float64)
    if L == 0:
        return dq, dk, dval, dv
    Pl = P[:, :L]
    dval[:L] = Pl.T @ dC                       # dV[j,:] = sum_i P[i,j] dC[i,:]
    dP = dC @ val[:L].T                        # dP[i,j] = sum_d dC[i,d] V[j,d]
    r = (Pl * dP).sum(axis=1, keepdims=True)
    dS = Pl * (dP - r)                         # softmax Jacobian
    T4 = tanh_map(q, k[:L])                    # recomputed, as the paper's backward does
    G = dS[:, :, None] * v[None, None, :] * (1.0 - T4 * T4)
    dq[:] = G.sum(axis=1)
    dk[:L] = G.sum(axis=0)
    dv[:] = np.einsum("ij,ijh->h", dS, T4)
    return dq, dk, dval, dv


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def forward(Qp, Kp, V, v, key_len):
    """Batch forward.  Returns (context [B,Tq,Dv], P [B,Tq,Tk]) in float64."""
    Qp, Kp, V, v = _f64(Qp), _f64(Kp), _f64(V), _f64(v)
    B, Tq, _ = Qp.shape
    Tk, Dv = Kp.shape[1], V.shape[2]
    C = np.zeros((B, Tq, Dv)); P = np.zeros((B, Tq, Tk))
    for b in range(B):
        C[b], P[b], _ = sample_forward(Qp[b], Kp[b], V[b], v, _valid_len(key_len[b], Tk))
    return C, P


def scores(Qp, Kp, v, key_len):
    """Unnormalised scores S[b,i,j]; entries at masked keys are -inf."""
    Qp, Kp, v = _f64(Qp), _f64(Kp), _f64(v)
    B, Tq, _ = Qp.shape
    Tk = Kp.shape[1]
    S = np.full((B, Tq, Tk), -np.inf)
    for b in range(B):
        L = _valid_len(key_len[b], Tk)
        if L:
            S[b, :, :L] = tanh_map(Qp[b], Kp[b, :L]) @ v
    return S


def backward(dContext, P, Qp, Kp, V, v, key_len):
    """Batch backward from the saved P.  Returns (dQp, dKp, dV, dv) in float64."""
    dC, P, Qp, Kp, V, v = map(_f64, (dContext, P, Qp, Kp, V, v))
    B, Tk = Qp.shape[0], Kp.shape[1]
    dQp = np.zeros_like(Qp); dKp = np.zeros_like(Kp); dV = np.zeros_like(V)
    dv = np.zeros_like(v)
    for b in range(B):
        L = _valid_len(key_len[b], Tk)
        dQp[b], dKp[b], dV[b], dvb = sample_backward(dC[b], P[b], Qp[b], Kp[b], V[b], v, L)
        dv += dvb
    return dQp, dKp, dV, dv


def forward_backward(Qp, Kp, V, v, key_len, dContext):
    """Convenience: forward, then backward from the oracle's own P."""
    C, P = forward(Qp, Kp, V, v, key_len)
    dQp, dKp, dV, dv = backward(dContext, P, Qp, Kp, V, v, key_len)
    return {"context": C, "P": P, "dQp": dQp, "dKp": dKp, "dV": dV, "dv": dv}


def loss(Qp, Kp, V, v, key_len, dContext) -> float:
    """Scalar sum(dContext * context): its gradient w.r.t. the inputs is what
    backward() returns; used by the finite-difference pin."""
    C, _ = forward(Qp, Kp, V, v, key_len)
    return float((_f64(dContext) * C).sum())
