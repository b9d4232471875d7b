"""Per-element loops for additive attention, forward and backward.

TEST INFRASTRUCTURE, tiny inputs only.  Written independently of attn_ref.py
(scalar math from the standard library, no array operations) so that an
indexing or transposition mistake in either shows up as a disagreement.
Follows the same passages: Section 2 (attention steps 1-2), Section 4.1
(broadcast add + tanh), Section 3.2 (tanh' = 1 - tanh^2), Eq. 2.
"""
from __future__ import annotations

import math


def forward_backward(Qp, Kp, V, v, key_len, dC):
    """Nested-list / array inputs, indexed [b][i][h] etc.  Returns dict of
    nested lists: context, P, dQp, dKp, dV, dv."""
    B, Tq, H = len(Qp), len(Qp[0]), len(v)
    Tk, Dv = len(Kp[0]), len(V[0][0])
    ctx = [[[0.0] * Dv for _ in range(Tq)] for _ in range(B)]
    P = [[[0.0] * Tk for _ in range(Tq)] for _ in range(B)]
    dQ = [[[0.0] * H for _ in range(Tq)] for _ in range(B)]
    dK = [[[0.0] * H for _ in range(Tk)] for _ in range(B)]
    dV = [[[0.0] * Dv for _ in range(Tk)] for _ in range(B)]
    dv = [0.0] * H
    for b in range(B):
        L = min(max(int(key_len[b]), 0), Tk)
        if L == 0:
            continue
        for i in range(Tq):
            s = []
            for j in range(L):
                acc = 0.0
                for h in range(H):
                    acc += float(v[h]) * math.tanh(float(Qp[b][i][h]) + float(Kp[b][j][h]))
                s.append(acc)
            m = max(s)
            e = [math.exp(x - m) for x in s]
            z = sum(e)
            for j in range(L):
                P[b][i][j] = e[j] / z
            for d in range(Dv):
                ctx[b][i][d] = sum(P[b][i][j] * float(V[b][j][d]) for j in range(L))
            # backward for this query row
            dp = [sum(float(dC[b][i][d]) * float(V[b][j][d]) for d in range(Dv)) for j in range(L)]
            r = sum(P[b][i][j] * dp[j] for j in range(L))
            for j in range(L):
                ds = P[b][i][j] * (dp[j] - r)
                for d in range(Dv):
                    dV[b][j][d] += P[b][i][j] * float(dC[b][i][d])
                for h in range(H):
                    t = math.tanh(float(Qp[b][i][h]) + float(Kp[b][j][h]))
                    g = ds * float(v[h]) * (1.0 - t * t)
                    dQ[b][i][h] += g
                    dK[b][j][h] += g
                    dv[h] += ds * t
    return {"context": ctx, "P": P, "dQp": dQ, "dKp": dK, "dV": dV, "dv": dv}
