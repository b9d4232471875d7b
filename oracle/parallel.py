"""Run the float64 oracle over the batch on several host cores.

TEST INFRASTRUCTURE.  Every output except dv is independent per sample, so the
batch is cut into contiguous shards, one worker process per shard, each calling
attn_ref unchanged; dv shards are added in shard order.
"""
from __future__ import annotations

import os
from concurrent.futures import ProcessPoolExecutor

import numpy as np

from . import attn_ref


def usable_cores() -> int:
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        return os.cpu_count() or 1


def _shard(args):
    Qp, Kp, V, v, key_len, dC = args
    return attn_ref.forward_backward(Qp, Kp, V, v, key_len, dC)


def forward_backward(Qp, Kp, V, v, key_len, dContext, workers: int | None = None):
    """Same result as attn_ref.forward_backward, batch sharded over `workers`
    processes (default: all usable cores, at most one sample per worker)."""
    B = Qp.shape[0]
    n = max(1, min(workers or usable_cores(), B))
    if n == 1:
        return attn_ref.forward_backward(Qp, Kp, V, v, key_len, dContext)
    cuts = np.linspace(0, B, n + 1).astype(int)
    jobs = [(Qp[a:b], Kp[a:b], V[a:b], v, key_len[a:b], dContext[a:b])
            for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
    with ProcessPoolExecutor(max_workers=len(jobs)) as ex:
        parts = list(ex.map(_shard, jobs))
    out = {k: np.concatenate([p[k] for p in parts], axis=0)
           for k in ("context", "P", "dQp", "dKp", "dV")}
    dv = np.zeros_like(parts[0]["dv"])
    for p in parts:
        dv += p["dv"]
    out["dv"] = dv
    return out
