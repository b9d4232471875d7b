"""Device-memory accounting for one forward+backward of the attention layer.

The paper's vocabulary (Section 3.2): *feature maps* are what the forward pass
leaves behind for the backward pass, *workspace* is scratch that lives only
inside one pass.  With the broadcast add + tanh recomputed in the backward
pass the only feature map of the layer is P (plus the layer inputs Qp and Kp,
which the caller holds anyway); the baseline also keeps the B x Tq x Tk x H
tanh map (Section 4.1 and Section 5.1: T^2 x N against T x 2N per sample).

Pure host arithmetic; no device code is involved.
"""
from __future__ import annotations

from dataclasses import dataclass


def _sz(in_dtype: str) -> int:
    if in_dtype == "f32":
        return 4
    if in_dtype == "bf16":
        return 2
    raise ValueError(f"unknown input dtype {in_dtype!r}")


def scoring_feature_map_elems(T: int, N: int, recompute: bool) -> int:
    """Per-sample feature-map elements of the scoring function when T queries
    of width N meet T keys of width N (Section 4.1 / 5.1 closed form)."""
    return T * 2 * N if recompute else T * T * N


@dataclass(frozen=True)
class Footprint:
    inputs: int          # Qp, Kp, V, v, key_len, dContext (caller-held)
    outputs: int         # context, dQp, dKp, dV, dv
    feature_maps: int    # persists from forward to backward
    workspace: int       # max over the two passes
    @property
    def total(self) -> int:
        return self.inputs + self.outputs + self.feature_maps + self.workspace


def tanh_map_bytes(B, Tq, Tk, H, elem_bytes: int = 4) -> int:
    return B * Tq * Tk * H * elem_bytes


def footprint(B, Tq, Tk, H, Dv, in_dtype="f32", *, stash: bool, fwd_ws: int = 0, bwd_ws: int = 0) -> Footprint:
    """Analytic bytes for one call pair.  `fwd_ws`/`bwd_ws` are the library's
    workspace sizes for this shape (pass the values the library reports)."""
    s = _sz(in_dtype)
    inputs = (B * Tq * H + B * Tk * H + B * Tk * Dv + H) * s + 4 * B + 4 * B * Tq * Dv
    outputs = 4 * (B * Tq * Dv + B * Tq * H + B * Tk * H + B * Tk * Dv + H)
    fmap = 4 * B * Tq * Tk + (tanh_map_bytes(B, Tq, Tk, H, 4) if stash else 0)
    return Footprint(inputs, outputs, fmap, max(fwd_ws, bwd_ws))
