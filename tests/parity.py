"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np

from oracle import attn_ref, parallel

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max-abs error relative to the largest reference entry, per tensor
KEYS = ("context", "P", "dQp", "dKp", "dV", "dv")


def oracle_outputs(inputs, workers=None):
    args = (inputs["Qp"], inputs["Kp"], inputs["V"], inputs["v"], inputs["key_len"], inputs["dContext"])
    if workers == 1:
        return attn_ref.forward_backward(*args)
    return parallel.forward_backward(*args, workers=workers)


def rel_err(got, ref):
    """max |got - ref| / max(max |ref|, 1e-30)"""
    return float(np.abs(got.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def elementwise_err(got, ref):
    """max_k |got_k - ref_k| / (|ref_k| + 1e-3 max|ref|): information beside the per-tensor figure; it weighs
    errors at small entries more."""
    ref = np.asarray(ref, dtype=np.float64)
    scale = 1e-3 * max(np.abs(ref).max(), 1e-30)
    return float((np.abs(got.astype(np.float64) - ref) / (np.abs(ref) + scale)).max())


def assert_parity(got, ref, inputs, in_dtype, what=""):
    tol = TOL[in_dtype]
    Tk = inputs["Kp"].shape[1]
    report = {}
    for k in KEYS:
        assert got[k].shape == ref[k].shape, (what, k)
        assert np.isfinite(got[k]).all(), f"{what} {k}: non-finite values (unwritten output?)"
        report[k] = rel_err(got[k], ref[k])
    print(f"{what}: max-abs error / max|ref| per tensor:", {k: f"{e:.2e}" for k, e in report.items()},
          "| element-wise variant (information):", {k: f"{elementwise_err(got[k], ref[k]):.2e}" for k in KEYS},
          flush=True)
    bad = {k: e for k, e in report.items() if not e <= tol}
    assert not bad, f"{what}: over tolerance {tol}: {bad} (all: {report})"
    # masked keys: exact zeros, bit for bit
    for b, L in enumerate(np.clip(inputs["key_len"], 0, Tk)):
        assert not got["P"][b, :, L:].any(), (what, "P", b)
        assert not got["dKp"][b, L:].any(), (what, "dKp", b)
        assert not got["dV"][b, L:].any(), (what, "dV", b)
        if L == 0:
            assert not got["context"][b].any() and not got["dQp"][b].any(), (what, "empty sample", b)
    return report
