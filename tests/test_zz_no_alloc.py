"""echo_attn_bwd_static, the backward entry point that takes its workspace from a buffer inside the library's
device image, against echo_attn_bwd on the same inputs: same kernels, so every output must agree bit for bit
(and therefore within the parity tolerance).  Two calls in a row, the second on a smaller batch, so that what
the first call left in the shared buffer must not matter."""
import numpy as np
import pytest

from paper_1805_08899_amd.workloads import WORKLOADS, Workload, make_inputs
from parity import TOL, rel_err

GRADS = (("dQp", "dQp"), ("dKp", "dKp"), ("dV", "dV"), ("dv", "dv"))


def _both(harness, eb, torch, wl, seed):
    inputs = make_inputs(wl, seed=seed)
    db = harness.DeviceBatch(wl, inputs)
    db.poison_outputs()
    db.fwd()
    db.bwd()
    want = db.results()
    for _, a in GRADS:
        getattr(db, a).fill_(float("nan"))
    eb.check(eb.echo_attn_bwd_static(db.desc, db.dC, db.P, db.Qp, db.Kp, db.V, db.v, db.key_len, db.dQp, db.dKp,
                                     db.dV, db.dv, stream=torch.cuda.current_stream(db.device)),
             "echo_attn_bwd_static")
    got = db.results()
    for k, _ in GRADS:
        assert np.isfinite(got[k]).all(), (wl.name, k)
        assert rel_err(got[k], want[k].astype(np.float64)) <= TOL[wl.in_dtype], (wl.name, k)
        assert np.array_equal(got[k], want[k]), (wl.name, k, "not bit-identical to echo_attn_bwd")


@pytest.mark.gpu
def test_static_workspace_backward_matches_the_caller_workspace_backward():
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from paper_1805_08899_amd import binding as eb, harness
    print("no-alloc backward: workload 1, then a smaller ragged batch", flush=True)
    _both(harness, eb, torch, WORKLOADS[1], seed=None)
    small = Workload("static_small", 5, 13, 27, 192, 36, "f32", 0.5, 1, 27)
    _both(harness, eb, torch, small, seed=11)
    bf = Workload("static_bf16", 3, 9, 14, 128, 16, "bf16", 0.5, 1, 14, True)
    _both(harness, eb, torch, bf, seed=12)


def test_static_workspace_rejects_shapes_beyond_its_buffer():
    """Host-side check only: nothing is launched."""
    from paper_1805_08899_amd import binding as eb
    A = 0x10000
    big = eb.make_desc(512, 300, 300, 64, 64)
    assert eb.echo_attn_bwd_workspace_bytes(big) > eb.ECHO_ATTN_STATIC_SCRATCH_BYTES
    assert eb.echo_attn_bwd_static(big, A, A, A, A, A, A, A, A, A, A, A) == eb.ECHO_ERR_WORKSPACE
    assert "bytes" in eb.echo_last_error_detail()
