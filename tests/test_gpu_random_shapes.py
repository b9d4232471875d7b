"""Seeded sweep of small random shapes through the C ABI against the float64 oracle: every dimension, the storage
type and the key counts are drawn, so tile edges that no hand-written case names still get exercised (ragged
rows and keys, H below and above one slice, Dv not a multiple of 16, batches that do not fill the eight-way
placement).  Same bar as the other parity tests."""
import numpy as np
import pytest

from paper_1805_08899_amd.workloads import Workload, make_inputs
from parity import assert_parity, oracle_outputs

pytestmark = pytest.mark.gpu

N_CASES = 24


def _draw(case):
    rng = np.random.default_rng(90210 + case)
    B = int(rng.integers(1, 20))
    Tq = int(rng.integers(1, 70))
    Tk = int(rng.integers(1, 150))
    H = int(rng.choice([1, 2, 3, 8, 20, 64, 65, 100, 256, 260, 300, 512, 516]))
    Dv = 4 * int(rng.integers(1, 70))
    dt = "bf16" if case % 3 == 2 else "f32"
    kl = rng.integers(0 if case % 4 == 0 else 1, Tk + 1, B).astype(np.int32)
    return B, Tq, Tk, H, Dv, dt, kl


@pytest.mark.parametrize("case", range(N_CASES))
def test_random_shape(case):
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from paper_1805_08899_amd import harness
    B, Tq, Tk, H, Dv, dt, kl = _draw(case)
    print("random shape", case, (B, Tq, Tk, H, Dv, dt), kl.tolist(), flush=True)
    wl = Workload(f"random{case}", B, Tq, Tk, H, Dv, dt, 0.5, 1, Tk, dt == "bf16")
    inputs = make_inputs(wl, seed=555 + case)
    inputs["key_len"] = kl
    db = harness.DeviceBatch(wl, inputs)
    db.poison_outputs()
    db.fwd()
    db.bwd()
    got = db.results()
    ref = oracle_outputs(inputs, workers=1)
    assert_parity(got, ref, inputs, dt, wl.name)
