"""The oracle still produces the stored workload-0 values (no GPU)."""
import os

import numpy as np

from oracle import attn_ref
from paper_1805_08899_amd.workloads import WORKLOADS, make_inputs

PATH = os.path.join(os.path.dirname(__file__), "golden", "cfg0_expected.txt")


def load_expected():
    out, lines = {}, [l for l in open(PATH) if not l.startswith("#")]
    out["key_len"] = np.array(lines[0].split()[1:], dtype=np.int32)
    for head, vals in zip(lines[1::2], lines[2::2]):
        name, *shape = head.split()
        out[name] = np.array(vals.split(), dtype=np.float64).reshape([int(s) for s in shape])
    return out


def test_oracle_matches_stored_values():
    exp = load_expected()
    d = make_inputs(WORKLOADS[0])
    assert np.array_equal(exp["key_len"], d["key_len"])
    got = attn_ref.forward_backward(d["Qp"], d["Kp"], d["V"], d["v"], d["key_len"], d["dContext"])
    for k, a in got.items():
        assert np.abs(a - exp[k]).max() <= 1e-14 * max(1.0, np.abs(exp[k]).max()), k
