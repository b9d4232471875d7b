"""Input generator: shapes, distributions, determinism, bf16 rounding (no GPU)."""
import numpy as np

from paper_1805_08899_amd.workloads import (WORKLOADS, bf16_bits_to_f32, make_inputs, round_to_bf16)


def test_shapes_and_ranges_cfg1():
    wl = WORKLOADS[1]
    d = make_inputs(wl)
    assert d["Qp"].shape == (64, 50, 512) and d["Kp"].shape == (64, 50, 512)
    assert d["V"].shape == (64, 50, 512) and d["v"].shape == (512,)
    assert d["dContext"].shape == (64, 50, 512) and d["key_len"].dtype == np.int32
    assert d["key_len"].min() >= 10 and d["key_len"].max() <= 50
    assert abs(d["Qp"].std() - 0.5) < 0.01 and abs(d["dContext"].std() - 1.0) < 0.01
    assert np.abs(d["v"]).max() <= 1 / np.sqrt(512)


def test_deterministic():
    a, b = make_inputs(WORKLOADS[0]), make_inputs(WORKLOADS[0])
    for k in a:
        assert np.array_equal(a[k], b[k])
    c = make_inputs(WORKLOADS[0], seed=1)
    assert not np.array_equal(a["Qp"], c["Qp"])


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -0.3, 3.14159], dtype=np.float32)
    bits = round_to_bf16(x)
    back = bf16_bits_to_f32(bits)
    # 1+2^-8 is a tie between 1 and 1+2^-7: even mantissa wins -> 1.0
    assert back[0] == 1.0 and back[1] == 1.0
    # 1+3*2^-8 is a tie between 1+2^-7 and 1+2^-6: even wins -> 1+2^-6
    assert back[2] == np.float32(1.0 + 2 ** -6) and back[3] == np.float32(1.0 + 2 ** -7)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2 ** -8)
    import torch
    t = torch.tensor(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(t, back)


def test_bf16_workload_values_are_representable():
    wl = WORKLOADS[4]
    # the full batch is 26 MB per tensor; a small workload of the same kind is enough here
    small = type(wl)("t", 2, 3, 4, 8, 8, "bf16", 0.5, 1, 4, True)
    d = make_inputs(small, seed=3)
    for k in ("Qp", "Kp", "V", "v"):
        assert d[k + "_bits"].dtype == np.uint16
        assert np.array_equal(bf16_bits_to_f32(d[k + "_bits"]), d[k])
