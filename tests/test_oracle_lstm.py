"""Pins of the LSTM-cell oracle (CPU only)."""
import math

import numpy as np
import pytest

from oracle import lstm_ref as lr


def _inputs(B, H, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    return (scale * rng.standard_normal((B, 4 * H)), scale * rng.standard_normal((B, 4 * H)),
            rng.standard_normal((B, H)), rng.standard_normal((B, H)), rng.standard_normal((B, H)))


def test_forward_against_a_per_element_loop():
    """Slicing order and the cell equations, written out with math.exp / math.tanh only."""
    B, H = 3, 5
    Gx, Gh, c_prev, _, _ = _inputs(B, H, 0)
    h, c, a = lr.forward(Gx, Gh, c_prev)
    sg = lambda x: 1.0 / (1.0 + math.exp(-x))
    for b in range(B):
        for k in range(H):
            ai, af = Gx[b, k] + Gh[b, k], Gx[b, H + k] + Gh[b, H + k]
            ag, ao = Gx[b, 2 * H + k] + Gh[b, 2 * H + k], Gx[b, 3 * H + k] + Gh[b, 3 * H + k]
            cc = sg(af) * c_prev[b, k] + sg(ai) * math.tanh(ag)
            assert abs(c[b, k] - cc) < 1e-15
            assert abs(h[b, k] - sg(ao) * math.tanh(cc)) < 1e-15
            assert a[b, 2 * H + k] == ag


def test_backward_against_finite_differences():
    """L = sum(dh * h) + sum(dc * c); central differences on every element of a and c_prev."""
    B, H = 2, 4
    Gx, Gh, c_prev, dh, dc = _inputs(B, H, 1)
    _, _, a = lr.forward(Gx, Gh, c_prev)
    da, dcp = lr.backward(dh, dc, a, c_prev)

    def loss(a_, cp_):
        i, f, g, o, c, tc = lr.activations(a_, cp_)
        return float((dh * o * tc).sum() + (dc * c).sum())

    eps = 1e-6
    for idx in np.ndindex(a.shape):
        ap, am = a.copy(), a.copy()
        ap[idx] += eps
        am[idx] -= eps
        fd = (loss(ap, c_prev) - loss(am, c_prev)) / (2 * eps)
        assert abs(fd - da[idx]) <= 1e-8 * max(1.0, abs(fd)), (idx, fd, da[idx])
    for idx in np.ndindex(c_prev.shape):
        cp, cm = c_prev.copy(), c_prev.copy()
        cp[idx] += eps
        cm[idx] -= eps
        fd = (loss(a, cp) - loss(a, cm)) / (2 * eps)
        assert abs(fd - dcp[idx]) <= 1e-8 * max(1.0, abs(fd)), (idx, fd, dcp[idx])


def test_against_the_library_cell():
    """With identity weights PyTorch's LSTM cell is this block: same gate order, and its autograd gives a
    third, independent gradient; the gradients of Gx and Gh are both da."""
    torch = pytest.importorskip("torch")
    B, H = 4, 6
    Gx, Gh, c_prev, dh, dc = _inputs(B, H, 2)
    x = torch.tensor(np.concatenate([Gx, Gh], axis=1), dtype=torch.float64, requires_grad=True)
    cx = torch.tensor(c_prev, dtype=torch.float64, requires_grad=True)
    eye = torch.eye(4 * H, dtype=torch.float64)
    w_ih = torch.cat([eye, eye], dim=1)
    w_hh = torch.zeros(4 * H, H, dtype=torch.float64)
    hx = torch.zeros(B, H, dtype=torch.float64)
    h_t, c_t = torch._VF.lstm_cell(x, (hx, cx), w_ih, w_hh, None, None)
    (h_t * torch.tensor(dh) + c_t * torch.tensor(dc)).sum().backward()
    h, c, a = lr.forward(Gx, Gh, c_prev)
    da, dcp = lr.backward(dh, dc, a, c_prev)
    np.testing.assert_allclose(h, h_t.detach().numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(c, c_t.detach().numpy(), rtol=0, atol=1e-14)
    gx = x.grad.numpy()
    np.testing.assert_allclose(gx[:, :4 * H], da, rtol=0, atol=1e-14)
    np.testing.assert_allclose(gx[:, 4 * H:], da, rtol=0, atol=1e-14)
    np.testing.assert_allclose(cx.grad.numpy(), dcp, rtol=0, atol=1e-14)


def test_closed_forms():
    B, H = 2, 3
    rng = np.random.default_rng(3)
    c_prev, dh, dc = rng.standard_normal((B, H)), rng.standard_normal((B, H)), rng.standard_normal((B, H))
    z = np.zeros((B, 4 * H))
    # a = 0: every sigmoid is 1/2 and the candidate is 0
    h, c, a = lr.forward(z, z, c_prev)
    np.testing.assert_allclose(c, 0.5 * c_prev, rtol=0, atol=1e-16)
    np.testing.assert_allclose(h, 0.5 * np.tanh(0.5 * c_prev), rtol=0, atol=1e-16)
    da, dcp = lr.backward(dh, dc, a, c_prev)
    dct = dc + 0.5 * dh * (1 - np.tanh(0.5 * c_prev) ** 2)
    np.testing.assert_allclose(dcp, 0.5 * dct, rtol=0, atol=1e-15)
    np.testing.assert_allclose(da[:, 0:H], 0, atol=0)                              # di = dct * g = 0
    np.testing.assert_allclose(da[:, H:2 * H], 0.25 * dct * c_prev, rtol=0, atol=1e-15)
    np.testing.assert_allclose(da[:, 2 * H:3 * H], 0.5 * dct, rtol=0, atol=1e-15)
    np.testing.assert_allclose(da[:, 3 * H:], 0.25 * dh * np.tanh(0.5 * c_prev), rtol=0, atol=1e-15)
    # forget gate open, input gate shut, output gate open: the cell copies its state
    big = np.zeros((B, 4 * H))
    big[:, 0:H], big[:, H:2 * H], big[:, 3 * H:] = -50, 50, 50
    h, c, a = lr.forward(big, z, c_prev)
    np.testing.assert_allclose(c, c_prev, rtol=1e-15)
    np.testing.assert_allclose(h, np.tanh(c_prev), rtol=1e-15)
    da, dcp = lr.backward(dh, dc, a, c_prev)
    np.testing.assert_allclose(dcp, dc + dh * (1 - np.tanh(c_prev) ** 2), rtol=1e-14)
    assert np.abs(da).max() < 1e-20                                                # saturated gates pass nothing
    # input gate open, forget gate shut: the state is the candidate
    big = np.zeros((B, 4 * H))
    big[:, 0:H], big[:, H:2 * H] = 50, -50
    g_pre = rng.standard_normal((B, H))
    big[:, 2 * H:3 * H] = g_pre
    _, c, _ = lr.forward(z, big, c_prev)
    np.testing.assert_allclose(c, np.tanh(g_pre), rtol=1e-14)


def test_saturation_is_finite():
    B, H = 2, 4
    rng = np.random.default_rng(4)
    Gx = 1000.0 * np.sign(rng.standard_normal((B, 4 * H)))
    c_prev, dh, dc = 100 * rng.standard_normal((B, H)), rng.standard_normal((B, H)), rng.standard_normal((B, H))
    with np.errstate(over="raise", invalid="raise", divide="raise"):
        h, c, a = lr.forward(Gx, np.zeros_like(Gx), c_prev)
        da, dcp = lr.backward(dh, dc, a, c_prev)
    for t in (h, c, da, dcp):
        assert np.isfinite(t).all()
    assert np.abs(h).max() <= 1.0


def test_sigmoid_symmetry_and_range():
    x = np.linspace(-800, 800, 3201)
    s = lr.sigmoid(x)
    np.testing.assert_allclose(s + lr.sigmoid(-x), 1.0, rtol=0, atol=2.3e-16)     # one rounding of 1 - s
    assert (np.diff(s) >= 0).all() and s[0] == 0.0 and s[-1] == 1.0 and lr.sigmoid(0.0) == 0.5


def test_kept_elements():
    """Recomputing keeps the summed pre-activations and the previous state: one [B, H] tensor fewer than the
    four activations, tanh(c) and the previous state (and half of what keeping both addends would take,
    Section 4.1)."""
    B, H = 128, 512
    assert lr.kept_elements(B, H, False) - lr.kept_elements(B, H, True) == B * H
    assert lr.kept_elements(B, H, True) == 5 * B * H < 9 * B * H
