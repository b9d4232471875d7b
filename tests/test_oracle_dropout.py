"""Pins of the one-bit dropout oracle (CPU only)."""
import os

import numpy as np
import pytest

from oracle import dropout_ref as dr

HERE = os.path.dirname(os.path.abspath(__file__))


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")) if l[0] not in "#\n"]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = dr.philox4x32_10(np.array([v[0:4]], dtype=np.uint32), np.array([v[4:6]], dtype=np.uint32))[0]
        assert [int(x) for x in out] == v[6:10]


def test_uniforms_layout_and_range():
    """Element i is word i mod 4 of block i div 4; the offset and the seed select other streams."""
    u = dr.uniforms(11, seed=7, offset=3)
    assert u.dtype == np.float32 and u.shape == (11,) and (u >= 0).all() and (u < 1).all()
    blk = dr.philox4x32_10(np.array([[2, 0, 3, 0]], dtype=np.uint32), np.array([[7, 0]], dtype=np.uint32))[0]
    assert u[9] == np.float32(int(blk[1]) >> 8) * np.float32(2.0 ** -24)
    assert not np.array_equal(u, dr.uniforms(11, seed=8, offset=3))
    assert not np.array_equal(u, dr.uniforms(11, seed=7, offset=4))
    assert np.array_equal(u[:8], dr.uniforms(8, seed=7, offset=3))
    big = dr.uniforms(1 << 16, seed=1, offset=0)
    assert abs(float(big.mean()) - 0.5) < 5e-3 and abs(float(big.var()) - 1 / 12) < 2e-3


def test_bit_order_against_a_loop():
    rng = np.random.default_rng(0)
    keep = rng.random(77) < 0.6
    bits = dr.pack_bits(keep)
    assert bits.shape == (3,) and bits.dtype == np.uint32
    for i, k in enumerate(keep):
        assert ((int(bits[i // 32]) >> (i % 32)) & 1) == int(k)
    assert int(bits[2]) >> (77 - 64) == 0                      # padding bits are zero
    assert np.array_equal(dr.unpack_bits(bits, 77), keep)


@pytest.mark.parametrize("p", [0.1, 0.3, 0.5])
def test_kept_fraction_and_scaling(p):
    n = 200_000
    x = np.random.default_rng(1).standard_normal(n)
    y, bits = dr.forward(x, p, seed=11, offset=0)
    keep = dr.unpack_bits(bits, n)
    assert abs(keep.mean() - (1 - p)) < 4 * np.sqrt(p * (1 - p) / n)
    assert np.array_equal(y == 0, ~keep | (x == 0))
    np.testing.assert_allclose(y[keep], x[keep] / (1 - float(np.float32(p))), rtol=1e-15)
    # expectation is preserved: the classic property of inverted dropout
    assert abs(np.ones(n)[keep].sum() / (1 - p) / n - 1) < 0.01


def test_p_zero_is_the_identity_and_backward_is_the_adjoint():
    rng = np.random.default_rng(2)
    x, dy = rng.standard_normal(1000), rng.standard_normal(1000)
    y, bits = dr.forward(x, 0.0, seed=5, offset=9)
    assert np.array_equal(y, x) and (dr.unpack_bits(bits, 1000)).all()
    y, bits = dr.forward(x, 0.25, seed=5, offset=9)
    dx = dr.backward(dy, bits, 0.25)
    # <dy, fwd(x)> == <bwd(dy), x>: the backward pass is the transpose of the (linear, diagonal) forward map
    assert abs(np.dot(dy, y) - np.dot(dx, x)) < 1e-9
    assert np.array_equal(dx == 0, y == 0)
