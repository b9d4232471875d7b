"""One-bit dropout: HIP path against the oracle.  The keep decisions and the packed bits must be bit-exact (the
random numbers and the comparison are the same on both sides); y and dx are one fp32 multiplication each and
are held to 1e-6 relative (the oracle divides in float64)."""
import numpy as np
import pytest

from oracle import dropout_ref as dr

pytestmark = pytest.mark.gpu

CASES = [
    # n, p, seed, offset
    (1, 0.5, 1, 0),
    (31, 0.3, 2, 5),
    (32, 0.3, 2, 5),
    (33, 0.1, 3, 1 << 40),
    (4 * 256 * 7 + 3, 0.5, (1 << 63) + 12345, 7),          # several blocks and a ragged tail
    (1 << 20, 0.2, 42, 0),
    (50 * 128 * 1024 + 17, 0.1, 7, 99),                      # 6400 blocks of 256 quads and a ragged tail
    ((1 << 24) + 4 * 256 * 3 + 2, 0.25, 11, 1 << 33),        # more than 65535 blocks, ragged
    (1000, 0.0, 9, 9),                                       # keep everything
]


@pytest.mark.parametrize("case", CASES, ids=[f"n{c[0]}_p{c[1]}" for c in CASES])
def test_dropout_parity(case):
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from paper_1805_08899_amd import binding as eb
    n, p, seed, offset = case
    print("dropout case", case, flush=True)
    rng = np.random.default_rng(n % 1000)
    x = rng.standard_normal(n).astype(np.float32)
    dy = rng.standard_normal(n).astype(np.float32)
    dev = torch.device("cuda:0")
    xd, dyd = torch.from_numpy(x).to(dev), torch.from_numpy(dy).to(dev)
    y = torch.full((n,), float("nan"), device=dev)
    dx = torch.full((n,), float("nan"), device=dev)
    words = eb.echo_dropout_mask_words(n)
    bits = torch.full((words,), -1, dtype=torch.int32, device=dev)
    st = torch.cuda.current_stream(dev)
    eb.check(eb.echo_dropout_fwd(xd, n, p, seed, offset, y, bits, stream=st), "echo_dropout_fwd")
    eb.check(eb.echo_dropout_bwd(dyd, bits, n, p, dx, stream=st), "echo_dropout_bwd")
    torch.cuda.synchronize(dev)
    y_ref, bits_ref = dr.forward(x, p, seed, offset)
    got_bits = bits.cpu().numpy().view(np.uint32)
    assert np.array_equal(got_bits, bits_ref), "one-bit feature map differs"
    dx_ref = dr.backward(dy, bits_ref, p)
    for name, got, ref in (("y", y.cpu().numpy(), y_ref), ("dx", dx.cpu().numpy(), dx_ref)):
        assert np.isfinite(got).all(), name
        assert np.array_equal(got == 0, ref == 0), name           # the same elements are dropped
        np.testing.assert_allclose(got, ref, rtol=1e-6, atol=0, err_msg=name)
