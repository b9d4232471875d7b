"""LSTM-cell non-linear block: HIP path against the float64 oracle.

Tolerance: each output is a product of at most six fp32 factors, each factor a sigmoid or tanh built from the
hardware exp2 and reciprocal (about one ulp each) with one or two roundings on top, so errors stay within a few
1e-7 of the tensor's scale; the bar is 1e-5 of the largest reference magnitude per tensor, and 2e-6 of it per
element on top of 1e-5 relative.  The kept sum a = Gx + Gh is one fp32 addition and must be bit-exact."""
import numpy as np
import pytest

from oracle import lstm_ref as lr
from paper_1805_08899_amd.workloads import make_lstm_inputs

pytestmark = pytest.mark.gpu

TOL = 1e-5

CASES = [
    # B, H, scale
    (1, 1, 1.0),
    (3, 5, 1.0),                 # H not a multiple of four: one element per lane
    (4, 16, 1.0),
    (128, 512, 1.0),             # the translation model's cell
    (128, 1024, 1.5),
    (7, 4 * 67, 3.0),            # ragged block tail, many saturated gates
    (4100, 1024, 1.0),           # 4100 blocks of 256 items
    (33, 1023, 1.0),             # long odd rows
]


def _close(name, got, ref):
    assert np.isfinite(got).all(), name
    scale = max(float(np.abs(ref).max()), 1e-30)
    err = float(np.abs(got.astype(np.float64) - ref).max()) / scale
    assert err <= TOL, f"{name}: max-abs-rel {err:.3e}"
    np.testing.assert_allclose(got, ref, rtol=1e-5, atol=2e-6 * scale, err_msg=name)


def _run(B, H, inp, *, with_dc=True, in_place=None, stash=False):
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from paper_1805_08899_amd import binding as eb
    dev = torch.device("cuda:0")
    d = {k: torch.from_numpy(v).to(dev) for k, v in inp.items()}
    nan = lambda *s: torch.full(s, float("nan"), device=dev)
    h, c, dcp, da = nan(B, H), nan(B, H), nan(B, H), nan(B, 4 * H)
    st = torch.cuda.current_stream(dev)
    dc = d["dc"] if with_dc else None
    if stash:
        acts, tc = nan(B, 4 * H), nan(B, H)
        eb.check(eb.echo_lstm_cell_fwd_stash(B, H, d["Gx"], d["Gh"], d["c_prev"], h, c, acts, tc, stream=st), "fwd_stash")
        eb.check(eb.echo_lstm_cell_bwd_stash(B, H, d["dh"], dc, acts, tc, d["c_prev"], da, dcp, stream=st), "bwd_stash")
        kept = acts
    else:
        a = {"Gx": d["Gx"], "Gh": d["Gh"], None: nan(B, 4 * H)}[in_place]
        eb.check(eb.echo_lstm_cell_fwd(B, H, d["Gx"], d["Gh"], d["c_prev"], h, c, a, stream=st), "fwd")
        eb.check(eb.echo_lstm_cell_bwd(B, H, d["dh"], dc, a, d["c_prev"], da, dcp, stream=st), "bwd")
        kept = a
    torch.cuda.synchronize(dev)
    return {k: v.cpu().numpy() for k, v in dict(h=h, c=c, kept=kept, da=da, dc_prev=dcp).items()}


def _reference(inp, with_dc=True):
    h, c, a = lr.forward(inp["Gx"], inp["Gh"], inp["c_prev"])
    a32 = inp["Gx"] + inp["Gh"]                                  # the kept sum as fp32 rounds it
    dc = inp["dc"] if with_dc else np.zeros_like(inp["dh"])
    da, dcp = lr.backward(inp["dh"], dc, a32, inp["c_prev"])
    return dict(h=h, c=c, a32=a32, da=da, dc_prev=dcp)


@pytest.mark.parametrize("case", CASES, ids=[f"B{c[0]}_H{c[1]}" for c in CASES])
def test_lstm_cell_parity(case):
    B, H, scale = case
    print("lstm case", case, flush=True)
    inp = make_lstm_inputs(B, H, seed=B + H, scale=scale)
    got = _run(B, H, inp)
    ref = _reference(inp)
    assert np.array_equal(got["kept"], ref["a32"]), "kept sum is one fp32 addition"
    for k in ("h", "c", "da", "dc_prev"):
        _close(k, got[k], ref[k])


def test_stash_path_matches_the_oracle_and_the_recompute_path():
    B, H = 64, 256
    inp = make_lstm_inputs(B, H, seed=5)
    print("lstm stash", B, H, flush=True)
    got_s, got_r, ref = _run(B, H, inp, stash=True), _run(B, H, inp), _reference(inp)
    i, f, g, o, _, _ = lr.activations(ref["a32"], inp["c_prev"])
    _close("acts", got_s["kept"], np.concatenate([i, f, g, o], axis=1))
    for k in ("h", "c", "da", "dc_prev"):
        _close(k + " (stash)", got_s[k], ref[k])
    # the two paths evaluate the same expressions in the same order
    for k in ("h", "c", "da", "dc_prev"):
        assert np.array_equal(got_s[k], got_r[k]), k


@pytest.mark.parametrize("where", ["Gx", "Gh"])
def test_kept_sum_may_replace_an_addend_in_place(where):
    B, H = 16, 128
    inp = make_lstm_inputs(B, H, seed=6)
    print("lstm in place", where, flush=True)
    got, ref = _run(B, H, inp, in_place=where), _reference(inp)
    assert np.array_equal(got["kept"], ref["a32"])
    for k in ("h", "c", "da", "dc_prev"):
        _close(k, got[k], ref[k])


def test_no_gradient_into_the_cell_state():
    B, H = 8, 64
    inp = make_lstm_inputs(B, H, seed=7)
    got, ref = _run(B, H, inp, with_dc=False), _reference(inp, with_dc=False)
    for k in ("da", "dc_prev"):
        _close(k, got[k], ref[k])


def test_saturated_gates_stay_finite():
    B, H = 4, 32
    inp = make_lstm_inputs(B, H, seed=8)
    inp["Gx"] = (200.0 * np.sign(inp["Gx"])).astype(np.float32)   # |a| ~ 200: exp2 overflows, sigmoid is 0 or 1
    inp["c_prev"] = (30.0 * inp["c_prev"]).astype(np.float32)
    got, ref = _run(B, H, inp), _reference(inp)
    for k in ("h", "c", "da", "dc_prev"):
        _close(k, got[k], ref[k])
    assert np.abs(got["h"]).max() <= 1.0


def test_bit_reproducible():
    B, H = 32, 512
    inp = make_lstm_inputs(B, H, seed=9)
    r1, r2 = _run(B, H, inp), _run(B, H, inp)
    for k in r1:
        assert np.array_equal(r1[k], r2[k]), k
