"""Host-side memory accounting against the paper's closed form (no GPU)."""
import os

import pytest

from paper_1805_08899_amd import footprint as fp
from paper_1805_08899_amd.workloads import WORKLOADS

GOLD = os.path.join(os.path.dirname(__file__), "golden", "footprint_closed_form.txt")


def _rows():
    for line in open(GOLD):
        if line.strip() and not line.startswith("#"):
            yield tuple(int(x) for x in line.split())


def test_closed_form_from_paper():
    rows = list(_rows())
    assert rows
    for T, N, stash, rec in rows:
        assert fp.scoring_feature_map_elems(T, N, recompute=False) == stash
        assert fp.scoring_feature_map_elems(T, N, recompute=True) == rec
        if 50 <= T <= 100:                     # "an order of magnitude smaller"
            assert stash / rec >= 10


@pytest.mark.parametrize("wl", WORKLOADS, ids=lambda w: w.name)
def test_stash_minus_recompute_is_the_4d_map(wl):
    a = fp.footprint(wl.B, wl.Tq, wl.Tk, wl.H, wl.Dv, wl.in_dtype, stash=True)
    b = fp.footprint(wl.B, wl.Tq, wl.Tk, wl.H, wl.Dv, wl.in_dtype, stash=False)
    assert a.total - b.total == wl.n4 * 4
    assert b.feature_maps == 4 * wl.B * wl.Tq * wl.Tk


def test_documented_map_sizes():
    mb = [fp.tanh_map_bytes(w.B, w.Tq, w.Tk, w.H) for w in WORKLOADS]
    assert mb[1] == 327_680_000 and mb[2] == 2_621_440_000
    assert mb[3] == 11_796_480_000 and mb[4] == 1_310_720_000
