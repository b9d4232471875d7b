"""HIP path against the float64 oracle, element by element, through the C ABI.

Tolerance (stated by the benchmark spec): per output tensor max|gpu - ref| / max|ref|
<= 1e-4 for fp32 inputs and <= 2e-2 for bf16-stored inputs; outputs at masked
keys must be exact zeros.
"""
import numpy as np
import pytest

from paper_1805_08899_amd.workloads import WORKLOADS, Workload, make_inputs
from parity import KEYS, assert_parity, oracle_outputs, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_1805_08899_amd import harness
    return harness


def run_gpu(H, wl, inputs, stash=False):
    db = H.DeviceBatch(wl, inputs, stash=stash)
    db.poison_outputs()
    if stash:
        db.fwd_stash(); db.bwd_stash()
    else:
        db.fwd(); db.bwd()
    return db, db.results()


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_workload_parity(H, idx):
    wl = WORKLOADS[idx]
    print(f"workload {wl.name}", flush=True)
    inputs = make_inputs(wl)
    db, got = run_gpu(H, wl, inputs)
    ref = oracle_outputs(inputs, workers=1 if idx == 0 else None)
    rep = assert_parity(got, ref, inputs, wl.in_dtype, wl.name)
    print(wl.name, {k: f"{e:.2e}" for k, e in rep.items()}, flush=True)
    # reproducible bit for bit
    db.poison_outputs(); db.fwd(); db.bwd()
    again = db.results()
    for k in KEYS:
        assert np.array_equal(got[k], again[k]), f"{k} differs between two runs"


EDGE = [
    # name, B, Tq, Tk, H, Dv, dtype, key_len (None = random 1..Tk)
    ("single_query", 3, 1, 9, 40, 8, "f32", None),
    ("single_key", 3, 5, 1, 33, 4, "f32", None),
    ("h_equals_1", 2, 4, 5, 1, 4, "f32", None),
    ("ragged_everything", 3, 37, 45, 200, 36, "f32", None),
    ("h_not_multiple_of_64", 2, 19, 23, 70, 12, "f32", None),
    ("empty_and_clamped_lengths", 5, 7, 12, 64, 16, "f32", [0, 12, 40, -3, 5]),
    ("rows_in_several_passes", 2, 150, 21, 64, 8, "f32", None),
    ("many_key_tiles", 1, 9, 1100, 64, 8, "f32", [1100]),
    ("bf16_ragged", 3, 21, 34, 130, 20, "bf16", None),
    ("bf16_empty_sample", 2, 6, 7, 16, 16, "bf16", [0, 7]),
    # placement paths: the forward kernel ranks samples only up to 128 per batch, the backward up to 1024
    ("batch_beyond_forward_ranking", 131, 5, 9, 32, 8, "f32", None),
    ("batch_beyond_backward_ranking", 1030, 3, 5, 16, 4, "f32", None),
    # short key axis with value width beyond one round of the dS kernel, and a key axis just past its limit
    ("wide_values_short_keys", 2, 20, 40, 64, 1040, "f32", None),
    ("keys_just_past_the_short_path", 2, 18, 129, 64, 24, "f32", None),
    ("fused_forward_h_not_multiple_of_256", 3, 11, 13, 300, 12, "f32", None),
    # fused forward with fewer keys than waves and every key valid: the waves without keys must stay inside Kp
    ("fused_forward_one_key", 3, 5, 1, 32, 4, "f32", [1, 1, 1]),
    ("fused_forward_two_keys", 2, 9, 2, 64, 8, "f32", [2, 2]),
    ("fused_forward_three_keys", 2, 9, 3, 260, 8, "f32", [3, 3]),
    # one-kernel forward whose row tile needs more LDS than the default limit (the limit is raised once per device)
    ("fused_forward_lds_beyond_default", 2, 9, 64, 2048, 64, "f32", None),
    # row tile beyond on-chip memory: the forward falls back to the score / softmax / context kernels
    ("forward_fallback_at_large_h", 2, 5, 9, 4864, 8, "f32", None),
    # placement by rank at batch sizes that do not fill the XCDs evenly
    ("ranked_placement_b47", 47, 9, 12, 64, 8, "f32", None),
    ("ranked_placement_b100", 100, 3, 20, 32, 4, "f32", None),
    ("ranked_placement_b127", 127, 2, 7, 16, 4, "f32", None),
    # row mode of the forward kernel at 2 and 4 slices of h, longest key shares, and streaming mode right past them
    ("row_mode_two_slices_eight_keys_per_wave", 2, 11, 64, 512, 16, "f32", [64, 37]),
    ("row_mode_four_slices", 2, 10, 32, 1024, 16, "f32", [32, 5]),
    ("row_mode_bf16_four_slices", 2, 9, 30, 900, 16, "bf16", None),
    ("streaming_mode_just_past_row_mode", 2, 11, 65, 512, 16, "f32", [65, 64]),
    # streaming mode runs blocks of four waves up to H = 512 and of eight beyond
    ("forward_four_wave_blocks", 3, 19, 100, 512, 64, "f32", [100, 61, 3]),
    ("forward_four_wave_blocks_ragged_h", 2, 9, 70, 300, 12, "f32", None),
    ("forward_eight_wave_streaming_past_512", 2, 9, 70, 516, 12, "f32", None),
    # context phase with two waves per group of 256 value columns, half of the keys each (eight waves at Dv = 1024,
    # four at Dv = 512): one to five keys (a second half with no keys), odd and even numbers of four-key chunks,
    # batches that end inside a chunk; and the forms next to it (value rows wider than the staged query rows, Dv = 768)
    ("context_key_halves_few_keys", 5, 9, 70, 1024, 1024, "f32", [1, 4, 5, 8, 70]),
    ("context_key_halves_odd_chunks", 3, 11, 76, 1024, 1024, "f32", [76, 41, 13]),
    ("context_key_halves_bf16", 2, 9, 50, 1024, 1024, "bf16", [50, 23]),
    ("context_key_halves_four_waves", 3, 13, 90, 512, 512, "f32", [90, 66, 3]),
    ("context_whole_keys_values_wider_than_h", 2, 9, 70, 768, 1024, "f32", [70, 9]),
    ("context_whole_keys_768_columns", 2, 9, 70, 1024, 768, "f32", [70, 9]),
    # dV: a block owns all keys up to four key tiles (Tk <= 64), one key tile beyond; value width not a multiple of 64
    ("dv_all_keys_form_four_tiles", 2, 21, 64, 64, 72, "f32", [64, 17]),
    ("dv_per_tile_form_just_past", 2, 21, 65, 64, 72, "f32", [65, 16]),
    # dS on long key axes: a wave's key tiles in groups of four (16 and 21 tiles) or five (19 tiles), tiles past a
    # sample's last one skipped
    ("ds_sixteen_key_tiles", 1, 17, 256, 64, 8, "f32", [250]),
    ("ds_groups_of_five_key_tiles", 3, 20, 300, 64, 24, "f32", [300, 260, 40]),
    ("ds_groups_of_four_past_twenty_tiles", 2, 10, 330, 64, 8, "f32", [330, 130]),
    # dS on short key axes: value rows of one round (up to 512 columns), two rounds (up to 1024, ragged) and more;
    # odd and even numbers of key tiles, a single key tile
    ("ds_short_keys_one_round_five_tiles", 2, 21, 80, 64, 512, "f32", [80, 33]),
    ("ds_short_keys_two_rounds_ragged", 3, 21, 40, 64, 600, "f32", [40, 7, 17]),
    ("ds_short_keys_two_rounds_eight_tiles", 2, 9, 128, 64, 1024, "f32", [128, 97]),
    ("ds_short_keys_three_rounds", 2, 9, 40, 64, 1100, "f32", [40, 16]),
    # dS on long key axes up to 384 keys: blocks of 32 query rows (ragged last block, fewer than 32 rows in all,
    # value width not a multiple of 16), 16 rows past 384 keys
    ("ds_32_row_blocks_ragged", 2, 45, 200, 64, 40, "f32", [200, 131]),
    ("ds_32_row_blocks_17_rows", 2, 17, 384, 64, 24, "f32", [384, 129]),
    ("ds_32_row_blocks_bf16", 2, 70, 300, 64, 72, "bf16", [300, 77]),
    ("ds_16_row_blocks_past_384_keys", 1, 40, 385, 64, 24, "f32", [385]),
    # dV on key axes past 128: panels of 64 keys x 256 columns when Tk is a multiple of four (ragged last panel,
    # value width not a multiple of 64, fewer rows than one batch, masked keys inside a panel), one key tile per
    # block otherwise and up to 128 keys
    ("dv_panels_of_64_keys", 2, 37, 164, 64, 264, "f32", [164, 35]),
    ("dv_panels_few_rows", 2, 3, 132, 64, 24, "f32", [132, 1]),
    ("dv_panels_bf16", 2, 21, 196, 64, 520, "bf16", [196, 64]),
    ("dv_key_tiles_when_tk_not_multiple_of_4", 2, 21, 165, 64, 264, "f32", [165, 35]),
    ("dv_key_tiles_up_to_128_keys", 2, 37, 100, 64, 264, "f32", [100, 35]),
]


@pytest.mark.parametrize("case", EDGE, ids=[c[0] for c in EDGE])
def test_edge_shapes(H, case):
    name, B, Tq, Tk, Hh, Dv, dt, kl = case
    print("edge case", case, flush=True)
    wl = Workload(name, B, Tq, Tk, Hh, Dv, dt, 0.5, 1, Tk, dt == "bf16")
    inputs = make_inputs(wl, seed=1234 + len(name))
    if kl is not None:
        inputs["key_len"] = np.asarray(kl, dtype=np.int32)
    _, got = run_gpu(H, wl, inputs)
    ref = oracle_outputs(inputs, workers=1)
    assert_parity(got, ref, inputs, dt, name)


GUARDED = [
    # name, B, Tq, Tk, H, Dv, dtype, stash
    ("guard_tiny", 4, 6, 7, 16, 16, "f32", False),
    ("guard_ragged", 3, 37, 45, 200, 36, "f32", False),
    ("guard_unfused_forward", 2, 19, 23, 70, 12, "f32", False),
    ("guard_bf16", 3, 21, 34, 130, 20, "bf16", False),
    ("guard_long_keys", 1, 9, 300, 64, 8, "f32", False),
    ("guard_dv_all_keys_form", 2, 21, 64, 64, 72, "f32", False),
    ("guard_four_wave_forward", 2, 9, 70, 300, 12, "f32", False),
    ("guard_stash", 4, 6, 7, 16, 16, "f32", True),
]


@pytest.mark.parametrize("case", GUARDED, ids=[c[0] for c in GUARDED])
def test_no_write_outside_the_buffers(H, case):
    """Every output and the workspace sit between 4 KB guard zones holding a pattern; after forward + backward
    (and the no-workspace backward) the zones must be untouched."""
    import torch
    from paper_1805_08899_amd import binding as eb
    name, B, Tq, Tk, Hh, Dv, dt, stash = case
    print("guarded case", case, flush=True)
    wl = Workload(name, B, Tq, Tk, Hh, Dv, dt, 0.5, 1, Tk, dt == "bf16")
    inputs = make_inputs(wl, seed=808 + len(name))
    db = H.DeviceBatch(wl, inputs, stash=stash, guard_bytes=4096)
    db.poison_outputs()
    if stash:
        db.fwd_stash(); db.bwd_stash()
    else:
        db.fwd(); db.bwd()
    assert db.check_guards() == []
    got = db.results()
    assert_parity(got, oracle_outputs(inputs, workers=1), inputs, dt, name)
    if not stash:
        eb.check(eb.echo_attn_bwd_static(db.desc, db.dC, db.P, db.Qp, db.Kp, db.V, db.v, db.key_len, db.dQp, db.dKp,
                                         db.dV, db.dv, stream=torch.cuda.current_stream(db.device)), "bwd_static")
        assert db.check_guards() == []


def test_guard_zones_notice_a_stray_write(H):
    """The checker itself: one byte written just past a buffer, or just before it, is reported."""
    import torch
    wl = Workload("guard_self_check", 2, 3, 5, 8, 4, "f32", 0.5, 1, 5)
    db = H.DeviceBatch(wl, make_inputs(wl, seed=1), guard_bytes=4096)
    assert db.check_guards() == []
    whole, nbytes = db._guarded[1]                       # P
    whole[4096 + nbytes] = 0
    assert db.check_guards() == ["P"]
    whole[4096 + nbytes] = H.GUARD_BYTE
    whole_ws, _ = db._guarded[6]
    whole_ws[4095] = 0
    assert db.check_guards() == ["workspace"]


def test_no_write_outside_the_buffers_in_the_step_calls(H):
    """The per-step entry points with guard zones round their outputs."""
    import torch
    from paper_1805_08899_amd import binding as eb
    B, Tk, Hh, Dv = 5, 21, 70, 36
    wl = Workload("guard_steps", B, 1, Tk, Hh, Dv, "f32", 0.5, 1, Tk)
    inputs = make_inputs(wl, seed=909)
    db = H.DeviceBatch(wl, inputs, guard_bytes=4096)
    dvp = db._alloc(B * Hh * 4).view(torch.float32)[:B * Hh].view(B, Hh)
    st = torch.cuda.current_stream(db.device)
    for t in (db.dKp, db.dV, db.dv, dvp):
        t.zero_()
    eb.check(eb.echo_attn_step_fwd(db.desc, db.Qp, db.Kp, db.V, db.v, db.key_len, db.context, db.P, stream=st))
    eb.check(eb.echo_attn_step_bwd(db.desc, db.dC, db.P, db.Qp, db.Kp, db.V, db.v, db.key_len, db.dQp, db.dKp, db.dV,
                                   dvp, stream=st))
    eb.check(eb.echo_attn_step_finish(db.desc, dvp, db.dv, stream=st))
    eb.check(eb.echo_attn_bwd_accumulate(db.desc, db.dC, db.P, db.Qp, db.Kp, db.V, db.v, db.key_len, db.dQp, db.dKp,
                                         db.dV, db.dv, db.ws, stream=st))
    assert db.check_guards() == []


def test_large_preactivations_take_the_exact_path(H):
    """|Qp + Kp| up to 100: tanh must saturate to +-1 with no NaN, and rows
    beyond the factorisation limit must still be right next to ordinary rows."""
    wl = Workload("saturating", 2, 10, 20, 96, 8, "f32", 0.5, 5, 20)
    inputs = make_inputs(wl, seed=77)
    inputs["Qp"][0, 3, :] = 60.0
    inputs["Kp"][0, 2, :] = 40.0
    inputs["Kp"][0, 4, :] = -59.5          # q + k = 0.5 with both far beyond the limit
    inputs["Qp"][1, 7, 5:50] = -45.0
    inputs["Kp"][1, 1, 10:60] = 44.0
    inputs["key_len"][:] = [20, 9]
    print("saturating case", flush=True)
    _, got = run_gpu(H, wl, inputs)
    ref = oracle_outputs(inputs, workers=1)
    assert_parity(got, ref, inputs, "f32", "saturating")


def test_extreme_entries_of_v(H):
    """The forward kernel divides by v (v r = 1 / (1/v + (exp(2q)/v) exp(2k))) and lets two neighbouring h share a
    reciprocal: entries of v that are zero, denormal or tiny must count as zero without disturbing their
    neighbour in the pair, whichever of the two they are, and a pair of them must vanish."""
    wl = Workload("tiny_v", 3, 9, 13, 64, 8, "f32", 0.5, 1, 13)
    inputs = make_inputs(wl, seed=91)
    v = inputs["v"]
    v[0] = 0.0            # first of a pair, neighbour ordinary
    v[3] = 1e-20          # second of a pair
    v[4] = -1e-30
    v[5] = 1e-38          # a pair of negligible entries, one of them denormal
    v[10] = -0.0
    v[11] = 0.0           # a pair of zeros
    v[17] = 1e-17         # just above the cut: kept
    print("tiny v case", flush=True)
    _, got = run_gpu(H, wl, inputs)
    ref = oracle_outputs(inputs, workers=1)
    assert_parity(got, ref, inputs, "f32", "tiny v")


def test_huge_entries_of_v_take_the_exact_path(H):
    """|v| beyond 1e15 would let products of two 1/v underflow: such blocks take the routine that exponentiates the
    sum.  The scores are then of the order of 1e16 and the softmax picks one key; forward outputs against the
    oracle, gradients finite (they are differences of rounding errors on both sides)."""
    wl = Workload("huge_v", 2, 9, 13, 64, 8, "f32", 0.5, 2, 13)
    inputs = make_inputs(wl, seed=92)
    inputs["v"][7] = 3e15
    inputs["v"][20] = -2e16
    print("huge v case", flush=True)
    _, got = run_gpu(H, wl, inputs)
    ref = oracle_outputs(inputs, workers=1)
    for k in ("context", "P"):
        assert rel_err(got[k], ref[k]) <= 1e-4, k
    for k in ("dQp", "dKp", "dV", "dv"):
        assert np.isfinite(got[k]).all(), k


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_stash_variant_matches(H, idx):
    """The keep-the-feature-map baseline gives the same results, and its map holds tanh(Qp + Kp) at the valid
    keys.  Workloads 0 and 1 against the oracle; the large ones (maps of 1.3 to 11.8 GB) against the recomputing
    path on the same inputs, which test_workload_parity holds to the oracle, and on sampled entries of the map."""
    wl = WORKLOADS[idx]
    print("stash variant", wl.name, flush=True)
    inputs = make_inputs(wl)
    db, got = run_gpu(H, wl, inputs, stash=True)
    if idx <= 1:
        ref = oracle_outputs(inputs, workers=1 if idx == 0 else None)
        assert_parity(got, ref, inputs, wl.in_dtype, wl.name + " (stash)")
    else:
        _, rec = run_gpu(H, wl, inputs)
        for k in KEYS:
            e = rel_err(got[k], rec[k])
            print(f"  {k}: stash against recompute {e:.2e}", flush=True)
            assert e <= 2e-5, k
    tm = db.tanh_map.view(wl.B, wl.Tq, wl.Tk, wl.H)
    for b in (0, wl.B - 1):
        L = int(inputs["key_len"][b])
        rows = range(wl.Tq) if idx <= 1 else (0, wl.Tq // 2, wl.Tq - 1)
        for i in rows:
            want = np.tanh(inputs["Qp"][b, i].astype(np.float64)[None, :] + inputs["Kp"][b, :L].astype(np.float64))
            assert np.abs(tm[b, i, :L].cpu().numpy() - want).max() < 5e-7


def test_forward_only_and_backward_from_given_P(H):
    """The backward call must use the P it is handed (here: the oracle's)."""
    import torch
    wl = WORKLOADS[0]
    inputs = make_inputs(wl, seed=5)
    ref = oracle_outputs(inputs, workers=1)
    db = H.DeviceBatch(wl, inputs)
    db.poison_outputs()
    db.P.copy_(torch.from_numpy(ref["P"].astype(np.float32)))
    db.bwd()
    got = db.results()
    for k in ("dQp", "dKp", "dV", "dv"):
        assert rel_err(got[k], ref[k]) <= 1e-4, k


def test_forward_alone_without_a_workspace(H):
    """A forward-only caller of a shape that takes the one-kernel forward allocates nothing: 0 bytes are asked
    for and workspace = NULL is accepted."""
    import torch
    from paper_1805_08899_amd import binding as eb
    wl = WORKLOADS[0]
    inputs = make_inputs(wl, seed=6)
    ref = oracle_outputs(inputs, workers=1)
    db = H.DeviceBatch(wl, inputs)
    assert eb.echo_attn_fwd_workspace_bytes(db.desc) == 0
    db.poison_outputs()
    eb.check(eb.echo_attn_fwd(db.desc, db.Qp, db.Kp, db.V, db.v, db.key_len, db.context, db.P, None, 0,
                              stream=torch.cuda.current_stream(db.device)), "echo_attn_fwd without workspace")
    got = db.results()
    for k in ("context", "P"):
        assert rel_err(got[k], ref[k]) <= 1e-4, k


STEP_CASES = [
    # name, B, T (decoder steps), Tk, H, Dv, dtype
    ("steps_tiny", 5, 6, 9, 64, 16, "f32"),
    ("steps_nmt_like", 16, 7, 50, 512, 512, "f32"),
    ("steps_bf16", 6, 4, 21, 128, 64, "bf16"),
    ("steps_ragged_h_many_keys", 3, 3, 77, 70, 36, "f32"),
    ("steps_h_not_multiple_of_4", 2, 2, 11, 33, 8, "f32"),
    ("steps_64_keys_ragged_second_chunk", 5, 3, 64, 260, 264, "f32"),      # the short-axis kernels at their limit
    ("steps_65_keys", 3, 2, 65, 64, 32, "bf16"),                           # one key beyond it
    ("steps_132_keys", 3, 5, 132, 64, 72, "f32"),                          # dV by panels of 64 keys, accumulating
    ("steps_with_empty_samples", 9, 2, 6, 32, 16, "f32"),                  # key_len drawn from 0..Tk
    ("steps_batch_beyond_the_four_block_form", 70, 2, 20, 64, 32, "f32"),  # 4 B blocks would not all run at once
]


@pytest.mark.parametrize("case", STEP_CASES, ids=[c[0] for c in STEP_CASES])
def test_decoder_steps_match_the_batched_layer(H, case):
    """Per-step decoder form: T calls with one query each (forward), then T calls of the accumulating backward,
    against the oracle run once on the T queries stacked along Tq.  The keys, values and v are shared by the
    steps, so dKp, dV and dv are sums over the steps."""
    import torch
    from paper_1805_08899_amd import binding as eb
    name, B, T, Tk, Hh, Dv, dt = case
    print("decoder steps", case, flush=True)
    wl = Workload(name, B, T, Tk, Hh, Dv, dt, 0.5, 0 if "empty" in name else 1, Tk, dt == "bf16")
    inputs = make_inputs(wl, seed=4321 + T)
    if "empty" in name:
        inputs["key_len"][0] = 0                          # at least one sample without a valid key
    ref = oracle_outputs(inputs, workers=1)
    full = H.DeviceBatch(wl, inputs)                     # device copies of Kp, V, v, key_len, dC
    step_desc = eb.make_desc(B, 1, Tk, Hh, Dv, dt)
    ws = torch.empty(max(eb.echo_attn_fwd_workspace_bytes(step_desc), eb.echo_attn_bwd_workspace_bytes(step_desc), 16),
                     dtype=torch.uint8, device=full.device)
    st = torch.cuda.current_stream(full.device)
    f32 = dict(dtype=torch.float32, device=full.device)
    # one allocation per step and tensor: the library wants 16-byte aligned pointers
    ctx = [torch.full((B, 1, Dv), float("nan"), **f32) for _ in range(T)]
    P = [torch.full((B, 1, Tk), float("nan"), **f32) for _ in range(T)]
    dQ = [torch.full((B, 1, Hh), float("nan"), **f32) for _ in range(T)]
    q_steps = [full.Qp[:, t:t + 1, :].contiguous() for t in range(T)]
    dc_steps = [full.dC[:, t:t + 1, :].contiguous() for t in range(T)]
    for t in range(T):
        eb.check(eb.echo_attn_fwd(step_desc, q_steps[t], full.Kp, full.V, full.v, full.key_len, ctx[t], P[t], ws,
                                  stream=st), "step fwd")
    dK = torch.zeros(B, Tk, Hh, **f32)
    dV = torch.zeros(B, Tk, Dv, **f32)
    dv = torch.zeros(Hh, **f32)
    for t in reversed(range(T)):                          # back-propagation through time visits the steps in reverse
        eb.check(eb.echo_attn_bwd_accumulate(step_desc, dc_steps[t], P[t], q_steps[t], full.Kp, full.V, full.v,
                                             full.key_len, dQ[t], dK, dV, dv, ws, stream=st), "step bwd")
    torch.cuda.synchronize(full.device)
    got = {"context": torch.cat(ctx, dim=1).cpu().numpy(), "P": torch.cat(P, dim=1).cpu().numpy(),
           "dQp": torch.cat(dQ, dim=1).cpu().numpy(), "dKp": dK.cpu().numpy(), "dV": dV.cpu().numpy(),
           "dv": dv.cpu().numpy()}
    assert_parity(got, ref, inputs, dt, name)
    # the same steps through the one-launch step kernel: per-sample parts of dv, summed once at the end
    dQ1 = [torch.full((B, 1, Hh), float("nan"), **f32) for _ in range(T)]
    dK1 = torch.zeros(B, Tk, Hh, **f32)
    dV1 = torch.zeros(B, Tk, Dv, **f32)
    dvp = torch.zeros(B, Hh, **f32)
    dv1 = torch.full((Hh,), float("nan"), **f32)
    ctx1 = [torch.full((B, 1, Dv), float("nan"), **f32) for _ in range(T)]
    P1 = [torch.full((B, 1, Tk), float("nan"), **f32) for _ in range(T)]
    for t in range(T):
        eb.check(eb.echo_attn_step_fwd(step_desc, q_steps[t], full.Kp, full.V, full.v, full.key_len, ctx1[t], P1[t],
                                       stream=st), "fused step fwd")
    for t in reversed(range(T)):
        eb.check(eb.echo_attn_step_bwd(step_desc, dc_steps[t], P1[t], q_steps[t], full.Kp, full.V, full.v,
                                       full.key_len, dQ1[t], dK1, dV1, dvp, stream=st), "fused step bwd")
    eb.check(eb.echo_attn_step_finish(step_desc, dvp, dv1, stream=st), "step finish")
    torch.cuda.synchronize(full.device)
    got1 = {"context": torch.cat(ctx1, dim=1).cpu().numpy(), "P": torch.cat(P1, dim=1).cpu().numpy(),
            "dQp": torch.cat(dQ1, dim=1).cpu().numpy(), "dKp": dK1.cpu().numpy(), "dV": dV1.cpu().numpy(),
            "dv": dv1.cpu().numpy()}
    assert_parity(got1, ref, inputs, dt, name + " (one-launch steps)")
    # the same steps with the key-side gradients deferred to one call per sentence
    sent_desc = eb.make_desc(B, T, Tk, Hh, Dv, dt)
    ds_rows = torch.full((eb.echo_attn_steps_ds_bytes(sent_desc),), 0xFF, dtype=torch.uint8, device=full.device)
    ws2 = torch.full((eb.echo_attn_bwd_workspace_bytes(sent_desc),), 0xFF, dtype=torch.uint8, device=full.device)
    dQ2 = [torch.full((B, 1, Hh), float("nan"), **f32) for _ in range(T)]
    dK2, dV2 = torch.full((B, Tk, Hh), float("nan"), **f32), torch.full((B, Tk, Dv), float("nan"), **f32)
    dv2 = torch.full((Hh,), float("nan"), **f32)
    for t in reversed(range(T)):
        eb.check(eb.echo_attn_step_bwd_query(step_desc, t, T, dc_steps[t], P1[t], q_steps[t], full.Kp, full.V, full.v,
                                             full.key_len, dQ2[t], ds_rows, stream=st), "step bwd, query side")
    P_all = torch.cat(P1, dim=1).contiguous()
    eb.check(eb.echo_attn_steps_bwd_keys(sent_desc, full.dC, P_all, full.Qp, full.Kp, full.v, full.key_len, ds_rows,
                                         dK2, dV2, dv2, ws2, stream=st), "sentence bwd, key side")
    torch.cuda.synchronize(full.device)
    got2 = dict(got1, dQp=torch.cat(dQ2, dim=1).cpu().numpy(), dKp=dK2.cpu().numpy(), dV=dV2.cpu().numpy(),
                dv=dv2.cpu().numpy())
    assert_parity(got2, ref, inputs, dt, name + " (key side deferred)")
