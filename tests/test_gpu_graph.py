"""The per-step decoder form replayed from a HIP graph (batched launch): every replay must give what the same
calls give when launched one by one.  The library's entry points allocate nothing and never synchronise, so a
sequence of them can be captured; the accumulators are cleared inside the graph with a fill kernel."""
import numpy as np
import pytest

from paper_1805_08899_amd.workloads import Workload, make_inputs
from parity import assert_parity, oracle_outputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("form", ["general_kernels", "step_kernels", "key_side_deferred"])
def test_decoder_steps_from_a_graph(form):
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from paper_1805_08899_amd import binding as eb, harness
    B, T, Tk, Hh, Dv = 8, 5, 30, 256, 128
    wl = Workload("graph_steps", B, T, Tk, Hh, Dv, "f32", 0.5, 3, Tk)
    inputs = make_inputs(wl, seed=99)
    ref = oracle_outputs(inputs, workers=1)
    full = harness.DeviceBatch(wl, inputs)
    dev = full.device
    desc = eb.make_desc(B, 1, Tk, Hh, Dv, "f32")
    ws = torch.empty(max(eb.echo_attn_fwd_workspace_bytes(desc), eb.echo_attn_bwd_workspace_bytes(desc), 16),
                     dtype=torch.uint8, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    q = [full.Qp[:, t:t + 1, :].contiguous() for t in range(T)]
    dc = [full.dC[:, t:t + 1, :].contiguous() for t in range(T)]
    ctx = [torch.empty(B, 1, Dv, **f32) for _ in range(T)]
    P = [torch.empty(B, 1, Tk, **f32) for _ in range(T)]
    dQ = [torch.empty(B, 1, Hh, **f32) for _ in range(T)]
    dK, dV, dv = torch.empty(B, Tk, Hh, **f32), torch.empty(B, Tk, Dv, **f32), torch.empty(Hh, **f32)
    dvp = torch.empty(B, Hh, **f32)

    def sentence_step_kernels():
        st = torch.cuda.current_stream(dev)
        for t in (dK, dV, dvp):
            t.zero_()                                   # a fill kernel, not a memset node
        for t in range(T):
            eb.check(eb.echo_attn_step_fwd(desc, q[t], full.Kp, full.V, full.v, full.key_len, ctx[t], P[t], stream=st))
        for t in reversed(range(T)):
            eb.check(eb.echo_attn_step_bwd(desc, dc[t], P[t], q[t], full.Kp, full.V, full.v, full.key_len, dQ[t], dK,
                                           dV, dvp, stream=st))
        eb.check(eb.echo_attn_step_finish(desc, dvp, dv, stream=st))

    def sentence_general():
        st = torch.cuda.current_stream(dev)
        for t in (dK, dV, dv):
            t.zero_()                                   # a fill kernel, not a memset node
        for t in range(T):
            eb.check(eb.echo_attn_fwd(desc, q[t], full.Kp, full.V, full.v, full.key_len, ctx[t], P[t], ws, stream=st))
        for t in reversed(range(T)):
            eb.check(eb.echo_attn_bwd_accumulate(desc, dc[t], P[t], q[t], full.Kp, full.V, full.v, full.key_len,
                                                 dQ[t], dK, dV, dv, ws, stream=st))

    sent_desc = eb.make_desc(B, T, Tk, Hh, Dv, "f32")
    ds_rows = torch.empty(eb.echo_attn_steps_ds_bytes(sent_desc), dtype=torch.uint8, device=dev)
    ws_sent = torch.empty(eb.echo_attn_bwd_workspace_bytes(sent_desc), dtype=torch.uint8, device=dev)
    P_all = torch.empty(B, T, Tk, **f32)

    def sentence_deferred():
        """Steps that only read; dKp, dV, dv by one call at the end (which runs inter-block flags through its
        workspace: the replays below must find them in a usable state each time)."""
        st = torch.cuda.current_stream(dev)
        for t in range(T):
            eb.check(eb.echo_attn_step_fwd(desc, q[t], full.Kp, full.V, full.v, full.key_len, ctx[t], P[t], stream=st))
        for t in reversed(range(T)):
            eb.check(eb.echo_attn_step_bwd_query(desc, t, T, dc[t], P[t], q[t], full.Kp, full.V, full.v, full.key_len,
                                                 dQ[t], ds_rows, stream=st))
        torch.cat(P, dim=1, out=P_all)
        eb.check(eb.echo_attn_steps_bwd_keys(sent_desc, full.dC, P_all, full.Qp, full.Kp, full.v, full.key_len,
                                             ds_rows, dK, dV, dv, ws_sent, stream=st))

    sentence = {"general_kernels": sentence_general, "step_kernels": sentence_step_kernels,
                "key_side_deferred": sentence_deferred}[form]

    def snapshot():
        torch.cuda.synchronize(dev)
        return {"context": torch.cat(ctx, 1).cpu().numpy(), "P": torch.cat(P, 1).cpu().numpy(),
                "dQp": torch.cat(dQ, 1).cpu().numpy(), "dKp": dK.cpu().numpy(), "dV": dV.cpu().numpy(),
                "dv": dv.cpu().numpy()}

    def poison():
        for t in ctx + P + dQ + [dK, dV, dv, dvp, P_all]:
            t.fill_(float("nan"))
        ds_rows.fill_(0xFF)

    sentence()                                          # eager: also the warm-up before capture
    eager = snapshot()
    assert_parity(eager, ref, inputs, "f32", "eager steps")

    side = torch.cuda.Stream(device=dev)
    side.wait_stream(torch.cuda.current_stream(dev))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sentence()
    torch.cuda.current_stream(dev).wait_stream(side)
    for replay in range(3):
        poison()
        full.fwd(); full.bwd()                          # the program's own eager work between replays
        torch.cuda.synchronize(dev)
        graph.replay()
        got = snapshot()
        for k, v in eager.items():
            assert np.array_equal(got[k], v), f"replay {replay}: {k} differs from the eager launches"
