"""Device-buffer plumbing around the binding for tests, smoke and benchmark:
uploads one generated batch with torch, allocates outputs and workspace, and
calls the C ABI on torch's current stream.  No arithmetic happens here.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as eb


class DeviceBatch:
    """Inputs of one workload resident on the GPU plus output/workspace buffers."""

    def __init__(self, wl, inputs, device="cuda:0", stash=False):
        self.wl, self.device = wl, torch.device(device)
        self.desc = eb.make_desc(wl.B, wl.Tq, wl.Tk, wl.H, wl.Dv, wl.in_dtype)
        dev = self.device

        def up(name):
            if wl.in_dtype == "bf16":
                bits = torch.from_numpy(inputs[name + "_bits"].view(np.int16)).to(dev)
                return bits.view(torch.bfloat16)
            return torch.from_numpy(inputs[name]).to(dev)

        self.Qp, self.Kp, self.V, self.v = up("Qp"), up("Kp"), up("V"), up("v")
        self.key_len = torch.from_numpy(inputs["key_len"]).to(dev)
        self.dC = torch.from_numpy(inputs["dContext"]).to(dev)
        f32 = dict(dtype=torch.float32, device=dev)
        self.context = torch.empty(wl.B, wl.Tq, wl.Dv, **f32)
        self.P = torch.empty(wl.B, wl.Tq, wl.Tk, **f32)
        self.dQp = torch.empty(wl.B, wl.Tq, wl.H, **f32)
        self.dKp = torch.empty(wl.B, wl.Tk, wl.H, **f32)
        self.dV = torch.empty(wl.B, wl.Tk, wl.Dv, **f32)
        self.dv = torch.empty(wl.H, **f32)
        self.fwd_ws_bytes = eb.echo_attn_fwd_workspace_bytes(self.desc)
        self.bwd_ws_bytes = eb.echo_attn_bwd_workspace_bytes(self.desc)
        self.ws = torch.empty(max(self.fwd_ws_bytes, self.bwd_ws_bytes, 16), dtype=torch.uint8, device=dev)
        self.tanh_map = None
        if stash:
            self.tanh_map = torch.empty(eb.echo_attn_stash_bytes(self.desc) // 4, **f32)

    def _stream(self):
        return torch.cuda.current_stream(self.device)

    def fwd(self):
        eb.check(eb.echo_attn_fwd(self.desc, self.Qp, self.Kp, self.V, self.v, self.key_len, self.context, self.P,
                                  self.ws, stream=self._stream()), "echo_attn_fwd")

    def bwd(self):
        eb.check(eb.echo_attn_bwd(self.desc, self.dC, self.P, self.Qp, self.Kp, self.V, self.v, self.key_len,
                                  self.dQp, self.dKp, self.dV, self.dv, self.ws, stream=self._stream()),
                 "echo_attn_bwd")

    def fwd_stash(self):
        eb.check(eb.echo_attn_fwd_stash(self.desc, self.Qp, self.Kp, self.V, self.v, self.key_len, self.context,
                                        self.P, self.tanh_map, self.ws, stream=self._stream()),
                 "echo_attn_fwd_stash")

    def bwd_stash(self):
        eb.check(eb.echo_attn_bwd_stash(self.desc, self.dC, self.P, self.tanh_map, self.V, self.v, self.key_len,
                                        self.dQp, self.dKp, self.dV, self.dv, self.ws, stream=self._stream()),
                 "echo_attn_bwd_stash")

    def poison_outputs(self):
        """Fill every output and the workspace with NaN patterns so that an
        element the kernels fail to write shows up."""
        for t in (self.context, self.P, self.dQp, self.dKp, self.dV, self.dv):
            t.fill_(float("nan"))
        self.ws.fill_(0xFF)

    def results(self):
        torch.cuda.synchronize(self.device)
        return {k: getattr(self, a).cpu().numpy() for k, a in
                (("context", "context"), ("P", "P"), ("dQp", "dQp"), ("dKp", "dKp"), ("dV", "dV"), ("dv", "dv"))}
