"""Device-buffer plumbing around the binding for tests, smoke and benchmark:
uploads one generated batch with torch, allocates outputs and workspace, and
calls the C ABI on torch's current stream.  No arithmetic happens here.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as eb


GUARD_BYTE = 0xA5


class DeviceBatch:
    """Inputs of one workload resident on the GPU plus output/workspace buffers.

    guard_bytes > 0 places every output and the workspace between two guard zones of that many bytes (a
    multiple of 16) filled with GUARD_BYTE; check_guards() tells whether a call wrote outside its buffers."""

    def __init__(self, wl, inputs, device="cuda:0", stash=False, guard_bytes=0):
        self.wl, self.device = wl, torch.device(device)
        assert guard_bytes % 16 == 0
        self.guard_bytes, self._guarded = guard_bytes, []
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

        def out(*shape):
            n = int(np.prod(shape))
            return self._alloc(n * 4).view(torch.float32)[:n].view(*shape)

        self.context = out(wl.B, wl.Tq, wl.Dv)
        self.P = out(wl.B, wl.Tq, wl.Tk)
        self.dQp = out(wl.B, wl.Tq, wl.H)
        self.dKp = out(wl.B, wl.Tk, wl.H)
        self.dV = out(wl.B, wl.Tk, wl.Dv)
        self.dv = out(wl.H)
        self.fwd_ws_bytes = eb.echo_attn_fwd_workspace_bytes(self.desc)
        self.bwd_ws_bytes = eb.echo_attn_bwd_workspace_bytes(self.desc)
        if stash:
            self.fwd_ws_bytes = eb.echo_attn_fwd_stash_workspace_bytes(self.desc)
        self.ws = self._alloc(max(self.fwd_ws_bytes, self.bwd_ws_bytes, 16))
        self.tanh_map = None
        if stash:
            self.tanh_map = torch.empty(eb.echo_attn_stash_bytes(self.desc) // 4, **f32)

    def _alloc(self, nbytes):
        """nbytes of uint8 (rounded up to 16) on the device, between guard zones if asked for."""
        g = self.guard_bytes
        if g == 0:
            return torch.empty((nbytes + 15) // 16 * 16, dtype=torch.uint8, device=self.device)
        # the rear zone starts right at the end of the buffer (at the next multiple of 4 bytes)
        nbytes = (nbytes + 3) // 4 * 4
        whole = torch.full((nbytes + 2 * g + 16,), GUARD_BYTE, dtype=torch.uint8, device=self.device)
        self._guarded.append((whole, nbytes))
        return whole[g:g + (nbytes + 15) // 16 * 16]

    def check_guards(self):
        """Names (by allocation order) of the buffers whose guard zones no longer hold GUARD_BYTE."""
        torch.cuda.synchronize(self.device)
        g, bad = self.guard_bytes, []
        for k, (whole, nbytes) in enumerate(self._guarded):
            ok = bool((whole[:g] == GUARD_BYTE).all()) and bool((whole[g + nbytes:] == GUARD_BYTE).all())
            if not ok:
                bad.append(("context", "P", "dQp", "dKp", "dV", "dv", "workspace")[k] if k < 7 else str(k))
        return bad

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
