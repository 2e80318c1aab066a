"""Helpers for the GPU parity tests: move seeded inputs to the device, call the
C ABI through the binding, bring results back as numpy arrays."""
from __future__ import annotations

import numpy as np

import mst_inputs as mi


from mst_inputs import bf16_tensor_to_f64, to_device_bf16  # noqa: F401  (re-exported for the tests)


class DeviceRun:
    """Runs forward and backward of the HIP path on device copies of `inp`."""

    def __init__(self, inp: mi.Inputs, M=None, pad_workspace=0):
        import torch
        import paper_2407_15892_amd as mst
        self.mst = mst
        self.torch = torch
        self.inp = inp
        self.M = inp.cfg.M if M is None else M
        self.S, self.d, self.V = inp.cfg.S, inp.cfg.d, inp.cfg.V
        self.H = to_device_bf16(inp.H_bits)
        self.W = to_device_bf16(inp.W_bits)
        self.labels = torch.from_numpy(inp.labels).cuda()
        self.fwd_bytes, self.bwd_bytes = mst.mst_workspace_bytes(self.S, self.d, self.V, self.M)
        self.pad = pad_workspace

    def _ws(self, nbytes, fill=0xA5):
        ws = self.torch.full((nbytes + self.pad,), fill, dtype=self.torch.uint8, device="cuda")
        return ws

    def forward(self, want_lse=True):
        t = self.torch
        ws = self._ws(self.fwd_bytes)
        loss = t.full((1,), float("nan"), dtype=t.float32, device="cuda")
        lse = t.full((self.S,), float("nan"), dtype=t.float32, device="cuda") if want_lse else None
        nv = t.full((1,), -7, dtype=t.int64, device="cuda")
        self.mst.mst_lmhead_ce_fwd(self.H, self.W, self.labels, self.inp.ignore_index, self.M,
                                   ws[: self.fwd_bytes], loss, lse, nv)
        t.cuda.synchronize()
        self.last_ws = ws
        self.lse = lse
        self.nv = nv
        return float(loss.item()), (lse.cpu().numpy().astype(np.float64) if want_lse else None), int(nv.item())

    def backward(self, grad_loss=1.0, use_lse=True, use_nv=True, poison=True):
        """use_lse / use_nv: hand the forward's lse / n_valid to the backward call (else it recomputes them)."""
        t = self.torch
        nv = self.nv if use_nv else None
        if use_lse:
            assert self.lse is not None, "call forward(want_lse=True) first"
            nbytes = self.bwd_bytes if use_nv else self.bwd_bytes + 512
            lse = self.lse
        else:
            nbytes = self.bwd_bytes + 512 + self.fwd_bytes + (self.S * 4 + 255) // 256 * 256
            lse = None
        self.bwd_bytes_used = nbytes
        ws = self._ws(nbytes)
        dH = t.empty((self.S, self.d), dtype=t.bfloat16, device="cuda")
        dW = t.empty((self.V, self.d), dtype=t.float32, device="cuda")
        if poison == "zero":                 # for checks that expect NaN results
            dH.zero_()
            dW.zero_()
        elif poison:
            dH.view(t.int16).fill_(0x7FC0)   # NaN pattern: every element must be overwritten
            dW.fill_(float("nan"))
        self.mst.mst_lmhead_ce_bwd(self.H, self.W, self.labels, self.inp.ignore_index, self.M, grad_loss,
                                   lse, nv, ws[:nbytes], dH, dW)
        t.cuda.synchronize()
        self.last_ws = ws
        self.dH_t, self.dW_t = dH, dW
        return dH, dW
