"""Helpers for the MLP GPU parity tests: device copies of seeded inputs, calls through the C ABI."""
from __future__ import annotations

import numpy as np

import mst_inputs as mi
from tests.gpu_harness import bf16_tensor_to_f64, to_device_bf16


class MlpDeviceRun:
    """Runs forward and backward of the HIP MLP path on device copies of `inp`."""

    def __init__(self, inp: mi.MlpInputs, M=None, pad_workspace=0):
        import torch
        import paper_2407_15892_amd as mst
        self.mst, self.torch, self.inp = mst, torch, inp
        self.M = inp.cfg.M if M is None else M
        self.S, self.d, self.I = inp.cfg.S, inp.cfg.d, inp.cfg.I
        self.X = to_device_bf16(inp.X_bits)
        self.Wg = to_device_bf16(inp.Wg_bits)
        self.Wu = to_device_bf16(inp.Wu_bits)
        self.Wd = to_device_bf16(inp.Wd_bits)
        self.dO = to_device_bf16(inp.dO_bits)
        self.fwd_bytes, self.bwd_bytes = mst.mst_mlp_workspace_bytes(self.S, self.d, self.I, self.M)
        self.pad = pad_workspace

    def _ws(self, nbytes, fill=0xA5):
        return self.torch.full((nbytes + self.pad,), fill, dtype=self.torch.uint8, device="cuda")

    def forward(self):
        t = self.torch
        ws = self._ws(self.fwd_bytes)
        O = t.empty((self.S, self.d), dtype=t.bfloat16, device="cuda")
        O.view(t.int16).fill_(0x7FC0)              # NaN pattern: every element must be overwritten
        self.mst.mst_mlp_fwd(self.X, self.Wg, self.Wu, self.Wd, self.M, ws[: self.fwd_bytes], O)
        t.cuda.synchronize()
        self.last_ws = ws
        self.O_t = O
        return O

    def backward(self, dO=None):
        t = self.torch
        ws = self._ws(self.bwd_bytes)
        dX = t.empty((self.S, self.d), dtype=t.bfloat16, device="cuda")
        dX.view(t.int16).fill_(0x7FC0)
        dWg = t.full((self.I, self.d), float("nan"), dtype=t.float32, device="cuda")
        dWu = t.full((self.I, self.d), float("nan"), dtype=t.float32, device="cuda")
        dWd = t.full((self.d, self.I), float("nan"), dtype=t.float32, device="cuda")
        self.mst.mst_mlp_bwd(self.X, self.Wg, self.Wu, self.Wd, self.dO if dO is None else dO, self.M,
                             ws[: self.bwd_bytes], dX, dWg, dWu, dWd)
        t.cuda.synchronize()
        self.last_ws = ws
        return dX, dWg, dWu, dWd


def f64(t) -> np.ndarray:
    import torch
    if t.dtype == torch.bfloat16:
        return bf16_tensor_to_f64(t)
    return t.cpu().numpy().astype(np.float64)
