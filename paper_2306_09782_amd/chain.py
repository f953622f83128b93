"""LOMO's backward loop through one LLaMA feed-forward block: sequencing of C-ABI calls only.

Algorithm 1 of the paper, with the two passes of section 3.3, over the block's parameters in backward
order (W_d, fused W_gu, RMSNorm gain w).  Each pass walks the chain from the block's output gradient dy
down to the gradient of its input: the dX of one linear tensor is the dY of the next.  Pass 1 only
accumulates squared norms and overflow flags; the coefficient is formed on the device; pass 2 walks
the chain again (the hand-on gradients are not kept between the passes) and updates every parameter
right after the gradient of its input has been taken from the old value.  No host wait anywhere.
"""
from __future__ import annotations

from typing import Dict

import torch

from . import binding as B


class LomoMlpBlock:
    """Scratch for the hand-on gradients of one block (da [T x F], [dgate|dup] [T x 2F], dxn [T x H]) plus
    the step state (accumulator, flags, workspace, scalars).  `saved` holds the forward activations the
    backward needs: a [T x F], xn and xhat [T x H], rstd [T] fp32, gate_up [T x 2F]."""

    def __init__(self, device, T: int, H: int, F: int):
        self.device = torch.device(device)
        f16 = dict(dtype=torch.float16, device=self.device)
        self.da = torch.empty(T, F, **f16)
        self.dgu = torch.empty(T, 2 * F, **f16)
        self.dxn = torch.empty(T, H, **f16)
        self.acc = torch.zeros(1, dtype=torch.float64, device=self.device)
        self.flags = torch.zeros(4, dtype=torch.int32, device=self.device)     # W_d, W_gu, w, any
        self.ws = torch.empty(max(B.lomo_vector_workspace_bytes(T, H), 256), dtype=torch.uint8, device=self.device)
        self.scalars = torch.zeros(32, dtype=torch.uint8, device=self.device)
        self._scalars_host = torch.zeros(32, dtype=torch.uint8).pin_memory()
        self._lists = None

    def _tensor_lists(self, dy, saved, w, W_gu, W_d):
        key = tuple(t.data_ptr() for t in (dy, saved["a"], saved["xn"], saved["xhat"], w, W_gu, W_d))
        if self._lists is None or self._lists[0] != key:
            down = B.make_tensor_list([{"kind": "linear", "X": saved["a"], "dY": dy, "W": W_d, "dX": self.da}])
            gu = B.make_tensor_list([{"kind": "linear", "X": saved["xn"], "dY": self.dgu, "W": W_gu, "dX": self.dxn}])
            gain = B.make_tensor_list([{"kind": "vector", "X": saved["xhat"], "dY": self.dxn, "W": w}])
            self._lists = (key, down, gu, gain)
        return self._lists[1:]

    def step(self, dy, saved: Dict, w, W_gu, W_d, dh, lr: float, loss_scale: float, max_norm: float = 1.0,
             eps: float = 1e-6, stream=None) -> None:
        """Queues the whole two-pass step; dh receives the gradient of the block input (residual included)."""
        down, gu, gain = self._tensor_lists(dy, saved, w, W_gu, W_d)
        f = self.flags
        self.acc.zero_()
        f.zero_()
        # ---- pass 1: walk the chain, keep only norms and flags
        B.lomo_linear_dgrad(dy, W_d, self.da, stream)
        B.lomo_wgrad_sqnorm(saved["a"], dy, self.acc, f[0:1], stream)
        B.lomo_swiglu_backward(self.da, saved["gate_up"], self.dgu, stream)
        B.lomo_linear_dgrad(self.dgu, W_gu, self.dxn, stream)
        B.lomo_wgrad_sqnorm(saved["xn"], self.dgu, self.acc, f[1:2], stream)
        B.lomo_vector_sqnorm(saved["xhat"], self.dxn, self.ws, self.acc, f[2:3], stream)
        B.lomo_reduce_flags(f[0:3], f[3:4], stream)
        B.lomo_step_scalars_device(self.acc, f[3:4], loss_scale, max_norm, eps, lr, self.scalars, stream)
        # ---- pass 2: walk it again; every parameter is updated right after its input gradient is taken
        B.lomo_step_update_pass_device(down, self.scalars, f[3:4], self.ws, stream)       # da, then W_d
        B.lomo_swiglu_backward(self.da, saved["gate_up"], self.dgu, stream)
        B.lomo_step_update_pass_device(gu, self.scalars, f[3:4], self.ws, stream)         # dxn, then W_gu
        B.lomo_rmsnorm_backward(self.dxn, saved["xhat"], saved["rstd"], w, dy, dh, stream)  # old gain
        B.lomo_step_update_pass_device(gain, self.scalars, f[3:4], self.ws, stream)       # then the gain
        if stream is None:
            self._scalars_host.copy_(self.scalars, non_blocking=True)
        else:
            with torch.cuda.stream(stream):
                self._scalars_host.copy_(self.scalars, non_blocking=True)

    def result(self) -> Dict:
        """Scalars and flags of the last step (synchronise first)."""
        out = B.unpack_step_scalars(self._scalars_host)
        host = torch.cat([self.acc.view(torch.int32), self.flags]).cpu()
        out["total_sqnorm"] = float(host[:2].view(torch.float64)[0])
        out["flags"] = [bool(v) for v in host[2:5].tolist()]
        return out
