"""Two-pass LOMO step over a list of tensors: sequencing of C-ABI calls only (no arithmetic).

Pass 1 adds every tensor's squared gradient norm into one device accumulator and raises
per-tensor overflow flags; one host read-back yields the clipping coefficient (computed by the
library's host function); pass 2 applies the fused updates.  Tensors are visited in the order
given (backward order: last layer first).
"""
from __future__ import annotations

from typing import Dict, List, Optional

import torch

from . import binding as B


class LomoStep:
    """grouped=True (default) hands the whole tensor list to lomo_step_norm_pass / lomo_step_update_pass;
    grouped=False makes one C call per tensor in list order.  Results are the same."""

    def __init__(self, device="cuda:0", max_T: int = 8192, max_H: int = 8192, max_tensors: int = 1024,
                 grouped: bool = True):
        self.grouped = grouped
        self._lists = {}
        self.device = torch.device(device)
        self.acc = torch.zeros(1, dtype=torch.float64, device=self.device)
        self.flags = torch.zeros(max_tensors + 1, dtype=torch.int32, device=self.device)
        nbytes = max(B.lomo_embedding_workspace_bytes(max_T, max_H), B.lomo_vector_workspace_bytes(max_T, max_H), 256)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        assert self.ws.data_ptr() % 256 == 0
        self.scalars = torch.zeros(32, dtype=torch.uint8, device=self.device)      # lomo_step_scalars
        self._scalars_host = torch.zeros(32, dtype=torch.uint8).pin_memory() if self.device.type == "cuda" else None

    def _list(self, tensors):
        key = tuple((id(t), t["W"].data_ptr(), t["dY"].data_ptr(), (t.get("dX").data_ptr() if t.get("dX") is not None else 0))
                    for t in tensors)
        cached = self._lists.get("k")
        if cached is None or cached[0] != key:
            cached = (key, B.make_tensor_list(tensors))
            self._lists["k"] = cached
        return cached[1]

    def norm_pass(self, tensors: List[Dict], stream=None):
        n = len(tensors)
        assert n < self.flags.numel()
        self.acc.zero_()
        self.flags.zero_()
        if self.grouped:
            B.lomo_step_norm_pass(self._list(tensors), self.acc, self.flags, self.ws, stream)
            return
        for i, t in enumerate(tensors):
            flag = self.flags[i:i + 1]
            if t["kind"] == "linear":
                B.lomo_wgrad_sqnorm(t["X"], t["dY"], self.acc, flag, stream)
            elif t["kind"] == "embedding":
                B.lomo_embedding_sqnorm(t["ids"], t["dY"], t["W"].shape[0], self.ws, self.acc, flag, stream)
            else:
                B.lomo_vector_sqnorm(t["X"], t["dY"], self.ws, self.acc, flag, stream)
        B.lomo_reduce_flags(self.flags[:n], self.flags[n:n + 1], stream)

    def update_pass(self, tensors: List[Dict], lr: float, inv_loss_scale: float, clip: float, stream=None):
        n = len(tensors)
        step_flag = self.flags[n:n + 1]
        if self.grouped:
            B.lomo_step_update_pass(self._list(tensors), lr, inv_loss_scale, clip, step_flag, self.ws, stream)
            return
        for t in tensors:
            if t["kind"] == "linear":
                B.lomo_linear_backward_update(t["X"], t["dY"], t["W"], t.get("dX"), lr, inv_loss_scale, clip,
                                              step_flag, stream)
            elif t["kind"] == "embedding":
                B.lomo_embedding_update(t["ids"], t["dY"], t["W"], lr, inv_loss_scale, clip, self.ws, step_flag, stream)
            else:
                B.lomo_vector_update(t["X"], t["dY"], t["W"], lr, inv_loss_scale, clip, self.ws, step_flag, stream)

    def read_back(self, n: int) -> Dict:
        """The one host read-back of a step: scaled squared norm, per-tensor flags, step flag."""
        host = torch.cat([self.acc.view(torch.int32), self.flags[:n + 1]]).cpu()
        return {"total_sqnorm": float(host[:2].view(torch.float64)[0]),
                "flags": [bool(v) for v in host[2:2 + n].tolist()], "overflow": bool(host[2 + n])}

    def run(self, tensors: List[Dict], lr: float, loss_scale: float, max_norm: float = 1.0, eps: float = 1e-6,
            stream=None, clip_override: Optional[float] = None) -> Dict:
        n = len(tensors)
        self.norm_pass(tensors, stream)
        back = self.read_back(n)
        sq, flags, overflow = back["total_sqnorm"], back["flags"], back["overflow"]
        clip = B.lomo_clip_coef(sq, loss_scale, max_norm, eps) if clip_override is None else clip_override
        if not overflow:
            self.update_pass(tensors, lr, 1.0 / loss_scale, clip, stream)
        return {"total_sqnorm": sq, "flags": flags, "overflow": overflow, "clip_coef": clip,
                "norm": (sq ** 0.5) / loss_scale if sq == sq else float("nan")}

    def run_async(self, tensors: List[Dict], lr: float, loss_scale: float, max_norm: float = 1.0, eps: float = 1e-6,
                  stream=None) -> None:
        """The same step with the coefficient formed on the device: pass 1, coefficient kernel, pass 2 and
        a copy of the step scalars to pinned host memory are queued without any host wait.  Call
        :meth:`result` after synchronising to read norm, coefficient and overflow of the last step."""
        assert self.grouped, "run_async uses the whole-pass calls"
        n = len(tensors)
        self.norm_pass(tensors, stream)
        step_flag = self.flags[n:n + 1]
        B.lomo_step_scalars_device(self.acc, step_flag, loss_scale, max_norm, eps, lr, self.scalars, stream)
        B.lomo_step_update_pass_device(self._list(tensors), self.scalars, step_flag, self.ws, stream)
        if stream is None:
            self._scalars_host.copy_(self.scalars, non_blocking=True)
        else:
            with torch.cuda.stream(stream):
                self._scalars_host.copy_(self.scalars, non_blocking=True)

    def result(self) -> Dict:
        """Scalars of the last run_async step (synchronise the stream first)."""
        return B.unpack_step_scalars(self._scalars_host)
