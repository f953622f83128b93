"""Two-pass LOMO step over a list of tensors: sequencing of C-ABI calls only (no arithmetic).

Pass 1 adds every tensor's squared gradient norm into one device accumulator and raises
per-tensor overflow flags; one host read-back yields the clipping coefficient (computed by the
library's host function); pass 2 applies the fused updates.  Tensors are visited in the order
given (backward order: last layer first).

Every method takes the stream its work is queued on (None: torch's current stream).  The fills and
copies that torch performs for the step (zeroing the accumulator and the flags, the read-back) are
queued on that same stream, and the read-back waits for that stream only.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import torch

from . import binding as B


class LomoStep:
    """grouped=True (default) hands the whole tensor list to lomo_step_norm_pass / lomo_step_update_pass;
    grouped=False makes one C call per tensor in list order.  Results are the same.

    norm_algorithm: route of the linear tensors in the whole-pass norm pass ('direct', 'auto', 'gram').
    The workspace is sized for the tensor list on first use (lomo_step_workspace_bytes) and grows when a
    later list needs more; max_T / max_H give it a floor so that per-tensor calls of that size fit as well."""

    def __init__(self, device="cuda:0", max_T: int = 8192, max_H: int = 8192, max_tensors: int = 1024,
                 grouped: bool = True, norm_algorithm: str = "direct"):
        self.grouped = grouped
        self.norm_algorithm = norm_algorithm
        self._list_cache = None
        self.device = torch.device(device)
        self.acc = torch.zeros(1, dtype=torch.float64, device=self.device)
        self.flags = torch.zeros(max_tensors + 1, dtype=torch.int32, device=self.device)
        nbytes = max(B.lomo_embedding_workspace_bytes(max_T, max_H), B.lomo_vector_workspace_bytes(max_T, max_H), 256)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        assert self.ws.data_ptr() % 256 == 0
        self.scalars = torch.zeros(32, dtype=torch.uint8, device=self.device)      # lomo_step_scalars
        self._scalars_host = torch.zeros(32, dtype=torch.uint8).pin_memory() if self.device.type == "cuda" else None

    @staticmethod
    def _key(tensors):
        """Everything make_tensor_list bakes into the C array: every pointer and every shape of every record."""
        def ptr(v):
            return v.data_ptr() if v is not None else 0
        return tuple((t["kind"], ptr(t.get("X")), ptr(t.get("ids")), ptr(t["dY"]), ptr(t["W"]), ptr(t.get("dX")),
                      tuple(t["dY"].shape), tuple(t["W"].shape)) for t in tensors)

    def _list(self, tensors):
        key = self._key(tensors)
        if self._list_cache is None or self._list_cache[0] != key:
            arr = B.make_tensor_list(tensors)
            need = B.lomo_step_workspace_bytes(arr)
            if need > self.ws.numel():
                self.ws = None          # released before the larger one is requested
                self.ws = torch.empty(need, dtype=torch.uint8, device=self.device)
                assert self.ws.data_ptr() % 256 == 0
            self._list_cache = (key, arr)
        return self._list_cache[1]

    def norm_pass(self, tensors: List[Dict], stream=None):
        n = len(tensors)
        assert n < self.flags.numel()
        with B.on_stream(stream):
            self.acc.zero_()
            self.flags.zero_()
        if self.grouped:
            B.lomo_step_norm_pass(self._list(tensors), self.acc, self.flags, self.ws, stream, self.norm_algorithm)
            return
        for i, t in enumerate(tensors):
            flag = self.flags[i:i + 1]
            if t["kind"] == "linear":
                B.lomo_wgrad_sqnorm_route(t["X"], t["dY"], self.acc, flag, self.norm_algorithm, stream)
            elif t["kind"] == "embedding":
                B.lomo_embedding_sqnorm(t["ids"], t["dY"], t["W"].shape[0], self.ws, self.acc, flag, stream)
            else:
                B.lomo_vector_sqnorm(t["X"], t["dY"], self.ws, self.acc, flag, stream)
        B.lomo_reduce_flags(self.flags[:n], self.flags[n:n + 1], stream)

    def update_pass(self, tensors: List[Dict], lr: float, inv_loss_scale: float, clip: float, stream=None,
                    reuse_grouping: bool = False):
        """reuse_grouping: norm_pass has just run on the same list and nothing else has used the workspace."""
        n = len(tensors)
        step_flag = self.flags[n:n + 1]
        if self.grouped:
            B.lomo_step_update_pass(self._list(tensors), lr, inv_loss_scale, clip, step_flag, self.ws, stream, reuse_grouping)
            return
        for t in tensors:
            if t["kind"] == "linear":
                B.lomo_linear_backward_update(t["X"], t["dY"], t["W"], t.get("dX"), lr, inv_loss_scale, clip,
                                              step_flag, stream)
            elif t["kind"] == "embedding":
                B.lomo_embedding_update(t["ids"], t["dY"], t["W"], lr, inv_loss_scale, clip, self.ws, step_flag, stream)
            else:
                B.lomo_vector_update(t["X"], t["dY"], t["W"], lr, inv_loss_scale, clip, self.ws, step_flag, stream)

    def clip_value_pass(self, tensors: List[Dict], lr: float, inv_loss_scale: float, clip_value: float, stream=None):
        """The single-pass step (section 3.3.1's clipping by value): every gradient element is unscaled, clamped to
        [-clip_value, clip_value] and applied in the same walk; flags[i] rises where tensor i met a non-finite
        element (that element's weight is left alone), flags[n] is their OR."""
        assert self.grouped, "the single-pass step uses the whole-pass call"
        assert len(tensors) < self.flags.numel()
        with B.on_stream(stream):
            self.flags.zero_()
        B.lomo_step_update_pass_clip_value(self._list(tensors), lr, inv_loss_scale, clip_value, self.flags, self.ws, stream)

    def read_back(self, n: int, stream=None) -> Dict:
        """The one host read-back of a step: scaled squared norm, per-tensor flags, step flag."""
        with B.on_stream(stream):      # the blocking copy is queued on, and waits for, the step's stream
            host = torch.cat([self.acc.view(torch.int32), self.flags[:n + 1]]).cpu()
        return {"total_sqnorm": float(host[:2].view(torch.float64)[0]),
                "flags": [bool(v) for v in host[2:2 + n].tolist()], "overflow": bool(host[2 + n])}

    def run(self, tensors: List[Dict], lr: float, loss_scale: float, max_norm: float = 1.0, eps: float = 1e-6,
            stream=None, clip_override: Optional[float] = None) -> Dict:
        n = len(tensors)
        self.norm_pass(tensors, stream)
        back = self.read_back(n, stream)
        sq, flags, overflow = back["total_sqnorm"], back["flags"], back["overflow"]
        clip = B.lomo_clip_coef(sq, loss_scale, max_norm, eps) if clip_override is None else clip_override
        if not overflow:
            self.update_pass(tensors, lr, 1.0 / loss_scale, clip, stream, reuse_grouping=True)
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
        B.lomo_step_update_pass_device(self._list(tensors), self.scalars, step_flag, self.ws, stream, reuse_grouping=True)
        with B.on_stream(stream):
            self._scalars_host.copy_(self.scalars, non_blocking=True)

    def result(self) -> Dict:
        """Scalars of the last run_async step (synchronise the stream first)."""
        return B.unpack_step_scalars(self._scalars_host)


class LomoStreamedStep:
    """The same two-pass step over GROUPS of tensors (say one decoder layer per group) whose inputs do not stay
    resident: before a group's calls in either pass, `prepare(g)` is called so that the caller can put that
    group's X / dY in place (regenerate them, recompute them, fetch them), typically into buffers shared by all
    groups.  Only the parameters stay in memory for the whole step.  One accumulator and one step flag span all
    groups, so norm, coefficient and the skip on overflow are those of the whole step; nothing waits on the host.
    Sequencing only: every computation is a C-ABI call."""

    def __init__(self, device="cuda:0", max_tensors: int = 4096, norm_algorithm: str = "direct"):
        self.device = torch.device(device)
        self.norm_algorithm = norm_algorithm
        self.acc = torch.zeros(1, dtype=torch.float64, device=self.device)
        self.flags = torch.zeros(max_tensors + 1, dtype=torch.int32, device=self.device)
        self.ws = torch.empty(256, dtype=torch.uint8, device=self.device)
        self.scalars = torch.zeros(32, dtype=torch.uint8, device=self.device)
        self._scalars_host = torch.zeros(32, dtype=torch.uint8).pin_memory()
        self._lists = None

    def bind(self, groups: List[List[Dict]]) -> None:
        """Builds the C descriptor arrays once (pointers and shapes must stay as they are until the next bind) and
        sizes the workspace for the most demanding group."""
        lists, bases, base = [], [], 0
        for g in groups:
            lists.append(B.make_tensor_list(g))
            bases.append(base)
            base += len(g) + 1          # each group's pass-1 call also writes its own any-flag behind its tensors' flags
        assert base < self.flags.numel()
        need = max([B.lomo_step_workspace_bytes(a) for a in lists] + [256])
        if need > self.ws.numel():
            self.ws = None
            self.ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        self._lists, self._bases, self._n_flags = lists, bases, base

    def run_async(self, prepare, lr: float, loss_scale: float, max_norm: float = 1.0, eps: float = 1e-6, stream=None,
                  after_update=None) -> None:
        lists, bases, nf = self._lists, self._bases, self._n_flags
        step_flag = self.flags[nf:nf + 1]
        with B.on_stream(stream):
            self.acc.zero_()
            self.flags.zero_()
        for g, (arr, b) in enumerate(zip(lists, bases)):
            prepare(g)
            B.lomo_step_norm_pass(arr, self.acc, self.flags[b:b + len(arr) + 1], self.ws, stream, self.norm_algorithm)
        B.lomo_reduce_flags(self.flags[:nf], step_flag, stream)
        B.lomo_step_scalars_device(self.acc, step_flag, loss_scale, max_norm, eps, lr, self.scalars, stream)
        for g, arr in enumerate(lists):
            prepare(g)
            B.lomo_step_update_pass_device(arr, self.scalars, step_flag, self.ws, stream)
            if after_update is not None:
                after_update(g)
        with B.on_stream(stream):
            self._scalars_host.copy_(self.scalars, non_blocking=True)

    def result(self) -> Dict:
        """Scalars and per-tensor flags (group by group) of the last step; synchronise the stream first."""
        out = B.unpack_step_scalars(self._scalars_host)
        host = self.flags[:self._n_flags].cpu().tolist()
        out["flags"] = [[bool(v) for v in host[b:b + len(arr)]] for arr, b in zip(self._lists, self._bases)]
        return out


class CapturedStep:
    """One whole step (LomoStep.run_async: fills, pass 1, coefficient kernel, pass 2, copy of the scalars to pinned
    memory) recorded once as a HIP graph and replayed with a single launch.  For steps whose kernels are short
    against their launch overhead (a single small layer); the tensors' pointers and shapes, lr and the loss scale are
    part of the recording.  Every node of the graph is a kernel launch or a device-to-host copy (the fills are torch's
    fill kernels, no memset nodes).  The library's timing must be off while recording."""

    def __init__(self, stepper: LomoStep, tensors: List[Dict], lr: float, loss_scale: float, max_norm: float = 1.0,
                 eps: float = 1e-6):
        assert stepper.grouped
        self.stepper = stepper
        side = torch.cuda.Stream(stepper.device)                 # default priority
        side.wait_stream(torch.cuda.current_stream(stepper.device))
        with torch.cuda.stream(side):                             # warm-up outside the recording: workspace, kernel attributes
            stepper.run_async(tensors, lr, loss_scale, max_norm, eps)
        torch.cuda.current_stream(stepper.device).wait_stream(side)
        torch.cuda.synchronize(stepper.device)
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            stepper.run_async(tensors, lr, loss_scale, max_norm, eps)

    def replay(self) -> None:
        self.graph.replay()

    def result(self) -> Dict:
        return self.stepper.result()
