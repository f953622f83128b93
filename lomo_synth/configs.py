"""The five synthetic workloads: tensor lists, shapes, distributions and scalars.

Shapes are those of LLaMA decoder layers (hidden/FFN sizes of the 7B, 13B and 65B
models; untied embedding and lm_head over a 32000-token vocabulary).  A linear
tensor is W [N x K] (N = out features, K = in features) with activations X [T x K]
and upstream gradients dY [T x N], T = batch * seq.  Standard deviations follow the
workload descriptions: X ~ N(0,1), W ~ N(0,0.02), dY ~ N(0, sigma_dy) * loss_scale.
Tensors are listed in backward order (lm_head first, embedding last).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

from .generators import (ROLE_DY, ROLE_W, ROLE_X, normal_f16_np, normal_f16_torch, normal_mult,
                         tensor_key, zipf_ids)

WORKLOAD_NAMES = ("linear1024", "llama7b_layer", "llama7b_stack", "llama13b_stack", "llama65b_stack")


@dataclass(frozen=True)
class TensorSpec:
    kind: str            # "linear" | "embedding" | "vector"
    name: str
    layer: int           # -1 for tensors outside the decoder layers
    index: int           # tensor index inside the layer (stream key component)
    T: int
    N: int               # linear: out features; embedding: vocabulary V; vector: 1
    K: int               # linear: in features; embedding/vector: hidden H
    sigma_x: float = 1.0
    sigma_dy: float = 1e-3
    sigma_w: float = 0.02
    w_const: Optional[float] = None   # gains start at 1.0

    @property
    def n_params(self) -> int:
        return self.N * self.K

    @property
    def w_shape(self) -> Tuple[int, ...]:
        return (self.K,) if self.kind == "vector" else (self.N, self.K)

    @property
    def x_shape(self) -> Tuple[int, int]:
        return (self.T, self.K)          # linear: X; vector: x_hat; embedding: unused

    @property
    def dy_shape(self) -> Tuple[int, int]:
        return (self.T, self.N) if self.kind == "linear" else (self.T, self.K)

    @property
    def gemm_flops(self) -> int:
        return 2 * self.T * self.N * self.K if self.kind == "linear" else 0


@dataclass
class Workload:
    name: str
    seed: int
    T: int
    lr: float
    max_norm: float
    eps: float
    loss_scale: float
    tensors: List[TensorSpec] = field(default_factory=list)
    inject_inf: Optional[Tuple[str, int, int]] = None   # (tensor name, row, col) of dY set to +inf

    # ---- generation -----------------------------------------------------------------
    def key(self, spec: TensorSpec, role: int) -> int:
        return tensor_key(self.seed, spec.layer + 1, spec.index, role)

    def dy_mult(self, spec: TensorSpec) -> np.float32:
        return normal_mult(spec.sigma_dy, self.loss_scale)

    def X_np(self, spec, rows=None, cols=None):
        return normal_f16_np(self.key(spec, ROLE_X), spec.x_shape, normal_mult(spec.sigma_x), rows, cols)

    def dY_np(self, spec, rows=None, cols=None):
        return normal_f16_np(self.key(spec, ROLE_DY), spec.dy_shape, self.dy_mult(spec), rows, cols)

    def W_np(self, spec, rows=None, cols=None):
        if spec.w_const is not None:
            n = spec.K if cols is None else len(cols)
            return np.full((n,), spec.w_const, dtype=np.float16)
        return normal_f16_np(self.key(spec, ROLE_W), spec.w_shape, normal_mult(spec.sigma_w), rows, cols)

    def ids_np(self, spec) -> np.ndarray:
        assert spec.kind == "embedding"
        return zipf_ids(self.seed, spec.T, spec.N, 1.1)

    def X_torch(self, spec, device, out=None):
        return normal_f16_torch(self.key(spec, ROLE_X), spec.x_shape, normal_mult(spec.sigma_x), device, out)

    def dY_torch(self, spec, device, out=None):
        return normal_f16_torch(self.key(spec, ROLE_DY), spec.dy_shape, self.dy_mult(spec), device, out)

    def W_torch(self, spec, device, out=None):
        import torch
        if spec.w_const is not None:
            if out is None:
                return torch.full((spec.K,), spec.w_const, dtype=torch.float16, device=device)
            out.fill_(spec.w_const)
            return out
        return normal_f16_torch(self.key(spec, ROLE_W), spec.w_shape, normal_mult(spec.sigma_w), device, out)

    # ---- bookkeeping ----------------------------------------------------------------
    @property
    def n_params(self) -> int:
        return sum(t.n_params for t in self.tensors)

    @property
    def gemm_flops_per_pass(self) -> int:
        return sum(t.gemm_flops for t in self.tensors)

    def by_name(self, name: str) -> TensorSpec:
        for t in self.tensors:
            if t.name == name:
                return t
        raise KeyError(name)


def _layer_tensors(layer: int, T: int, hidden: int, ffn: int, gains: bool, sigma_dy: float) -> List[TensorSpec]:
    """One decoder layer in backward order: MLP first, attention projections last."""
    L = f"layers.{layer}."
    out = [
        TensorSpec("linear", L + "down_proj", layer, 0, T, hidden, ffn, sigma_dy=sigma_dy),
        TensorSpec("linear", L + "up_proj", layer, 1, T, ffn, hidden, sigma_dy=sigma_dy),
        TensorSpec("linear", L + "gate_proj", layer, 2, T, ffn, hidden, sigma_dy=sigma_dy),
    ]
    if gains:
        out.append(TensorSpec("vector", L + "post_attention_norm", layer, 3, T, 1, hidden,
                              sigma_dy=sigma_dy, w_const=1.0))
    out += [
        TensorSpec("linear", L + "o_proj", layer, 4, T, hidden, hidden, sigma_dy=sigma_dy),
        TensorSpec("linear", L + "v_proj", layer, 5, T, hidden, hidden, sigma_dy=sigma_dy),
        TensorSpec("linear", L + "k_proj", layer, 6, T, hidden, hidden, sigma_dy=sigma_dy),
        TensorSpec("linear", L + "q_proj", layer, 7, T, hidden, hidden, sigma_dy=sigma_dy),
    ]
    if gains:
        out.append(TensorSpec("vector", L + "input_norm", layer, 8, T, 1, hidden,
                              sigma_dy=sigma_dy, w_const=1.0))
    return out


def llama_tensor_list(T: int, hidden: int, ffn: int, n_layers: int, vocab: int,
                      sigma_dy: float = 1e-3, final_norm: bool = False) -> List[TensorSpec]:
    """Whole stack in backward order: lm_head, (final norm), layers L-1..0, embedding."""
    out = [TensorSpec("linear", "lm_head", -1, 0, T, vocab, hidden, sigma_dy=sigma_dy)]
    if final_norm:
        out.append(TensorSpec("vector", "final_norm", -1, 1, T, 1, hidden, sigma_dy=sigma_dy, w_const=1.0))
    for layer in range(n_layers - 1, -1, -1):
        out += _layer_tensors(layer, T, hidden, ffn, True, sigma_dy)
    out.append(TensorSpec("embedding", "embed_tokens", -1, 2, T, vocab, hidden, sigma_dy=sigma_dy))
    return out


def count_params(tensors) -> int:
    return sum(t.n_params for t in tensors)


def workload(name: str) -> Workload:
    """Return one of the five named workloads (or a reduced stack ``<name>:<n_layers>``)."""
    layers_override = None
    if ":" in name:
        name, n = name.split(":")
        layers_override = int(n)
    if name == "linear1024":
        w = Workload(name, 0, 512, 1e-2, 1.0, 1e-6, 1024.0)
        w.tensors = [TensorSpec("linear", "linear", 0, 0, 512, 1024, 1024, sigma_dy=0.01)]
        return w
    if name == "llama7b_layer":
        w = Workload(name, 0, 4096, 1e-2, 1.0, 1e-6, 65536.0)
        w.tensors = _layer_tensors(0, 4096, 4096, 11008, False, 1e-3)
        return w
    table = {
        "llama7b_stack": (8 * 512, 4096, 11008, 32),
        "llama13b_stack": (8 * 1024, 5120, 13824, 40),
        "llama65b_stack": (4 * 512, 8192, 22016, 80),
    }
    if name not in table:
        raise KeyError(f"unknown workload {name!r}; known: {WORKLOAD_NAMES}")
    T, hidden, ffn, n_layers = table[name]
    if layers_override is not None:
        n_layers = layers_override
    w = Workload(name, 0, T, 1e-2, 1.0, 1e-6, 65536.0)
    w.tensors = llama_tensor_list(T, hidden, ffn, n_layers, 32000)
    if name == "llama7b_stack":
        inj_layer = min(17, n_layers - 1)
        w.inject_inf = (f"layers.{inj_layer}.down_proj", 0, 0)
    return w


class StreamedStack:
    """A stack workload whose activations do not stay resident: every parameter tensor is generated once and kept,
    while X / dY (and the dX outputs) live in ONE set of buffers per tensor position of a decoder layer, shared by
    all layers and refilled from the seed whenever a layer's turn comes ("activations regenerated per layer").

    groups[g] is a list of records {kind, name, spec, X | ids, dY, W, dX?} as the step sequencing expects them:
    group 0 = lm_head, groups 1..L = decoder layers from the last to the first, group L + 1 = the embedding.
    prepare(g) refills the shared buffers with group g's inputs (same bits as Workload.X_np / dY_np give on the CPU)."""

    def __init__(self, wl: Workload, device):
        import torch
        self.wl, self.device = wl, device
        f16 = dict(dtype=torch.float16, device=device)
        shared = {}

        def buffers(spec: TensorSpec, slot):
            key = (slot, spec.kind, spec.T, spec.N, spec.K)
            if key not in shared:
                b = {"dY": torch.empty(spec.dy_shape, **f16)}
                if spec.kind != "embedding":
                    b["X"] = torch.empty(spec.x_shape, **f16)
                if spec.kind == "linear":
                    b["dX"] = torch.empty(spec.T, spec.K, **f16)
                shared[key] = b
            return shared[key]

        self.groups, self.specs = [], []
        order = []          # (group key, spec) in list order
        for spec in wl.tensors:
            gkey = spec.layer if spec.layer >= 0 else spec.name
            if not order or order[-1][0] != gkey:
                order.append((gkey, []))
            order[-1][1].append(spec)
        for gkey, specs in order:
            recs = []
            for spec in specs:
                slot = spec.index if spec.layer >= 0 else spec.name
                rec = {"kind": spec.kind, "name": spec.name, "spec": spec, "W": wl.W_torch(spec, device)}
                rec.update(buffers(spec, slot))
                if spec.kind == "embedding":
                    rec["ids"] = torch.from_numpy(wl.ids_np(spec)).to(device)
                recs.append(rec)
            self.groups.append(recs)
        self.shared_bytes = sum(t.numel() * 2 for b in shared.values() for t in b.values())

    def prepare(self, g: int) -> None:
        for rec in self.groups[g]:
            spec = rec["spec"]
            self.wl.dY_torch(spec, self.device, out=rec["dY"])
            if spec.kind != "embedding":
                self.wl.X_torch(spec, self.device, out=rec["X"])
