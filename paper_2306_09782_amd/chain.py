"""LOMO's backward loop through a LLaMA decoder layer: sequencing of C-ABI calls only (no arithmetic).

Algorithm 1 of the paper with the two passes of section 3.3.  Each pass walks the chain from the layer's
output gradient dy down to the gradient of its input: the dX of one linear tensor, passed through the
element-wise / attention backward kernels, is the dY of the next.  Pass 1 only accumulates squared norms
and overflow flags; the coefficient is formed on the device; pass 2 walks the chain again (the hand-on
gradients are not kept between the passes) and updates every parameter right after the gradient of its
input has been taken from the old value.  Nothing waits on the host.

  feed-forward block:  dy -> W_d -> SwiGLU backward -> fused W_gu -> gain w -> RMSNorm backward (+ dy) -> dh
  attention block:     dy -> W_o -> attention + rotary backward -> fused W_qkv -> gain w -> RMSNorm backward (+ dy) -> dh
  decoder layer:       feed-forward block, then the attention block on its dh; one norm over all six parameters
"""
from __future__ import annotations

from typing import Dict

import torch

from . import binding as B


class StepState:
    """Accumulator, per-parameter flags (+ the step flag), workspace and scalars of one chained step."""

    def __init__(self, device, n_params: int, T: int, H: int, with_embedding: bool = False):
        self.n = n_params
        self.acc = torch.zeros(1, dtype=torch.float64, device=device)
        self.flags = torch.zeros(n_params + 1, dtype=torch.int32, device=device)
        nbytes = max(B.lomo_vector_workspace_bytes(T, H), 256)
        if with_embedding:
            nbytes = max(nbytes, B.lomo_embedding_workspace_bytes(T, H))
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.scalars = torch.zeros(32, dtype=torch.uint8, device=device)
        self._scalars_host = torch.zeros(32, dtype=torch.uint8).pin_memory()
        self.device = torch.device(device)
        self.side = None          # second stream for the norm-pass GEMMs (see use_side_stream)

    def use_side_stream(self):
        """Pass 1's norm contractions do not feed the walk: with a second stream (default priority) they run beside
        the dgrad / element-wise / attention kernels that do, and fill each other's partial last rounds.  Only safe
        when no hand-on buffer is reused within a pass (every layer has its own)."""
        self.side = torch.cuda.Stream(self.device)

    def fork(self, stream):
        """Stream for work that depends only on what is already queued on `stream`: the side stream, made to wait
        for that; or `stream` itself when there is no side stream."""
        if self.side is None:
            return stream
        main = stream if stream is not None else torch.cuda.current_stream(self.device)
        ev = torch.cuda.Event()
        ev.record(main)
        self.side.wait_event(ev)
        return self.side

    def join(self, stream):
        if self.side is None:
            return
        main = stream if stream is not None else torch.cuda.current_stream(self.device)
        ev = torch.cuda.Event()
        ev.record(self.side)
        main.wait_event(ev)

    @property
    def step_flag(self):
        return self.flags[self.n:self.n + 1]

    def begin(self, stream=None):
        with B.on_stream(stream):      # the fills are queued on the step's stream, ahead of pass 1's atomics
            self.acc.zero_()
            self.flags.zero_()

    def coefficient(self, lr, loss_scale, max_norm, eps, stream):
        self.join(stream)
        B.lomo_reduce_flags(self.flags[:self.n], self.step_flag, stream)
        B.lomo_step_scalars_device(self.acc, self.step_flag, loss_scale, max_norm, eps, lr, self.scalars, stream)

    def finish(self, stream):
        with B.on_stream(stream):
            self._scalars_host.copy_(self.scalars, non_blocking=True)

    def result(self) -> Dict:
        """Scalars and flags of the last step (synchronise first)."""
        out = B.unpack_step_scalars(self._scalars_host)
        host = torch.cat([self.acc.view(torch.int32), self.flags]).cpu()
        out["total_sqnorm"] = float(host[:2].view(torch.float64)[0])
        out["flags"] = [bool(v) for v in host[2:2 + self.n].tolist()]
        return out


def _fork(state, stream):
    return state.fork(stream) if getattr(state, "side", None) is not None else stream


def _linear(state: StepState, slot: int, X, dY, W, dX, tensor_list, update: bool, stream):
    """One linear tensor of the walk: hand-on gradient from the old W, then norm (pass 1) or fused update (pass 2)."""
    if update:
        B.lomo_step_update_pass_device(tensor_list, state.scalars, state.step_flag, state.ws, stream)
    else:
        side = _fork(state, stream)          # the norm contraction reads X and dY only: it may run beside the dgrad
        B.lomo_linear_dgrad(dY, W, dX, stream)
        B.lomo_wgrad_sqnorm(X, dY, state.acc, state.flags[slot:slot + 1], side)


def _gain(state: StepState, slot: int, xhat, dxn, w, tensor_list, update: bool, stream):
    if update:
        B.lomo_step_update_pass_device(tensor_list, state.scalars, state.step_flag, state.ws, stream)
    else:
        B.lomo_vector_sqnorm(xhat, dxn, state.ws, state.acc, state.flags[slot:slot + 1], _fork(state, stream))


class LomoMlpBlock:
    """Hand-on buffers of the feed-forward block: da [T x F], [dgate|dup] [T x 2F], dxn [T x H].
    `saved`: a [T x F], xn and xhat [T x H], rstd [T] fp32, gate_up [T x 2F]."""

    def __init__(self, device, T: int, H: int, F: int, state: StepState = None, slot0: int = 0, share=None):
        self.device = torch.device(device)
        f16 = dict(dtype=torch.float16, device=self.device)
        # hand-on buffers are transient: blocks of different layers may share them (`share` = another block)
        self.da = share.da if share is not None else torch.empty(T, F, **f16)
        self.dgu = share.dgu if share is not None else torch.empty(T, 2 * F, **f16)
        self.dxn = share.dxn if share is not None else torch.empty(T, H, **f16)
        self.state = state if state is not None else StepState(self.device, 3, T, H)
        self.slot0 = slot0
        self._lists = None

    def _tensor_lists(self, dy, saved, w, W_gu, W_d):
        key = tuple(t.data_ptr() for t in (dy, saved["a"], saved["xn"], saved["xhat"], w, W_gu, W_d))
        if self._lists is None or self._lists[0] != key:
            down = B.make_tensor_list([{"kind": "linear", "X": saved["a"], "dY": dy, "W": W_d, "dX": self.da}])
            gu = B.make_tensor_list([{"kind": "linear", "X": saved["xn"], "dY": self.dgu, "W": W_gu, "dX": self.dxn}])
            gain = B.make_tensor_list([{"kind": "vector", "X": saved["xhat"], "dY": self.dxn, "W": w}])
            self._lists = (key, down, gu, gain)
        return self._lists[1:]

    def walk(self, dy, saved: Dict, w, W_gu, W_d, dh, update: bool, stream=None):
        down, gu, gain = self._tensor_lists(dy, saved, w, W_gu, W_d)
        st, k = self.state, self.slot0
        _linear(st, k, saved["a"], dy, W_d, self.da, down, update, stream)
        B.lomo_swiglu_backward(self.da, saved["gate_up"], self.dgu, stream)
        _linear(st, k + 1, saved["xn"], self.dgu, W_gu, self.dxn, gu, update, stream)
        B.lomo_rmsnorm_backward(self.dxn, saved["xhat"], saved["rstd"], w, dy, dh, stream)     # old gain
        _gain(st, k + 2, saved["xhat"], self.dxn, w, gain, update, stream)

    def step(self, dy, saved: Dict, w, W_gu, W_d, dh, lr: float, loss_scale: float, max_norm: float = 1.0,
             eps: float = 1e-6, stream=None) -> None:
        """Queues the whole two-pass step of this block alone; dh receives the gradient of the block input."""
        self.state.begin(stream)
        self.walk(dy, saved, w, W_gu, W_d, dh, False, stream)
        self.state.coefficient(lr, loss_scale, max_norm, eps, stream)
        self.walk(dy, saved, w, W_gu, W_d, dh, True, stream)
        self.state.finish(stream)

    def result(self) -> Dict:
        return self.state.result()


class LomoAttentionBlock:
    """Hand-on buffers of the attention block: do [T x H], [dq|dk|dv] [T x 3H], dxn [T x H], delta [T x heads].
    `saved`: o, xn, xhat [T x H], rstd [T] fp32, qkv [T x 3H] (rotated q and k, v), lse [T x heads] fp32."""

    def __init__(self, device, batch: int, seq: int, H: int, n_heads: int, state: StepState = None, slot0: int = 0,
                 share=None):
        self.device = torch.device(device)
        T = batch * seq
        self.batch, self.seq, self.n_heads = batch, seq, n_heads
        f16 = dict(dtype=torch.float16, device=self.device)
        self.do = share.do if share is not None else torch.empty(T, H, **f16)
        self.dqkv = share.dqkv if share is not None else torch.empty(T, 3 * H, **f16)
        self.dxn = share.dxn if share is not None else torch.empty(T, H, **f16)
        self.delta = share.delta if share is not None else torch.empty(T * n_heads, dtype=torch.float32, device=self.device)
        self.state = state if state is not None else StepState(self.device, 3, T, H)
        self.slot0 = slot0
        self._lists = None

    def _tensor_lists(self, dy, saved, w, W_qkv, W_o):
        key = tuple(t.data_ptr() for t in (dy, saved["o"], saved["xn"], saved["xhat"], w, W_qkv, W_o))
        if self._lists is None or self._lists[0] != key:
            out = B.make_tensor_list([{"kind": "linear", "X": saved["o"], "dY": dy, "W": W_o, "dX": self.do}])
            qkv = B.make_tensor_list([{"kind": "linear", "X": saved["xn"], "dY": self.dqkv, "W": W_qkv, "dX": self.dxn}])
            gain = B.make_tensor_list([{"kind": "vector", "X": saved["xhat"], "dY": self.dxn, "W": w}])
            self._lists = (key, out, qkv, gain)
        return self._lists[1:]

    def walk(self, dy, saved: Dict, w, W_qkv, W_o, rope_cos, rope_sin, dh, update: bool, stream=None):
        out, qkv, gain = self._tensor_lists(dy, saved, w, W_qkv, W_o)
        st, k = self.state, self.slot0
        _linear(st, k, saved["o"], dy, W_o, self.do, out, update, stream)
        B.lomo_attention_backward(saved["qkv"], saved["o"], self.do, saved["lse"], rope_cos, rope_sin, self.delta,
                                  self.dqkv, self.batch, self.seq, self.n_heads, stream)
        _linear(st, k + 1, saved["xn"], self.dqkv, W_qkv, self.dxn, qkv, update, stream)
        B.lomo_rmsnorm_backward(self.dxn, saved["xhat"], saved["rstd"], w, dy, dh, stream)
        _gain(st, k + 2, saved["xhat"], self.dxn, w, gain, update, stream)

    def step(self, dy, saved: Dict, w, W_qkv, W_o, rope_cos, rope_sin, dh, lr: float, loss_scale: float,
             max_norm: float = 1.0, eps: float = 1e-6, stream=None) -> None:
        self.state.begin(stream)
        self.walk(dy, saved, w, W_qkv, W_o, rope_cos, rope_sin, dh, False, stream)
        self.state.coefficient(lr, loss_scale, max_norm, eps, stream)
        self.walk(dy, saved, w, W_qkv, W_o, rope_cos, rope_sin, dh, True, stream)
        self.state.finish(stream)

    def result(self) -> Dict:
        return self.state.result()


class LomoDecoderLayer:
    """Both blocks under one step: flags in backward order W_d, W_gu, w2, W_o, W_qkv, w1."""

    def __init__(self, device, batch: int, seq: int, H: int, F: int, n_heads: int):
        self.device = torch.device(device)
        T = batch * seq
        self.state = StepState(self.device, 6, T, H)
        self.mlp = LomoMlpBlock(self.device, T, H, F, self.state, 0)
        self.attn = LomoAttentionBlock(self.device, batch, seq, H, n_heads, self.state, 3)
        self.dh_mid = torch.empty(T, H, dtype=torch.float16, device=self.device)

    def _walk(self, dy, saved_attn, saved_mlp, p, rope_cos, rope_sin, dh, update, stream):
        self.mlp.walk(dy, saved_mlp, p["w2"], p["W_gu"], p["W_d"], self.dh_mid, update, stream)
        self.attn.walk(self.dh_mid, saved_attn, p["w1"], p["W_qkv"], p["W_o"], rope_cos, rope_sin, dh, update, stream)

    def step(self, dy, saved_attn: Dict, saved_mlp: Dict, p: Dict, rope_cos, rope_sin, dh, lr: float, loss_scale: float,
             max_norm: float = 1.0, eps: float = 1e-6, stream=None) -> None:
        """p: {"w1", "W_qkv", "W_o", "w2", "W_gu", "W_d"} device tensors, updated in place; dh: gradient of the layer input."""
        self.state.begin(stream)
        self._walk(dy, saved_attn, saved_mlp, p, rope_cos, rope_sin, dh, False, stream)
        self.state.coefficient(lr, loss_scale, max_norm, eps, stream)
        self._walk(dy, saved_attn, saved_mlp, p, rope_cos, rope_sin, dh, True, stream)
        self.state.finish(stream)

    def result(self) -> Dict:
        return self.state.result()


class LomoModelChain:
    """Algorithm 1 over a whole decoder-only model: output projection W_lm, final RMSNorm gain, the layers from
    the last to the first, and the embedding table, under one two-pass step.  Parameter (= flag) order:
    W_lm, w_f, then per layer (last first) W_d, W_gu, w2, W_o, W_qkv, w1, finally W_emb.

    The hand-on gradients live only until the next stage has read them, so by default all layers share one set
    of buffers and the gradient between layers alternates between two [T x H] buffers (section 3.2: no gradient
    outlives its use).  `share_buffers=False` keeps every layer's hand-ons, for inspection.

    `keep_handons=True` trades memory for arithmetic: every layer keeps the hand-on gradients of pass 1 (about
    as many bytes again as the saved activations: 0.54 GB per 7B layer at 4096 tokens), so pass 2 has no walk to
    repeat and is one grouped launch of the fused gradient + update over every tensor of the model: three GEMMs
    per linear tensor instead of four, and no second attention / SwiGLU / RMSNorm backward.  The parameters come
    out bit-identical to the re-walked step, since the hand-ons of both passes are the same bits."""

    def __init__(self, device, batch: int, seq: int, H: int, F: int, n_heads: int, n_layers: int,
                 share_buffers: bool = True, keep_handons: bool = False, overlap_norm_pass: bool = False):
        self.device = torch.device(device)
        T = batch * seq
        self.n_layers = n_layers
        self.keep_handons = keep_handons
        share_buffers = share_buffers and not keep_handons
        assert not overlap_norm_pass or not share_buffers, "a side stream needs hand-on buffers that are not reused"
        self._all = None
        self.state = StepState(self.device, 2 + 6 * n_layers + 1, T, H, with_embedding=True)
        if overlap_norm_pass:
            self.state.use_side_stream()
        self.mlp, self.attn = [], []
        for k in range(n_layers):                      # k-th layer of the walk = layer n_layers - 1 - k
            slot = 2 + 6 * k
            first = k == 0 or not share_buffers
            self.mlp.append(LomoMlpBlock(self.device, T, H, F, self.state, slot, share=None if first else self.mlp[0]))
            self.attn.append(LomoAttentionBlock(self.device, batch, seq, H, n_heads, self.state, slot + 3,
                                                share=None if first else self.attn[0]))
        f16 = dict(dtype=torch.float16, device=self.device)
        self.dxn_f = torch.empty(T, H, **f16)
        n_dy = 2 if share_buffers else n_layers + 1
        self.dy = [torch.empty(T, H, **f16) for _ in range(n_dy)]          # dy[k % n_dy]: gradient entering walk step k
        self.dh_mid = [torch.empty(T, H, **f16) for _ in range(1 if share_buffers else n_layers)]
        self._top = None

    def grad_in(self, k: int):
        """Buffer holding the gradient that enters the k-th layer of the walk (k = n_layers: the embedding's)."""
        return self.dy[k % len(self.dy)]

    def grad_mid(self, k: int):
        return self.dh_mid[k % len(self.dh_mid)]

    def _top_lists(self, dlogits, final, m, ids, dh0):
        key = tuple(t.data_ptr() for t in (dlogits, final["xn"], final["xhat"], m["W_lm"], m["w_f"], m["W_emb"], ids, dh0))
        if self._top is None or self._top[0] != key:
            lm = B.make_tensor_list([{"kind": "linear", "X": final["xn"], "dY": dlogits, "W": m["W_lm"], "dX": self.dxn_f}])
            gain = B.make_tensor_list([{"kind": "vector", "X": final["xhat"], "dY": self.dxn_f, "W": m["w_f"]}])
            emb = B.make_tensor_list([{"kind": "embedding", "ids": ids, "dY": dh0, "W": m["W_emb"]}])
            self._top = (key, lm, gain, emb)
        return self._top[1:]

    def _walk(self, ids, dlogits, saved, m, rope_cos, rope_sin, update, stream, before_layer=None):
        st = self.state
        final = saved["final"]
        L = self.n_layers
        dh0 = self.grad_in(L)
        lm, gain, emb = self._top_lists(dlogits, final, m, ids, dh0)
        _linear(st, 0, final["xn"], dlogits, m["W_lm"], self.dxn_f, lm, update, stream)
        B.lomo_rmsnorm_backward(self.dxn_f, final["xhat"], final["rstd"], m["w_f"], None, self.grad_in(0), stream)
        _gain(st, 1, final["xhat"], self.dxn_f, m["w_f"], gain, update, stream)
        for k in range(L):
            li = L - 1 - k
            p = m["layers"][li]
            sa, sm = saved["layers"][li]
            if before_layer is not None:
                before_layer(li, k)          # e.g. recompute this layer's activations from its checkpoint
            dy, mid, dh = self.grad_in(k), self.grad_mid(k), self.grad_in(k + 1)
            self.mlp[k].walk(dy, sm, p["w2"], p["W_gu"], p["W_d"], mid, update, stream)
            self.attn[k].walk(mid, sa, p["w1"], p["W_qkv"], p["W_o"], rope_cos, rope_sin, dh, update, stream)
        slot = st.n - 1
        if update:
            B.lomo_step_update_pass_device(emb, st.scalars, st.step_flag, st.ws, stream)
        else:
            B.lomo_embedding_sqnorm(ids, dh0, m["W_emb"].shape[0], st.ws, st.acc, st.flags[slot:slot + 1], _fork(st, stream))

    def step(self, ids, dlogits, saved: Dict, m: Dict, rope_cos, rope_sin, lr: float, loss_scale: float,
             max_norm: float = 1.0, eps: float = 1e-6, stream=None, before_layer=None) -> None:
        """m: {"W_emb", "layers": [{"w1","W_qkv","W_o","w2","W_gu","W_d"}, ...], "w_f", "W_lm"}, updated in place.
        saved: {"layers": [(attention-block activations, feed-forward-block activations), ...], "final": {...}}.
        before_layer(layer index, walk index) is called before the walk enters a layer, in both passes."""
        assert before_layer is None or not self.keep_handons, "kept hand-ons need every layer's activations in pass 2"
        self.state.begin(stream)
        self._walk(ids, dlogits, saved, m, rope_cos, rope_sin, False, stream, before_layer)
        self.state.coefficient(lr, loss_scale, max_norm, eps, stream)
        if self.keep_handons:
            st = self.state
            B.lomo_step_update_pass_device(self._all_tensors(ids, dlogits, saved, m), st.scalars, st.step_flag, st.ws, stream)
        else:
            self._walk(ids, dlogits, saved, m, rope_cos, rope_sin, True, stream, before_layer)
        self.state.finish(stream)

    def _all_tensors(self, ids, dlogits, saved, m):
        """Every tensor of the model with the hand-on gradient pass 1 left for it (no input gradients asked for)."""
        L = self.n_layers
        final = saved["final"]
        key = tuple(t.data_ptr() for t in [ids, dlogits, final["xn"], m["W_lm"], m["W_emb"]] +
                    [p["W_d"] for p in m["layers"]] + [sm["a"] for _, sm in saved["layers"]])
        if self._all is None or self._all[0] != key:
            lin = lambda X, dY, W: {"kind": "linear", "X": X, "dY": dY, "W": W}
            vec = lambda X, dY, W: {"kind": "vector", "X": X, "dY": dY, "W": W}
            recs = [lin(final["xn"], dlogits, m["W_lm"]), vec(final["xhat"], self.dxn_f, m["w_f"])]
            for k in range(L):
                p = m["layers"][L - 1 - k]
                sa, sm = saved["layers"][L - 1 - k]
                mlp, attn = self.mlp[k], self.attn[k]
                recs += [lin(sm["a"], self.grad_in(k), p["W_d"]), lin(sm["xn"], mlp.dgu, p["W_gu"]),
                         vec(sm["xhat"], mlp.dxn, p["w2"]), lin(sa["o"], self.grad_mid(k), p["W_o"]),
                         lin(sa["xn"], attn.dqkv, p["W_qkv"]), vec(sa["xhat"], attn.dxn, p["w1"])]
            recs.append({"kind": "embedding", "ids": ids, "dY": self.grad_in(L), "W": m["W_emb"]})
            self._all = (key, B.make_tensor_list(recs))
        return self._all[1]

    def result(self) -> Dict:
        return self.state.result()


class _GroupState:
    """What the blocks need of a step state, for one parameter group: its own accumulator cell, tensor flags,
    step flag and scalars; the workspace is shared (stream order keeps the groups apart)."""

    def __init__(self, acc, flags, step_flag, chain_flags, ws, scalars):
        self.acc, self.flags, self.step_flag, self.ws, self.scalars = acc, flags, step_flag, ws, scalars
        self.chain_flags = chain_flags          # [previous group's step flag | this group's tensor flags]
        self.n = flags.numel()

    def coefficient(self, lr, loss_scale, max_norm, eps, stream):
        B.lomo_reduce_flags(self.chain_flags, self.step_flag, stream)
        B.lomo_step_scalars_device(self.acc, self.step_flag, loss_scale, max_norm, eps, lr, self.scalars, stream)


class LomoGroupedNormChain:
    """Single backward walk over the whole model with the grouped norm that section 3.3.1 closes with: the norm of a
    group of adjacent layers stands in for the norm of all parameters, so each group is updated as soon as the walk
    has left it and there is no second pass.  Groups in walk order: {W_lm, w_f}, runs of `layers_per_group` layers
    from the last to the first, {W_emb}.  Within a group the hand-on gradients are kept until its update (one set of
    buffers per layer of a group, reused by the next group): one dgrad, one norm GEMM and one fused-update GEMM per
    linear tensor, one attention / SwiGLU / RMSNorm backward.

    Overflow: a group's step flag is the OR of its tensors' flags and of the previous group's step flag, so a group
    with a non-finite gradient and every group after it keep their bits; groups above have been updated already."""

    def __init__(self, device, batch: int, seq: int, H: int, F: int, n_heads: int, n_layers: int, layers_per_group: int = 1):
        self.device = torch.device(device)
        T = batch * seq
        per = max(1, min(layers_per_group, n_layers))
        self.n_layers, self.per = n_layers, per
        self.bounds = [(k0, min(k0 + per, n_layers)) for k0 in range(0, n_layers, per)]
        sizes = [2] + [6 * (k1 - k0) for k0, k1 in self.bounds] + [1]
        G = len(sizes)
        self.acc = torch.zeros(G, dtype=torch.float64, device=self.device)
        # flag cells: a zero carry, then for every group its tensor flags followed by its step flag
        self.flags = torch.zeros(1 + sum(sizes) + G, dtype=torch.int32, device=self.device)
        self.scalars = torch.zeros(G * 32, dtype=torch.uint8, device=self.device)
        self._scalars_host = torch.zeros(G * 32, dtype=torch.uint8).pin_memory()
        nbytes = max(B.lomo_vector_workspace_bytes(T, H), B.lomo_embedding_workspace_bytes(T, H), 256)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.groups, self._flag_slices = [], []
        cell = 1
        for g, n in enumerate(sizes):
            self.groups.append(_GroupState(self.acc[g:g + 1], self.flags[cell:cell + n], self.flags[cell + n:cell + n + 1],
                                           self.flags[cell - 1:cell + n], self.ws, self.scalars[32 * g:32 * g + 32]))
            self._flag_slices.append((cell, n))
            cell += n + 1
        self.mlp, self.attn = [], []
        for k in range(n_layers):
            g, j = 1 + k // per, k % per
            share = j < len(self.mlp) and k >= per          # later groups reuse the first group's buffers
            self.mlp.append(LomoMlpBlock(self.device, T, H, F, self.groups[g], 6 * j, share=self.mlp[j] if share else None))
            self.attn.append(LomoAttentionBlock(self.device, batch, seq, H, n_heads, self.groups[g], 6 * j + 3,
                                                share=self.attn[j] if share else None))
        f16 = dict(dtype=torch.float16, device=self.device)
        self.dxn_f = torch.empty(T, H, **f16)
        self.dy = [torch.empty(T, H, **f16) for _ in range(per + 1)]
        self.dh_mid = [torch.empty(T, H, **f16) for _ in range(per)]
        self._lists = None

    def grad_in(self, k: int):
        return self.dy[k % len(self.dy)]

    def grad_mid(self, k: int):
        return self.dh_mid[k % len(self.dh_mid)]

    def _tensor_lists(self, ids, dlogits, saved, m):
        final = saved["final"]
        key = tuple(t.data_ptr() for t in [ids, dlogits, final["xn"], m["W_lm"], m["W_emb"]] +
                    [p["W_d"] for p in m["layers"]] + [sm["a"] for _, sm in saved["layers"]])
        if self._lists is None or self._lists[0] != key:
            L = self.n_layers
            lin = lambda X, dY, W: {"kind": "linear", "X": X, "dY": dY, "W": W}
            vec = lambda X, dY, W: {"kind": "vector", "X": X, "dY": dY, "W": W}
            lists = [B.make_tensor_list([lin(final["xn"], dlogits, m["W_lm"]), vec(final["xhat"], self.dxn_f, m["w_f"])])]
            for k0, k1 in self.bounds:
                recs = []
                for k in range(k0, k1):
                    p = m["layers"][L - 1 - k]
                    sa, sm = saved["layers"][L - 1 - k]
                    mlp, attn = self.mlp[k], self.attn[k]
                    recs += [lin(sm["a"], self.grad_in(k), p["W_d"]), lin(sm["xn"], mlp.dgu, p["W_gu"]),
                             vec(sm["xhat"], mlp.dxn, p["w2"]), lin(sa["o"], self.grad_mid(k), p["W_o"]),
                             lin(sa["xn"], attn.dqkv, p["W_qkv"]), vec(sa["xhat"], attn.dxn, p["w1"])]
                lists.append(B.make_tensor_list(recs))
            lists.append(B.make_tensor_list([{"kind": "embedding", "ids": ids, "dY": self.grad_in(L), "W": m["W_emb"]}]))
            self._lists = (key, lists)
        return self._lists[1]

    def step(self, ids, dlogits, saved: Dict, m: Dict, rope_cos, rope_sin, lr: float, loss_scale: float,
             max_norm: float = 1.0, eps: float = 1e-6, stream=None, before_layer=None) -> None:
        lists = self._tensor_lists(ids, dlogits, saved, m)
        with B.on_stream(stream):
            self.acc.zero_()
            self.flags.zero_()
        L = self.n_layers
        final = saved["final"]

        def close(g):
            st = self.groups[g]
            st.coefficient(lr, loss_scale, max_norm, eps, stream)
            B.lomo_step_update_pass_device(lists[g], st.scalars, st.step_flag, st.ws, stream)

        top = self.groups[0]
        _linear(top, 0, final["xn"], dlogits, m["W_lm"], self.dxn_f, None, False, stream)
        B.lomo_rmsnorm_backward(self.dxn_f, final["xhat"], final["rstd"], m["w_f"], None, self.grad_in(0), stream)
        _gain(top, 1, final["xhat"], self.dxn_f, m["w_f"], None, False, stream)
        close(0)
        for g, (k0, k1) in enumerate(self.bounds, start=1):
            for k in range(k0, k1):
                p = m["layers"][L - 1 - k]
                sa, sm = saved["layers"][L - 1 - k]
                if before_layer is not None:
                    before_layer(L - 1 - k, k)
                self.mlp[k].walk(self.grad_in(k), sm, p["w2"], p["W_gu"], p["W_d"], self.grad_mid(k), False, stream)
                self.attn[k].walk(self.grad_mid(k), sa, p["w1"], p["W_qkv"], p["W_o"], rope_cos, rope_sin,
                                  self.grad_in(k + 1), False, stream)
            close(g)
        last = self.groups[-1]
        B.lomo_embedding_sqnorm(ids, self.grad_in(L), m["W_emb"].shape[0], last.ws, last.acc, last.flags[0:1], stream)
        close(len(self.groups) - 1)
        if stream is None:
            self._scalars_host.copy_(self.scalars, non_blocking=True)
        else:
            with torch.cuda.stream(stream):
                self._scalars_host.copy_(self.scalars, non_blocking=True)

    def result(self) -> Dict:
        """Per-group scalars and the tensors' flags in walk order (synchronise first)."""
        per = [B.unpack_step_scalars(self._scalars_host[32 * g:32 * g + 32]) for g in range(len(self.groups))]
        host = self.flags.cpu().tolist()
        flags = [bool(v) for cell, n in self._flag_slices for v in host[cell:cell + n]]
        stops = [bool(host[cell + n]) for cell, n in self._flag_slices]
        return {"group_norms": [r["norm"] for r in per], "group_coefs": [r["clip_coef"] for r in per],
                "group_overflow": stops, "overflow": stops[-1], "flags": flags}


# --------------------------------------------------------------------------- forward, checkpoints, recomputation


class LayerActivations:
    """The activations of one decoder layer that the backward loop reads: attention block {xhat, rstd, xn, qkv
    (rotated q | rotated k | v), o, lse}, feed-forward block {xhat, rstd, xn, gate_up, a}, and y1, the attention
    block's output (the feed-forward block's input)."""

    def __init__(self, device, T: int, H: int, F: int, n_heads: int):
        f16 = dict(dtype=torch.float16, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.attn = {"xhat": torch.empty(T, H, **f16), "rstd": torch.empty(T, **f32), "xn": torch.empty(T, H, **f16),
                     "qkv": torch.empty(T, 3 * H, **f16), "o": torch.empty(T, H, **f16), "lse": torch.empty(T, n_heads, **f32)}
        self.mlp = {"xhat": torch.empty(T, H, **f16), "rstd": torch.empty(T, **f32), "xn": torch.empty(T, H, **f16),
                    "gate_up": torch.empty(T, 2 * F, **f16), "a": torch.empty(T, F, **f16)}
        self.y1 = torch.empty(T, H, **f16)


def layer_forward(h, p: Dict, act: LayerActivations, rope_cos, rope_sin, batch: int, seq: int, n_heads: int, eps: float,
                  h_next=None, stream=None) -> None:
    """Forward of one decoder layer from its input h into `act`; with h_next also the layer output
    h_next = y1 + a W_d^T (a recomputation before the backward walk does not need it)."""
    sa, sm = act.attn, act.mlp
    B.lomo_rmsnorm_forward(h, p["w1"], eps, sa["xhat"], sa["rstd"], sa["xn"], stream)
    B.lomo_linear_forward(sa["xn"], p["W_qkv"], sa["qkv"], False, stream)
    B.lomo_rope_forward(sa["qkv"], rope_cos, rope_sin, seq, n_heads, stream)
    B.lomo_attention_forward(sa["qkv"], sa["o"], sa["lse"], batch, seq, n_heads, stream)
    B.lomo_linear_forward_residual(sa["o"], p["W_o"], h, act.y1, stream)           # y1 = h + o W_o^T, one rounding
    B.lomo_rmsnorm_forward(act.y1, p["w2"], eps, sm["xhat"], sm["rstd"], sm["xn"], stream)
    B.lomo_linear_forward(sm["xn"], p["W_gu"], sm["gate_up"], False, stream)
    B.lomo_swiglu_forward(sm["gate_up"], sm["a"], stream)
    if h_next is not None:
        B.lomo_linear_forward_residual(sm["a"], p["W_d"], act.y1, h_next, stream)


class LomoFineTuneStep:
    """One whole LOMO training step of a decoder-only model from token ids: forward pass keeping only each layer's
    input (activation checkpointing), token-level cross-entropy with the loss scale folded into its gradient, then
    Algorithm 1's backward loop with each layer's activations recomputed from its checkpoint just before the walk
    enters it.  norm="global": two passes (the norm of all parameters), so every layer is recomputed twice;
    norm="grouped": one walk with per-group norms, one recomputation.  Activation memory: (n_layers + 1) [T x H]
    checkpoints, one layer's activations (per layer of a group), the logits.

    Two switches trade memory for arithmetic where the memory is there (at 7B and 4096 tokens each costs 17 GB):
    checkpoint=False keeps every layer's activations from the forward pass, so nothing is recomputed;
    keep_handons=True (global norm, needs checkpoint=False) also keeps pass 1's hand-on gradients, so pass 2 is
    one grouped fused-update launch over the whole model.  Neither changes a bit of the result.
    overlap_norm_pass=True (with keep_handons) runs pass 1's norm contractions on a second stream beside the walk."""

    def __init__(self, device, batch: int, seq: int, H: int, F: int, n_heads: int, n_layers: int, V: int,
                 eps: float = 1e-5, norm: str = "global", layers_per_group: int = 1, checkpoint: bool = True,
                 keep_handons: bool = False, overlap_norm_pass: bool = False):
        assert norm in ("global", "grouped")
        assert not keep_handons or (norm == "global" and not checkpoint), "kept hand-ons: global norm, no checkpointing"
        self.device = torch.device(device)
        T = batch * seq
        self.batch, self.seq, self.n_heads, self.n_layers, self.eps = batch, seq, n_heads, n_layers, eps
        self.checkpoint = checkpoint
        f16 = dict(dtype=torch.float16, device=self.device)
        self.ckpt = [torch.empty(T, H, **f16) for _ in range(n_layers + 1)]
        per = layers_per_group if norm == "grouped" else 1
        n_sets = max(1, min(per, n_layers)) if checkpoint else n_layers
        self.acts = [LayerActivations(self.device, T, H, F, n_heads) for _ in range(n_sets)]
        self.final = {"xhat": torch.empty(T, H, **f16), "rstd": torch.empty(T, dtype=torch.float32, device=self.device),
                      "xn": torch.empty(T, H, **f16)}
        self.logits = torch.empty(T, V, **f16)           # overwritten by its own gradient
        self.token_loss = torch.empty(T, dtype=torch.float32, device=self.device)
        self.loss_stats = torch.zeros(3, dtype=torch.float64, device=self.device)     # mean loss, counted targets, scratch
        if norm == "grouped":
            self.chain = LomoGroupedNormChain(self.device, batch, seq, H, F, n_heads, n_layers, layers_per_group=per)
        else:
            self.chain = LomoModelChain(self.device, batch, seq, H, F, n_heads, n_layers, keep_handons=keep_handons,
                                        overlap_norm_pass=overlap_norm_pass)
        # walk index k = n_layers - 1 - layer index; the layers of one group use different activation sets
        self.saved = {"layers": [(self._act(li).attn, self._act(li).mlp) for li in range(n_layers)], "final": self.final}

    def _act(self, li: int) -> LayerActivations:
        return self.acts[(self.n_layers - 1 - li) % len(self.acts)]

    def forward(self, ids, targets, loss_scale: float, m: Dict, rope_cos, rope_sin, stream=None) -> None:
        """Checkpoints, final norm, logits, token losses, and the scaled loss gradient in place of the logits."""
        B.lomo_embedding_forward(ids, m["W_emb"], self.ckpt[0], stream)
        for li, p in enumerate(m["layers"]):
            layer_forward(self.ckpt[li], p, self._act(li), rope_cos, rope_sin, self.batch, self.seq, self.n_heads, self.eps,
                          self.ckpt[li + 1], stream)
        f = self.final
        B.lomo_rmsnorm_forward(self.ckpt[self.n_layers], m["w_f"], self.eps, f["xhat"], f["rstd"], f["xn"], stream)
        B.lomo_linear_forward(f["xn"], m["W_lm"], self.logits, False, stream)
        B.lomo_cross_entropy_mean(self.logits, targets, loss_scale, self.token_loss, self.logits, self.loss_stats, stream)

    def step(self, ids, targets, m: Dict, rope_cos, rope_sin, lr: float, loss_scale: float,
             max_norm: float = 1.0, eps_clip: float = 1e-6, stream=None) -> None:
        """m as for LomoModelChain, updated in place.  targets [T] int32 (outside [0, V): not counted); the mean loss's
        denominator, the number of counted targets, is taken on the device."""
        self.forward(ids, targets, loss_scale, m, rope_cos, rope_sin, stream)
        fresh = [self.n_layers - 1]          # the forward pass has just left the last layer's activations in place

        def recompute(li, k):
            if fresh and fresh[0] == li:
                fresh.clear()
                return
            layer_forward(self.ckpt[li], m["layers"][li], self._act(li), rope_cos, rope_sin, self.batch, self.seq,
                          self.n_heads, self.eps, None, stream)

        self.chain.step(ids, self.logits, self.saved, m, rope_cos, rope_sin, lr, loss_scale, max_norm, eps_clip, stream,
                        before_layer=recompute if self.checkpoint else None)

    def result(self) -> Dict:
        """The chain's scalars and flags plus the mean loss over the counted tokens (synchronise first)."""
        out = self.chain.result()
        out["loss"] = float(self.loss_stats[0].item())
        return out


class LomoTrainer:
    """Training steps with the dynamic loss scaler of section 3.3.2 around them: a step that overflowed was dropped
    on the device (no parameter touched, or from the overflowing group on with the grouped norm) and halves the
    scale; `growth_interval` clean steps in a row double it.  One host synchronisation per step, to read the
    step's flag before the next step's scale is known."""

    def __init__(self, step: LomoFineTuneStep, lr: float, loss_scale: float = 65536.0, growth_interval: int = 1000,
                 max_norm: float = 1.0, eps_clip: float = 1e-6):
        self.step, self.lr, self.loss_scale, self.growth_interval = step, lr, float(loss_scale), growth_interval
        self.max_norm, self.eps_clip, self.clean_steps = max_norm, eps_clip, 0

    def train_step(self, ids, targets, m: Dict, rope_cos, rope_sin, stream=None) -> Dict:
        used = self.loss_scale
        self.step.step(ids, targets, m, rope_cos, rope_sin, self.lr, used, self.max_norm, self.eps_clip, stream)
        if stream is None:
            torch.cuda.synchronize(self.step.device)
        else:
            stream.synchronize()
        res = self.step.result()
        res["loss_scale"] = used
        self.loss_scale, self.clean_steps = B.lomo_scaler_step(used, self.clean_steps, self.growth_interval, res["overflow"])
        return res
