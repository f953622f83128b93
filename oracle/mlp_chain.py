"""CPU oracle for LOMO's backward loop through one LLaMA feed-forward block -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file; the HIP path
never does, and this file imports nothing from it (it builds on oracle/lomo_oracle.py only).

What it computes.  Algorithm 1 of the paper walks the layers from the last to the first; at each
parameter it forms the gradient, applies p <- p - lr * g at once and drops the gradient, while the
gradient with respect to the layer's input is handed on to the layer below (section 3.2).  Here that
loop is written out for the feed-forward half of a decoder layer of the models the paper fine-tunes
(LLaMA, section 4): RMSNorm with gain w, fused gate/up projection W_gu [2F x H], SwiGLU, down projection
W_d [H x F], residual connection:

    r_t   = 1 / sqrt(mean_j h[t,j]^2 + eps)          xhat = h * r          xn = xhat * w
    [gate | up] = xn W_gu^T                           a = silu(gate) * up,  silu(g) = g / (1 + exp(-g))
    y = h + a W_d^T

Backward, given dy = dL/dy (carrying the loss scale):
    da     = dy W_d                       G_d  = dy^T a
    dup    = da * silu(gate)              dgate = da * up * s (1 + gate (1 - s)),  s = 1 / (1 + exp(-gate))
    dxn    = [dgate | dup] W_gu           G_gu = [dgate | dup]^T xn
    g_w[j] = sum_t dxn[t,j] xhat[t,j]
    dh     = dy + r * (dxn * w - xhat * mean_j(dxn * w * xhat))

The two-pass step of section 3.3 runs this chain twice: pass 1 only accumulates the squared norms of
G_d, G_gu, g_w (and the overflow flag), pass 2 repeats it and updates every parameter right after the
gradient of its input has been taken from the old value.  All arithmetic is fp64; tensors that the
mixed-precision run keeps in fp16 (da, [dgate|dup], dxn, dh, the parameters) are rounded once where they
are stored, so the chain sees exactly the stored values (section 3.3.2: fp16 storage, full-precision
computation).

Pins (tests/test_oracle_pins.py): central finite differences of a scalar loss through the forward block
for every gradient above; dh - dy orthogonal to h for eps = 0 (RMSNorm ignores the scale of its input);
silu'(0) = 1/2 and the large-|g| limits; hand-computed 1 x 2 example; fused order == materialised order.
"""
from __future__ import annotations

import math
from typing import Dict

import numpy as np

from . import lomo_oracle as O


# --------------------------------------------------------------------------- forward (input preparation)


def sigmoid(g: np.ndarray) -> np.ndarray:
    g = np.asarray(g, dtype=np.float64)
    with np.errstate(over="ignore"):
        return 1.0 / (1.0 + np.exp(-g))


def silu(g: np.ndarray) -> np.ndarray:
    return np.asarray(g, dtype=np.float64) * sigmoid(g)


def rmsnorm_forward(h, w, eps: float):
    """(xhat, r, xn) in fp64: xhat = h * r with r = 1 / sqrt(mean(h^2) + eps) per row, xn = xhat * w."""
    h64 = O.as_f64(h)
    r = 1.0 / np.sqrt((h64 * h64).mean(axis=1) + eps)
    xhat = h64 * r[:, None]
    return xhat, r, xhat * O.as_f64(w)[None, :]


def block_forward_f64(h, w, W_gu, W_d, eps: float) -> np.ndarray:
    """y of the block in plain fp64, no storage rounding (used by the finite-difference pin)."""
    F = W_d.shape[1]
    _, _, xn = rmsnorm_forward(h, w, eps)
    gu = xn @ O.as_f64(W_gu).T
    a = silu(gu[:, :F]) * gu[:, F:]
    return O.as_f64(h) + a @ O.as_f64(W_d).T


def block_forward_stored(h, w, W_gu, W_d, eps: float) -> Dict:
    """Forward with every saved activation rounded to its storage type (fp16; r in fp32)."""
    F = W_d.shape[1]
    xhat64, r64, _ = rmsnorm_forward(h, w, eps)
    xhat = O.round_f16(xhat64)
    xn = O.round_f16(O.as_f64(xhat) * O.as_f64(w)[None, :])
    gu = O.round_f16(O.as_f64(xn) @ O.as_f64(W_gu).T)
    a = O.round_f16(silu(O.as_f64(gu[:, :F])) * O.as_f64(gu[:, F:]))
    return {"xhat": xhat, "r": r64.astype(np.float32), "xn": xn, "gate_up": gu, "a": a}


# --------------------------------------------------------------------------- backward pieces


def swiglu_backward(da, gate_up) -> np.ndarray:
    """[dgate | dup] in fp64 from da [T x F] and the saved [gate | up] [T x 2F]."""
    F = da.shape[1]
    d = O.as_f64(da)
    g, u = O.as_f64(gate_up[:, :F]), O.as_f64(gate_up[:, F:])
    s = sigmoid(g)
    with np.errstate(invalid="ignore", over="ignore"):
        dgate = d * u * (s * (1.0 + g * (1.0 - s)))
        dup = d * (g * s)
    return np.concatenate((dgate, dup), axis=1)


def rmsnorm_backward(dxn, xhat, r, w, dres=None) -> np.ndarray:
    """dh in fp64: r * (dxn * w - xhat * mean_j(dxn * w * xhat)) (+ the residual branch's gradient)."""
    dxh = O.as_f64(dxn) * O.as_f64(w)[None, :]
    xh = O.as_f64(xhat)
    with np.errstate(invalid="ignore", over="ignore"):
        c = (dxh * xh).mean(axis=1)
        dh = np.asarray(r, dtype=np.float64)[:, None] * (dxh - xh * c[:, None])
        if dres is not None:
            dh = dh + O.as_f64(dres)
    return dh


# --------------------------------------------------------------------------- the chain


def chain_gradients(dy, saved: Dict, w, W_gu, W_d) -> Dict:
    """One walk down the block with the current parameters: stored fp16 hand-ons and fp64 gradients."""
    da = O.input_grad(dy, W_d)                                   # fp16, from W_d before any update
    G_d = O.linear_grad(saved["a"], dy)
    dgu = O.round_f16(swiglu_backward(da, saved["gate_up"]))
    dxn = O.input_grad(dgu, W_gu)
    G_gu = O.linear_grad(saved["xn"], dgu)
    g_w = O.vector_grad(saved["xhat"], dxn)
    dh = O.round_f16(rmsnorm_backward(dxn, saved["xhat"], saved["r"], w, dres=dy))
    return {"da": da, "dgu": dgu, "dxn": dxn, "dh": dh, "G_d": G_d, "G_gu": G_gu, "g_w": g_w}


def block_step(dy, saved: Dict, w, W_gu, W_d, lr: float, loss_scale: float, max_norm: float = 1.0,
               eps_clip: float = 1e-6) -> Dict:
    """Two-pass LOMO step over the block (sections 3.2 and 3.3), parameters in backward order W_d, W_gu, w.

    Pass 1 walks the chain and keeps only the squared norms and flags; pass 2 walks it again from the same
    (old) parameters, so the hand-on gradients are identical, and updates each parameter after its input
    gradient has been taken.  Because no hand-on gradient depends on an updated parameter, the result equals
    the materialised step, which is what is computed here.
    """
    c = chain_gradients(dy, saved, w, W_gu, W_d)
    grads = [c["G_d"], c["G_gu"], c["g_w"]]
    flags = [O.has_overflow(g) for g in grads]
    sq = [O.sqnorm(g) for g in grads]
    overflow = any(flags)
    total = math.fsum(sq) if not overflow else float("nan")
    norm = O.grad_norm(total, loss_scale) if not overflow else float("nan")
    coef = O.clip_coef(norm, max_norm, eps_clip) if not overflow else float("nan")
    params = [W_d, W_gu, w]
    new = [np.array(p, copy=True) if overflow else O.sgd_update(p, g, lr, coef, loss_scale)
           for p, g in zip(params, grads)]
    return {"W_d": new[0], "W_gu": new[1], "w": new[2], "dh": c["dh"], "da": c["da"], "dgu": c["dgu"],
            "dxn": c["dxn"], "flags": flags, "sqnorms": sq, "overflow": overflow, "total_sqnorm": total,
            "norm": norm, "clip_coef": coef}


def block_step_fused_order(dy, saved: Dict, w, W_gu, W_d, lr: float, loss_scale: float, max_norm: float = 1.0,
                           eps_clip: float = 1e-6) -> Dict:
    """The same step in Algorithm 1's order: in pass 2 each parameter is overwritten before the walk goes on."""
    first = chain_gradients(dy, saved, w, W_gu, W_d)
    grads = [first["G_d"], first["G_gu"], first["g_w"]]
    flags = [O.has_overflow(g) for g in grads]
    overflow = any(flags)
    total = math.fsum(O.sqnorm(g) for g in grads) if not overflow else float("nan")
    norm = O.grad_norm(total, loss_scale) if not overflow else float("nan")
    coef = O.clip_coef(norm, max_norm, eps_clip) if not overflow else float("nan")
    W_d2, W_gu2, w2 = (np.array(p, copy=True) for p in (W_d, W_gu, w))
    da = O.input_grad(dy, W_d2)
    if not overflow:
        W_d2 = O.sgd_update(W_d2, O.linear_grad(saved["a"], dy), lr, coef, loss_scale)
    dgu = O.round_f16(swiglu_backward(da, saved["gate_up"]))
    dxn = O.input_grad(dgu, W_gu2)
    if not overflow:
        W_gu2 = O.sgd_update(W_gu2, O.linear_grad(saved["xn"], dgu), lr, coef, loss_scale)
    g_w = O.vector_grad(saved["xhat"], dxn)
    dh = O.round_f16(rmsnorm_backward(dxn, saved["xhat"], saved["r"], w2, dres=dy))   # gain before its update
    if not overflow:
        w2 = O.sgd_update(w2, g_w, lr, coef, loss_scale)
    return {"W_d": W_d2, "W_gu": W_gu2, "w": w2, "dh": dh, "overflow": overflow, "norm": norm, "clip_coef": coef}
