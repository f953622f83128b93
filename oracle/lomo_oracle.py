"""CPU oracle for one LOMO step -- TEST INFRASTRUCTURE, not part of the product.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
file; the HIP path never does, and this file imports nothing from it.

What it computes.  LOMO (paper section 3.2, Algorithm 1) applies p <- p - lr * dL/dp
to each parameter as soon as its gradient exists during back-propagation and then
discards the gradient.  The introduction states that this update is still equivalent
to SGD, so the oracle is the plain definition written the memory-hungry way:
materialise every gradient in fp64, take the global gradient norm over all parameters
(section 3.3.1, the additional backward pass), clip, undo the loss scale (section
3.3.2), apply SGD, and round the result once to fp16.  Section 3.3.2 says gradient and
parameter are converted to full precision inside these computations; fp64 here.

Conventions (readings of points the paper leaves open):
  * linear tensor: W [N x K] row-major, forward Y = X W^T, X [T x K], dY [T x N];
    scaled gradient G = dY^T X, input gradient dX = dY W (pre-update W).
  * embedding: G[v, :] = sum of dY[t, :] over positions t with ids[t] == v.
  * RMSNorm gain: g[j] = sum_t dY[t, j] * xhat[t, j].
  * dY carries the loss scale S; the true gradient is G / S.
  * "overflow" = any non-finite value in any scaled gradient of the step; then no tensor
    is updated and S is halved (section 3.3.2, dynamic loss scaler).
  * clipping: coef = min(1, max_norm / (norm + eps)), norm = sqrt(sum G^2) / S
    (appendix A: max grad norm 1.0).
  * update: W' = round_to_fp16( W - lr * coef * G / S ), one rounding, fp64 -> fp16 direct.

Pins (tests/test_oracle_pins.py): finite differences through a tiny two-layer model,
hand-computed small examples stored under tests/golden/, LOMO-order == batch-order,
brute-force / closed-form / Gram-identity norms, one-hot and diagonal reductions of the
embedding and gain gradients to the linear one, exact-rational rounding checks, the
printed clip-by-value example.  No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence

import numpy as np

# --------------------------------------------------------------------------- widening


def as_f64(a) -> np.ndarray:
    """Exact widening of fp16 inputs (subnormals, infinities, NaN preserved)."""
    a = np.asarray(a)
    if a.dtype == np.float16:
        return a.astype(np.float64)
    if a.dtype == np.float64:
        return a
    raise TypeError(f"oracle inputs are fp16 (or already-widened fp64), got {a.dtype}")


def round_f16(a64: np.ndarray) -> np.ndarray:
    """fp64 -> fp16, round-to-nearest-even, directly (no intermediate fp32 rounding)."""
    with np.errstate(over="ignore"):
        return np.asarray(a64, dtype=np.float64).astype(np.float16)


# --------------------------------------------------------------------------- gradients


def linear_grad(X, dY) -> np.ndarray:
    """Scaled weight gradient of Y = X W^T in W's layout: G[n, k] = sum_t dY[t, n] X[t, k].

    Algorithm 1, the line g_l <- dl/dtheta_l, for a linear layer.
    """
    with np.errstate(invalid="ignore", over="ignore"):
        return as_f64(dY).T @ as_f64(X)


def input_grad_f64(dY, W) -> np.ndarray:
    """dX[t, k] = sum_n dY[t, n] W[n, k] -- what back-propagation hands to layer l-1."""
    with np.errstate(invalid="ignore", over="ignore"):
        return as_f64(dY) @ as_f64(W)


def input_grad(dY, W) -> np.ndarray:
    """dX rounded once to fp16 (activations and their gradients are stored in fp16)."""
    return round_f16(input_grad_f64(dY, W))


def embedding_grad(ids, dY, V: int) -> np.ndarray:
    """G[v, :] = sum over positions t with ids[t] == v of dY[t, :]; zero rows for absent ids."""
    ids = np.asarray(ids)
    d = as_f64(dY)
    G = np.zeros((V, d.shape[1]), dtype=np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        for t in range(ids.shape[0]):
            G[int(ids[t])] += d[t]
    return G


def vector_grad(xhat, dY) -> np.ndarray:
    """Gradient of an RMSNorm gain w in y = xhat * w: g[j] = sum_t dY[t, j] * xhat[t, j]."""
    with np.errstate(invalid="ignore", over="ignore"):
        return (as_f64(dY) * as_f64(xhat)).sum(axis=0)


def embedding_grouping(ids):
    """Stable grouping of positions by token id.

    Returns (unique_ids ascending, seg_offsets [n_unique + 1], perm) where perm lists the
    positions sorted by (id, position) and segment u is perm[seg_offsets[u]:seg_offsets[u+1]].
    """
    ids = np.asarray(ids, dtype=np.int64)
    perm = np.argsort(ids, kind="stable")
    s = ids[perm]
    if s.size == 0:
        return (np.zeros(0, np.int32), np.zeros(1, np.int32), np.zeros(0, np.int32))
    heads = np.flatnonzero(np.concatenate(([True], s[1:] != s[:-1])))
    seg_offsets = np.concatenate((heads, [s.size]))
    return s[heads].astype(np.int32), seg_offsets.astype(np.int32), perm.astype(np.int32)


# --------------------------------------------------------------------------- norm, clip, scaler


def has_overflow(G) -> bool:
    """True iff the scaled gradient holds an inf or NaN (first backward pass of section 3.3.2)."""
    return not bool(np.all(np.isfinite(G)))


def sqnorm(G) -> float:
    """Sum of squares of one scaled gradient, fp64."""
    with np.errstate(invalid="ignore", over="ignore"):
        g = np.asarray(G, dtype=np.float64).ravel()
        return float(np.dot(g, g))


def grad_norm(total_sqnorm_scaled: float, loss_scale: float) -> float:
    """Global L2 norm of the true (unscaled) gradient over all parameters of the step."""
    return math.sqrt(total_sqnorm_scaled) / loss_scale


def clip_coef(norm: float, max_norm: float = 1.0, eps: float = 1e-6) -> float:
    """Global-norm clipping coefficient: gradients are scaled down, never up."""
    return min(1.0, max_norm / (norm + eps))


def scaler_step(loss_scale: float, clean_steps: int, growth_interval: int, overflow: bool,
                min_scale: float = 1.0, max_scale: float = 2.0 ** 24):
    """Dynamic loss scaler of section 3.3.2.

    Overflow: the step is dropped and the scale halved.  Otherwise, after
    ``growth_interval`` consecutive clean backward passes the scale is doubled.
    """
    if overflow:
        return max(min_scale, loss_scale / 2.0), 0
    clean_steps += 1
    if clean_steps >= growth_interval:
        return min(max_scale, loss_scale * 2.0), 0
    return loss_scale, clean_steps


# --------------------------------------------------------------------------- update


def sgd_update(W, G, lr: float, coef: float, loss_scale: float) -> np.ndarray:
    """theta <- theta - lr * g with g = coef * G / S, in fp64, rounded once to fp16."""
    with np.errstate(invalid="ignore", over="ignore"):
        return round_f16(as_f64(W) - (lr * coef) * (np.asarray(G, dtype=np.float64) / loss_scale))


def sgd_update_clip_value(W, G, lr: float, clip_value: float, loss_scale: float) -> np.ndarray:
    """Single-pass alternative of section 3.3.1: clamp each gradient element to +-clip_value.

    The paper does not say what a single pass does on overflow; reading taken here: an element whose
    gradient is inf/NaN keeps its weight (the caller learns of it through has_overflow).
    """
    with np.errstate(invalid="ignore", over="ignore"):
        g = np.asarray(G, dtype=np.float64) / loss_scale
        fin = np.isfinite(g)
        stepped = round_f16(as_f64(W) - lr * np.clip(np.where(fin, g, 0.0), -clip_value, clip_value))
    return np.where(fin, stepped, np.asarray(W, dtype=np.float16))


# --------------------------------------------------------------------------- whole steps


def tensor_grad(t: Dict) -> np.ndarray:
    """Scaled fp64 gradient of one tensor record in the layout of its parameter."""
    kind = t["kind"]
    if kind == "linear":
        return linear_grad(t["X"], t["dY"])
    if kind == "embedding":
        return embedding_grad(t["ids"], t["dY"], t["W"].shape[0])
    if kind == "vector":
        return vector_grad(t["X"], t["dY"])
    raise ValueError(kind)


def step_materialised(tensors: Sequence[Dict], lr: float, loss_scale: float,
                      max_norm: float = 1.0, eps: float = 1e-6) -> Dict:
    """Ordinary SGD with global-norm clipping and loss scaling: all gradients held at once.

    ``tensors`` is a list of records {kind, W, dY, X (linear: activations, vector: xhat),
    ids (embedding)} in backward order.  Returns per-tensor new weights, dX (linear only),
    flags and squared norms plus the step scalars.
    """
    grads = [tensor_grad(t) for t in tensors]
    flags = [has_overflow(g) for g in grads]
    sq = [sqnorm(g) for g in grads]
    overflow = any(flags)
    total = math.fsum(sq) if not overflow else float("nan")
    norm = grad_norm(total, loss_scale) if not overflow else float("nan")
    coef = clip_coef(norm, max_norm, eps) if not overflow else float("nan")
    new_W, dX = [], []
    for t, g in zip(tensors, grads):
        dX.append(input_grad(t["dY"], t["W"]) if t["kind"] == "linear" else None)
        new_W.append(np.array(t["W"], copy=True) if overflow else sgd_update(t["W"], g, lr, coef, loss_scale))
    return {"W": new_W, "dX": dX, "flags": flags, "sqnorms": sq, "overflow": overflow,
            "total_sqnorm": total, "norm": norm, "clip_coef": coef}


def step_fused_order(tensors: Sequence[Dict], lr: float, loss_scale: float,
                     max_norm: float = 1.0, eps: float = 1e-6) -> Dict:
    """The same step in LOMO's order (Algorithm 1 with the two passes of section 3.3).

    Pass 1 walks the tensors in backward order keeping one gradient alive at a time and
    accumulates the squared norm and the overflow flag.  Pass 2 walks them again: dX from the
    pre-update weights, then the gradient is formed, applied and dropped before the next tensor.
    """
    sq, flags = [], []
    for t in tensors:
        g = tensor_grad(t)
        flags.append(has_overflow(g))
        sq.append(sqnorm(g))
        del g
    overflow = any(flags)
    total = math.fsum(sq) if not overflow else float("nan")
    norm = grad_norm(total, loss_scale) if not overflow else float("nan")
    coef = clip_coef(norm, max_norm, eps) if not overflow else float("nan")
    weights = [np.array(t["W"], copy=True) for t in tensors]
    dX: List = []
    for i, t in enumerate(tensors):
        dX.append(input_grad(t["dY"], weights[i]) if t["kind"] == "linear" else None)
        if not overflow:
            g = tensor_grad(t)
            weights[i] = sgd_update(weights[i], g, lr, coef, loss_scale)
            del g
    return {"W": weights, "dX": dX, "flags": flags, "sqnorms": sq, "overflow": overflow,
            "total_sqnorm": total, "norm": norm, "clip_coef": coef}


# --------------------------------------------------------------------------- sampled rows


def linear_grad_rows(X, dY_cols) -> np.ndarray:
    """Rows of G for a subset of output features: dY_cols is dY[:, rows] ([T x R]) -> [R x K]."""
    return linear_grad(X, dY_cols)


def ulp_distance_f16(a, b) -> np.ndarray:
    """Distance in units of fp16 spacing: bits mapped to a monotone integer line, +-0 equal."""
    def key(x):
        u = np.asarray(x, dtype=np.float16).view(np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a) - key(b))
