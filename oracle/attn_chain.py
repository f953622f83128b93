"""CPU oracle for the attention half of LOMO's backward loop through a decoder layer -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file; the HIP path
never does, and this file imports nothing from it (it builds on oracle/lomo_oracle.py and oracle/mlp_chain.py).

What it computes.  Algorithm 1 of the paper walks the layers backwards, updating each parameter as soon as
its gradient exists and handing the gradient of the layer input down (section 3.2).  Here the walk goes
through the self-attention block of the models the paper fine-tunes (LLaMA, section 4): RMSNorm with gain
w, fused projection W_qkv [3H x H], rotary position embedding on q and k, causal softmax attention over
n_heads heads of width d, output projection W_o [H x H], residual connection.  Tokens are laid out
t = b * s + pos (B sequences of length s); head n owns columns [n d, (n + 1) d) of q, k, v and o.

    xhat = h * r,  xn = xhat * w,  [q | k | v] = xn W_qkv^T
    rotary: for c < d/2 and angle a = pos * theta_c:  q'_c = q_c cos a - q_{c+d/2} sin a,
                                                      q'_{c+d/2} = q_{c+d/2} cos a + q_c sin a   (same for k)
    S_ij = (q'_i . k'_j) / sqrt(d) for j <= i (same sequence),  P = softmax_j(S),  o_i = sum_j P_ij v_j
    y = h + o W_o^T

Backward, given dy (carrying the loss scale), with lse_i = log sum_j exp(S_ij) saved by the forward pass:
    do = dy W_o                               G_o = dy^T o
    P_ij = exp(S_ij - lse_i),  dP_ij = do_i . v_j,  delta_i = do_i . o_i
    dS = P * (dP - delta) / sqrt(d)           dv_j = sum_i P_ij do_i
    dq'_i = sum_j dS_ij k'_j                  dk'_j = sum_i dS_ij q'_i
    rotary backward = rotation by -a:  dq_c = dq'_c cos a + dq'_{c+d/2} sin a,  dq_{c+d/2} = dq'_{c+d/2} cos a - dq'_c sin a
    dxn = [dq | dk | dv] W_qkv                G_qkv = [dq | dk | dv]^T xn
    g_w = sum_t dxn * xhat                    dh = dy + rmsnorm_backward(dxn)

Precision (section 3.3.2: fp16 storage, full-precision computation): every tensor the mixed-precision run
keeps in fp16 is rounded once where it is stored -- do, [dq|dk|dv] (after the rotary step), dxn, dh, and
also the attention probabilities P and their gradients dS, which fp16 training holds as fp16 tensors before
they enter the next matrix product.  dS is formed from the unrounded P.  The cos / sin table and lse are
fp32 inputs.  All arithmetic in between is fp64.

Pins (tests/test_oracle_pins.py): central finite differences of a scalar loss through the forward block for
dq, dk, dv (before the rotary step) and through the whole block for G_o, G_qkv, g_w, dh; softmax rows sum
to one and delta equals sum_j P dP; causality (the last key receives gradient from the last query only);
the rotary step is a rotation (norm preserving, backward = inverse); a hand-worked two-token example.
"""
from __future__ import annotations

import math
from typing import Dict

import numpy as np

from . import lomo_oracle as O
from . import mlp_chain as M


# --------------------------------------------------------------------------- rotary embedding


def rope_tables(s: int, d: int, base: float = 10000.0):
    """cos, sin [s x d/2] in fp32: angle(pos, c) = pos * base^(-2c/d).  The stored table is the input."""
    c = np.arange(d // 2, dtype=np.float64)
    ang = np.arange(s, dtype=np.float64)[:, None] * base ** (-2.0 * c / d)[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def _heads(x, n_heads: int):
    T, H = x.shape
    return x.reshape(T, n_heads, H // n_heads)


def rope_rotate(x, cos, sin, s: int, n_heads: int, inverse: bool = False) -> np.ndarray:
    """Rotary step on x [T x H] (fp64 out).  inverse=True rotates by the negative angle (the backward step)."""
    x64 = _heads(O.as_f64(x) if x.dtype == np.float16 else np.asarray(x, dtype=np.float64), n_heads)
    T, _, d = x64.shape
    pos = np.arange(T) % s
    co = np.asarray(cos, dtype=np.float64)[pos][:, None, :]
    si = np.asarray(sin, dtype=np.float64)[pos][:, None, :]
    if inverse:
        si = -si
    x1, x2 = x64[..., : d // 2], x64[..., d // 2:]
    out = np.concatenate((x1 * co - x2 * si, x2 * co + x1 * si), axis=-1)
    return out.reshape(T, -1)


# --------------------------------------------------------------------------- attention


def _scores(qh, kh, d):
    """Causal scaled scores of one sequence and head: [s x s] with -inf above the diagonal."""
    S = (qh @ kh.T) / math.sqrt(d)
    s = S.shape[0]
    S[np.triu_indices(s, 1)] = -np.inf
    return S


def attention_forward_f64(q, k, v, s: int, n_heads: int):
    """o [T x H] and lse [T x n_heads] in plain fp64 (q, k already rotated)."""
    T, H = q.shape
    d = H // n_heads
    qh, kh, vh = (_heads(np.asarray(a, dtype=np.float64), n_heads) for a in (q, k, v))
    o = np.zeros((T, n_heads, d))
    lse = np.zeros((T, n_heads))
    for b in range(T // s):
        sl = slice(b * s, (b + 1) * s)
        for n in range(n_heads):
            S = _scores(qh[sl, n], kh[sl, n], d)
            m = S.max(axis=1, keepdims=True)
            e = np.exp(S - m)
            z = e.sum(axis=1, keepdims=True)
            lse[sl, n] = (m + np.log(z))[:, 0]
            o[sl, n] = (e / z) @ vh[sl, n]
    return o.reshape(T, H), lse


def attention_forward_stored(qkv, s: int, n_heads: int) -> Dict:
    """What the forward pass leaves behind: o in fp16 (from fp16 probabilities) and lse in fp32."""
    T, H3 = qkv.shape
    H = H3 // 3
    d = H // n_heads
    q, k, v = (O.as_f64(qkv[:, i * H:(i + 1) * H]) for i in range(3))
    qh, kh, vh = (_heads(a, n_heads) for a in (q, k, v))
    o = np.zeros((T, n_heads, d))
    lse = np.zeros((T, n_heads), dtype=np.float32)
    for b in range(T // s):
        sl = slice(b * s, (b + 1) * s)
        for n in range(n_heads):
            S = _scores(qh[sl, n], kh[sl, n], d)
            m = S.max(axis=1, keepdims=True)
            l = (m + np.log(np.exp(S - m).sum(axis=1, keepdims=True)))[:, 0].astype(np.float32)
            lse[sl, n] = l
            P16 = O.round_f16(np.exp(S - l.astype(np.float64)[:, None]))
            o[sl, n] = O.as_f64(P16) @ vh[sl, n]
    return {"o": O.round_f16(o.reshape(T, H)), "lse": lse}


def attention_backward(qkv, o, do, lse, s: int, n_heads: int, round_probabilities: bool = True) -> np.ndarray:
    """[dq' | dk' | dv] in fp64 (before the rotary backward step) from the saved fp16 qkv (rotated q and k),
    fp16 o, fp32 lse and the incoming do.  With round_probabilities the probabilities P and their scaled
    gradients dS pass through fp16 before the matrix products that consume them."""
    T, H3 = qkv.shape
    H = H3 // 3
    d = H // n_heads
    cast = (lambda a: O.as_f64(a)) if qkv.dtype == np.float16 else (lambda a: np.asarray(a, dtype=np.float64))
    q, k, v = (_heads(cast(qkv[:, i * H:(i + 1) * H]), n_heads) for i in range(3))
    oh = _heads(cast(o), n_heads)
    doh = _heads(cast(do), n_heads)
    rnd = (lambda a: O.as_f64(O.round_f16(a))) if round_probabilities else (lambda a: a)
    out = np.zeros((T, 3, n_heads, d))
    with np.errstate(invalid="ignore", over="ignore"):
        for b in range(T // s):
            sl = slice(b * s, (b + 1) * s)
            for n in range(n_heads):
                S = _scores(q[sl, n], k[sl, n], d)
                P = np.exp(S - np.asarray(lse[sl, n], dtype=np.float64)[:, None])
                dP = doh[sl, n] @ v[sl, n].T
                delta = (doh[sl, n] * oh[sl, n]).sum(axis=1, keepdims=True)
                dS = np.where(P > 0, P * (dP - delta), 0.0) / math.sqrt(d)
                out[sl, 0, n] = rnd(dS) @ k[sl, n]
                out[sl, 1, n] = rnd(dS).T @ q[sl, n]
                out[sl, 2, n] = rnd(P).T @ doh[sl, n]
    return out.reshape(T, 3 * H)


def attention_rounding_sensitivity(qkv, o, do, lse, s: int, n_heads: int) -> np.ndarray:
    """How far one fp16 ulp of a single entry of P or dS can move each element of [dq | dk | dv] (after the
    rotary step, where a pair shares its two bounds): 2^-11 * max_j |dS_ij| * max_j |k_jc| for dq, and likewise
    for dk and dv.  The probabilities are recomputed in fp32 by an implementation and in fp64 here, so an entry
    that sits on a rounding boundary may legitimately round either way; tests allow two such flips."""
    T, H3 = qkv.shape
    H = H3 // 3
    d = H // n_heads
    q, k, v = (_heads(O.as_f64(qkv[:, i * H:(i + 1) * H]), n_heads) for i in range(3))
    oh, doh = _heads(O.as_f64(o), n_heads), _heads(O.as_f64(do), n_heads)
    out = np.zeros((T, 3, n_heads, d))
    with np.errstate(invalid="ignore", over="ignore"):
        for b in range(T // s):
            sl = slice(b * s, (b + 1) * s)
            for n in range(n_heads):
                S = _scores(q[sl, n], k[sl, n], d)
                P = np.exp(S - np.asarray(lse[sl, n], dtype=np.float64)[:, None])
                dP = doh[sl, n] @ v[sl, n].T
                delta = (doh[sl, n] * oh[sl, n]).sum(axis=1, keepdims=True)
                dS = np.abs(np.where(P > 0, P * (dP - delta), 0.0)) / math.sqrt(d)
                out[sl, 0, n] = dS.max(axis=1)[:, None] * np.abs(k[sl, n]).max(axis=0)[None, :]
                out[sl, 1, n] = dS.max(axis=0)[:, None] * np.abs(q[sl, n]).max(axis=0)[None, :]
                out[sl, 2, n] = P.max(axis=0)[:, None] * np.abs(doh[sl, n]).max(axis=0)[None, :]
    # the rotary step mixes columns c and c + d/2 with weights of magnitude <= 1
    for part in (0, 1):
        pair = out[:, part, :, : d // 2] + out[:, part, :, d // 2:]
        out[:, part, :, : d // 2] = pair
        out[:, part, :, d // 2:] = pair
    return 2.0 ** -11 * out.reshape(T, 3 * H)


def attention_rope_backward(qkv, o, do, lse, cos, sin, s: int, n_heads: int) -> np.ndarray:
    """[dq | dk | dv] as stored (fp16): attention backward, rotary backward on the q and k parts, one rounding."""
    T, H3 = qkv.shape
    H = H3 // 3
    g = attention_backward(qkv, o, do, lse, s, n_heads)
    dq = rope_rotate(g[:, :H], cos, sin, s, n_heads, inverse=True)
    dk = rope_rotate(g[:, H:2 * H], cos, sin, s, n_heads, inverse=True)
    return O.round_f16(np.concatenate((dq, dk, g[:, 2 * H:]), axis=1))


# --------------------------------------------------------------------------- the block


def block_forward_f64(h, w, W_qkv, W_o, cos, sin, s: int, n_heads: int, eps: float) -> np.ndarray:
    """y of the attention block in plain fp64 (finite-difference pin)."""
    H = h.shape[1]
    _, _, xn = M.rmsnorm_forward(h, w, eps)
    qkv = xn @ np.asarray(W_qkv, dtype=np.float64).T
    q = rope_rotate(qkv[:, :H], cos, sin, s, n_heads)
    k = rope_rotate(qkv[:, H:2 * H], cos, sin, s, n_heads)
    o, _ = attention_forward_f64(q, k, qkv[:, 2 * H:], s, n_heads)
    return np.asarray(h, dtype=np.float64) + o @ np.asarray(W_o, dtype=np.float64).T


def block_forward_stored(h, w, W_qkv, W_o, cos, sin, s: int, n_heads: int, eps: float) -> Dict:
    """Saved activations of the forward pass, each rounded to its storage type."""
    H = h.shape[1]
    xhat64, r64, _ = M.rmsnorm_forward(h, w, eps)
    xhat = O.round_f16(xhat64)
    xn = O.round_f16(O.as_f64(xhat) * O.as_f64(w)[None, :])
    qkv = O.round_f16(O.as_f64(xn) @ O.as_f64(W_qkv).T)
    q = O.round_f16(rope_rotate(qkv[:, :H], cos, sin, s, n_heads))
    k = O.round_f16(rope_rotate(qkv[:, H:2 * H], cos, sin, s, n_heads))
    qkv_rot = np.concatenate((q, k, qkv[:, 2 * H:]), axis=1)
    att = attention_forward_stored(qkv_rot, s, n_heads)
    y = O.round_f16(O.as_f64(h) + O.as_f64(att["o"]) @ O.as_f64(W_o).T)
    return {"xhat": xhat, "r": r64.astype(np.float32), "xn": xn, "qkv": qkv_rot, "o": att["o"], "lse": att["lse"], "y": y}


def chain_gradients(dy, saved: Dict, w, W_qkv, W_o, cos, sin, s: int, n_heads: int) -> Dict:
    do = O.input_grad(dy, W_o)
    G_o = O.linear_grad(saved["o"], dy)
    dqkv = attention_rope_backward(saved["qkv"], saved["o"], do, saved["lse"], cos, sin, s, n_heads)
    dxn = O.input_grad(dqkv, W_qkv)
    G_qkv = O.linear_grad(saved["xn"], dqkv)
    g_w = O.vector_grad(saved["xhat"], dxn)
    dh = O.round_f16(M.rmsnorm_backward(dxn, saved["xhat"], saved["r"], w, dres=dy))
    return {"do": do, "dqkv": dqkv, "dxn": dxn, "dh": dh, "G_o": G_o, "G_qkv": G_qkv, "g_w": g_w}


def block_step(dy, saved: Dict, w, W_qkv, W_o, cos, sin, s: int, n_heads: int, lr: float, loss_scale: float,
               max_norm: float = 1.0, eps_clip: float = 1e-6) -> Dict:
    """Two-pass LOMO step over the attention block, parameters in backward order W_o, W_qkv, w.  As in the
    feed-forward block no hand-on gradient depends on an updated parameter, so the fused order of
    Algorithm 1 gives the materialised result computed here."""
    c = chain_gradients(dy, saved, w, W_qkv, W_o, cos, sin, s, n_heads)
    grads = [c["G_o"], c["G_qkv"], c["g_w"]]
    flags = [O.has_overflow(g) for g in grads]
    sq = [O.sqnorm(g) for g in grads]
    overflow = any(flags)
    total = math.fsum(sq) if not overflow else float("nan")
    norm = O.grad_norm(total, loss_scale) if not overflow else float("nan")
    coef = O.clip_coef(norm, max_norm, eps_clip) if not overflow else float("nan")
    params = [W_o, W_qkv, w]
    new = [np.array(p, copy=True) if overflow else O.sgd_update(p, g, lr, coef, loss_scale)
           for p, g in zip(params, grads)]
    return {"W_o": new[0], "W_qkv": new[1], "w": new[2], "dh": c["dh"], "do": c["do"], "dqkv": c["dqkv"],
            "dxn": c["dxn"], "flags": flags, "sqnorms": sq, "overflow": overflow, "total_sqnorm": total,
            "norm": norm, "clip_coef": coef}


# --------------------------------------------------------------------------- the whole decoder layer


def layer_forward_f64(h, p: Dict, cos, sin, s: int, n_heads: int, eps: float) -> np.ndarray:
    """Output of the decoder layer (attention block, then feed-forward block) in plain fp64."""
    y1 = block_forward_f64(h, p["w1"], p["W_qkv"], p["W_o"], cos, sin, s, n_heads, eps)
    return M.block_forward_f64(y1, p["w2"], p["W_gu"], p["W_d"], eps)


def layer_forward_stored(h, p: Dict, cos, sin, s: int, n_heads: int, eps: float):
    """Saved activations of both blocks; the feed-forward block reads the stored (fp16) attention-block output."""
    sa = block_forward_stored(h, p["w1"], p["W_qkv"], p["W_o"], cos, sin, s, n_heads, eps)
    sm = M.block_forward_stored(sa["y"], p["w2"], p["W_gu"], p["W_d"], eps)
    return sa, sm


LAYER_ORDER = ("W_d", "W_gu", "w2", "W_o", "W_qkv", "w1")      # backward order of the six parameters


def layer_step(dy, saved_attn: Dict, saved_mlp: Dict, p: Dict, cos, sin, s: int, n_heads: int, lr: float,
               loss_scale: float, max_norm: float = 1.0, eps_clip: float = 1e-6) -> Dict:
    """Two-pass LOMO step over one decoder layer: the walk of Algorithm 1 goes through the feed-forward block,
    hands its input gradient to the attention block, and one global norm over the six parameters sets the
    clipping coefficient (section 3.3.1)."""
    cm = M.chain_gradients(dy, saved_mlp, p["w2"], p["W_gu"], p["W_d"])
    ca = chain_gradients(cm["dh"], saved_attn, p["w1"], p["W_qkv"], p["W_o"], cos, sin, s, n_heads)
    grads = [cm["G_d"], cm["G_gu"], cm["g_w"], ca["G_o"], ca["G_qkv"], ca["g_w"]]
    flags = [O.has_overflow(g) for g in grads]
    sq = [O.sqnorm(g) for g in grads]
    overflow = any(flags)
    total = math.fsum(sq) if not overflow else float("nan")
    norm = O.grad_norm(total, loss_scale) if not overflow else float("nan")
    coef = O.clip_coef(norm, max_norm, eps_clip) if not overflow else float("nan")
    new = {k: (np.array(p[k], copy=True) if overflow else O.sgd_update(p[k], g, lr, coef, loss_scale))
           for k, g in zip(LAYER_ORDER, grads)}
    return {"params": new, "dh": ca["dh"], "dh_mid": cm["dh"], "mlp": cm, "attn": ca, "flags": flags, "sqnorms": sq,
            "overflow": overflow, "total_sqnorm": total, "norm": norm, "clip_coef": coef}


# --------------------------------------------------------------------------- the whole model


def model_forward_stored(ids, m: Dict, cos, sin, s: int, n_heads: int, eps: float) -> Dict:
    """Saved activations of a decoder-only model: embedding rows, the layers, final RMSNorm (the input of the
    output projection W_lm).  m: {"W_emb", "layers": [layer parameter dicts], "w_f", "W_lm"}."""
    h = np.array(m["W_emb"][np.asarray(ids)], copy=True)
    saved = []
    for p in m["layers"]:
        sa, sm = layer_forward_stored(h, p, cos, sin, s, n_heads, eps)
        saved.append((sa, sm))
        h = O.round_f16(O.as_f64(sa["y"]) + O.as_f64(sm["a"]) @ O.as_f64(p["W_d"]).T)
    xhat64, r64, _ = M.rmsnorm_forward(h, m["w_f"], eps)
    xhat = O.round_f16(xhat64)
    xn = O.round_f16(O.as_f64(xhat) * O.as_f64(m["w_f"])[None, :])
    return {"layers": saved, "final": {"xhat": xhat, "r": r64.astype(np.float32), "xn": xn}}


def model_gradients(ids, dlogits, saved: Dict, m: Dict, cos, sin, s: int, n_heads: int) -> Dict:
    """One walk of Algorithm 1's loop over the whole model with the current parameters: every tensor's fp64
    gradient and the stored fp16 hand-ons.  Tensor order: W_lm, w_f, then for each layer from the last to the
    first W_d, W_gu, w2, W_o, W_qkv, w1, finally W_emb."""
    f = saved["final"]
    names, params, grads, handons = [], [], [], {}
    dxn = O.input_grad(dlogits, m["W_lm"])
    names.append("W_lm"); params.append(m["W_lm"]); grads.append(O.linear_grad(f["xn"], dlogits))
    names.append("w_f"); params.append(m["w_f"]); grads.append(O.vector_grad(f["xhat"], dxn))
    dy = O.round_f16(M.rmsnorm_backward(dxn, f["xhat"], f["r"], m["w_f"]))
    handons["dxn_f"], handons["dy_top"] = dxn, dy
    per_layer = []
    for li in range(len(m["layers"]) - 1, -1, -1):
        p = m["layers"][li]
        sa, sm = saved["layers"][li]
        cm = M.chain_gradients(dy, sm, p["w2"], p["W_gu"], p["W_d"])
        ca = chain_gradients(cm["dh"], sa, p["w1"], p["W_qkv"], p["W_o"], cos, sin, s, n_heads)
        for k, g in zip(LAYER_ORDER, (cm["G_d"], cm["G_gu"], cm["g_w"], ca["G_o"], ca["G_qkv"], ca["g_w"])):
            names.append(f"layers.{li}.{k}"); params.append(p[k]); grads.append(g)
        per_layer.append((li, cm, ca))
        dy = ca["dh"]
    names.append("W_emb"); params.append(m["W_emb"]); grads.append(O.embedding_grad(ids, dy, m["W_emb"].shape[0]))
    return {"names": names, "params": params, "grads": grads, "dh0": dy, "handons": handons, "per_layer": per_layer}


def model_step(ids, dlogits, saved: Dict, m: Dict, cos, sin, s: int, n_heads: int, lr: float, loss_scale: float,
               max_norm: float = 1.0, eps_clip: float = 1e-6) -> Dict:
    """Two-pass LOMO step over the whole model (Algorithm 1 from the output projection down to the embedding):
    every hand-on gradient is computed from the old parameters, one norm over every tensor sets the clipping
    coefficient, then every parameter is updated."""
    w = model_gradients(ids, dlogits, saved, m, cos, sin, s, n_heads)
    names, params, grads = w["names"], w["params"], w["grads"]
    flags = [O.has_overflow(g) for g in grads]
    sq = [O.sqnorm(g) for g in grads]
    overflow = any(flags)
    total = math.fsum(sq) if not overflow else float("nan")
    norm = O.grad_norm(total, loss_scale) if not overflow else float("nan")
    coef = O.clip_coef(norm, max_norm, eps_clip) if not overflow else float("nan")
    new = {n_: (np.array(p_, copy=True) if overflow else O.sgd_update(p_, g_, lr, coef, loss_scale))
           for n_, p_, g_ in zip(names, params, grads)}
    return {"params": new, "names": names, "flags": flags, "sqnorms": sq, "overflow": overflow, "total_sqnorm": total,
            "norm": norm, "clip_coef": coef, "dh0": w["dh0"], "handons": w["handons"], "per_layer": w["per_layer"]}


def model_groups(n_layers: int, layers_per_group: int = 1):
    """Tensor indices of the parameter groups in walk order: {W_lm, w_f}, then the layers from the last to the
    first in runs of `layers_per_group` adjacent layers (six tensors each), then {W_emb}."""
    groups = [[0, 1]]
    for k0 in range(0, n_layers, layers_per_group):
        k1 = min(k0 + layers_per_group, n_layers)
        groups.append(list(range(2 + 6 * k0, 2 + 6 * k1)))
    groups.append([2 + 6 * n_layers])
    return groups


def model_step_grouped(ids, dlogits, saved: Dict, m: Dict, cos, sin, s: int, n_heads: int, lr: float,
                       loss_scale: float, max_norm: float = 1.0, eps_clip: float = 1e-6, layers_per_group: int = 1) -> Dict:
    """Single backward walk with the grouped norm of section 3.3.1's closing paragraph: the norm of a group of
    parameters (adjacent layers) stands in for the norm of all of them, so a group can be updated as soon as the
    walk has left it and no second backward pass is needed.  Every group g gets its own coefficient
    min(1, max_norm / (||g_group|| + eps)) -- a biased stand-in for the global one, never smaller than it.

    Each hand-on gradient is taken from a parameter before that parameter's update and the walk never returns
    to a group above, so the gradients are those of the two-pass step.  Overflow: a group with a non-finite
    gradient is not updated, nor is any group after it in the walk; groups above it have been updated already
    and stay so; the step reports overflow to the loss scaler (section 3.3.2)."""
    w = model_gradients(ids, dlogits, saved, m, cos, sin, s, n_heads)
    names, params, grads = w["names"], w["params"], w["grads"]
    flags = [O.has_overflow(g) for g in grads]
    sq = [O.sqnorm(g) for g in grads]
    groups = model_groups(len(m["layers"]), layers_per_group)
    new, g_norm, g_coef, g_over = {}, [], [], []
    stopped = False
    for idx in groups:
        stopped = stopped or any(flags[i] for i in idx)
        g_over.append(stopped)
        if stopped:
            g_norm.append(float("nan")); g_coef.append(float("nan"))
            for i in idx:
                new[names[i]] = np.array(params[i], copy=True)
            continue
        norm = O.grad_norm(math.fsum(sq[i] for i in idx), loss_scale)
        coef = O.clip_coef(norm, max_norm, eps_clip)
        g_norm.append(norm); g_coef.append(coef)
        for i in idx:
            new[names[i]] = O.sgd_update(params[i], grads[i], lr, coef, loss_scale)
    return {"params": new, "names": names, "flags": flags, "sqnorms": sq, "groups": groups, "group_norms": g_norm,
            "group_coefs": g_coef, "group_overflow": g_over, "overflow": stopped, "dh0": w["dh0"],
            "handons": w["handons"], "per_layer": w["per_layer"]}
