"""CPU oracle for the loss that starts LOMO's backward loop -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file; the HIP path never
does, and this file imports nothing from it.

The paper fine-tunes causal language models (section 4), whose loss is the mean token-level cross-entropy of the
logits z = xn W_lm^T against the next token; with loss scaling (section 3.3.2) the loss is multiplied by the
scale S before the backward pass, so the gradient that enters Algorithm 1's loop is

    loss_t   = log sum_v exp(z[t, v]) - z[t, target_t]
    dz[t, v] = S / n * (softmax(z_t)[v] - [v == target_t])          n = number of counted tokens

A token whose target lies outside [0, V) is not counted (loss 0, zero gradient row): the usual way to leave out
padding or prompt positions.  fp64 throughout; the gradient is rounded once to fp16 where it is stored.

Pins (tests/test_oracle_pins.py): central finite differences of the scaled mean loss; rows of dz sum to zero and
dz[t, target] < 0; uniform logits give log V; agreement with scipy.special.log_softmax; ignored tokens.
"""
from __future__ import annotations

from typing import Dict

import numpy as np

from . import lomo_oracle as O


def token_losses(logits, targets) -> np.ndarray:
    """loss_t in fp64 (0 for tokens that are not counted)."""
    z = np.asarray(logits, dtype=np.float64)
    T, V = z.shape
    out = np.zeros(T)
    for t in range(T):
        tgt = int(targets[t])
        if 0 <= tgt < V:
            m = z[t].max()
            out[t] = m + np.log(np.exp(z[t] - m).sum()) - z[t, tgt]
    return out


def cross_entropy(logits, targets, loss_scale: float) -> Dict:
    """Mean loss over the counted tokens and the gradient of (loss_scale * mean loss) w.r.t. the logits."""
    z = np.asarray(logits, dtype=np.float64)
    T, V = z.shape
    tg = np.asarray(targets).astype(np.int64)
    counted = (tg >= 0) & (tg < V)
    n = int(counted.sum())
    losses = token_losses(z, tg)
    dz = np.zeros((T, V))
    for t in range(T):
        if counted[t]:
            m = z[t].max()
            e = np.exp(z[t] - m)
            p = e / e.sum()
            p[tg[t]] -= 1.0
            dz[t] = p * (loss_scale / n)
    return {"loss": float(losses.sum() / n) if n else 0.0, "token_losses": losses, "n": n, "dlogits": dz,
            "dlogits_f16": O.round_f16(dz)}
