"""CPU oracle for a run of LOMO training steps with the dynamic loss scaler -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file; the HIP path never
does, and this file imports nothing from it.  It composes the other oracle modules and adds no arithmetic of
its own: per step, the stored forward pass (attn_chain.model_forward_stored), the logits of the output
projection rounded to fp16, the cross-entropy and its scaled gradient (loss.cross_entropy), the step over the
whole model (attn_chain.model_step, or model_step_grouped for the grouped norm of section 3.3.1), and the
dynamic loss scaler of section 3.3.2 (lomo_oracle.scaler_step): an overflowing step is dropped and halves the
scale; `growth_interval` clean steps in a row double it.

Pins (tests/test_oracle_pins.py): on a repeated batch the loss of a small model goes down step after step; a
scale that overflows fp16 drops the step (parameters bit-unchanged) and halves; after `growth_interval` clean
steps the scale doubles; a dropped step leaves the next loss exactly where it was.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import attn_chain as A
from . import loss as LS
from . import lomo_oracle as O


def _with_params(m: Dict, new: Dict) -> Dict:
    layers = [{k: new[f"layers.{li}.{k}"] for k in p} for li, p in enumerate(m["layers"])]
    return {"W_emb": new["W_emb"], "layers": layers, "w_f": new["w_f"], "W_lm": new["W_lm"]}


def training_steps(ids, targets, m: Dict, cos, sin, s: int, n_heads: int, eps: float, n_steps: int, lr: float,
                   loss_scale: float, growth_interval: int, max_norm: float = 1.0, eps_clip: float = 1e-6,
                   grouped: bool = False):
    """Runs n_steps on the same batch.  Returns (final parameters, per-step records {loss, loss_scale (the one the
    step used), overflow, norm})."""
    clean = 0
    log: List[Dict] = []
    for _ in range(n_steps):
        saved = A.model_forward_stored(ids, m, cos, sin, s, n_heads, eps)
        logits = O.round_f16(O.as_f64(saved["final"]["xn"]) @ O.as_f64(m["W_lm"]).T)
        ce = LS.cross_entropy(logits, targets, loss_scale)
        stepper = A.model_step_grouped if grouped else A.model_step
        with np.errstate(over="ignore", invalid="ignore"):
            out = stepper(ids, ce["dlogits_f16"], saved, m, cos, sin, s, n_heads, lr, loss_scale, max_norm=max_norm,
                          eps_clip=eps_clip)
        log.append({"loss": ce["loss"], "loss_scale": loss_scale, "overflow": bool(out["overflow"]),
                    "norm": out.get("norm", None)})
        m = _with_params(m, out["params"])
        loss_scale, clean = O.scaler_step(loss_scale, clean, growth_interval, out["overflow"])
    return m, log
