"""A whole LOMO training step from token ids on the GPU: forward with checkpoints, loss, backward loop with
recomputation, update (paper sections 3.2, 3.3 and the activation checkpointing of sections 2 and 4.1).

Three layers of evidence.  (1) The layer forward, stage by stage against the oracle on the bits each stage read.
(2) The checkpointed step is bit-identical to the same device forward with every activation kept, followed by the
chained step on those activations (which tests/test_gpu_model.py holds to the oracle): recomputation changes
nothing.  (3) End to end against the oracle from the token ids: loss, norm, and every tensor's update in the
Frobenius norm (device and oracle forward passes differ in last bits, which the backward chain then carries).
"""
import math

import numpy as np
import pytest
import torch

from oracle import lomo_oracle as O
from oracle import mlp_chain as M
from oracle import attn_chain as A
from oracle import loss as LS
from test_gpu_attention import L, DEV, dev, f16, f64, ulps_ok  # noqa: F401
from test_gpu_forward import attention_reference
from test_gpu_model import make_model, to_dev_model, model_tensors

pytestmark = pytest.mark.gpu


def mixed_ok(got, ref64, what, mag=None, frac=0.999):
    """1 ulp on `frac`, everywhere 2 ulp or 2^-9 of the row's rms (stages whose input already carries a rounding)."""
    want = O.round_f16(ref64)
    d = O.ulp_distance_f16(got, want)
    rms = np.sqrt((ref64 ** 2).mean(axis=1, keepdims=True)) if mag is None else mag
    near = np.abs(f64(got) - ref64) <= 2.0 ** -9 * rms
    assert ((d <= 2) | near).all(), (what, d[~((d <= 2) | near)].max())
    assert ((d <= 1) | (np.abs(f64(got) - ref64) <= 2.0 ** -12 * rms)).mean() >= frac, what


@pytest.mark.parametrize("B,s,nh,F", [(2, 128, 2, 344), (3, 192, 3, 1032),
                                      pytest.param(8, 512, 32, 11008, marks=pytest.mark.timeout(900), id="llama7b_layer")])
def test_layer_forward_stage_by_stage(L, B, s, nh, F):
    from paper_2306_09782_amd.chain import LayerActivations, layer_forward
    rng = np.random.default_rng(61)
    H, T = nh * 128, B * s
    p = make_model(rng, 8, H, F, 1)["layers"][0]
    h = f16(rng, (T, H), 1.0)
    cos, sin = A.rope_tables(s, 128)
    act = LayerActivations(DEV, T, H, F, nh)
    h_next = torch.empty(T, H, dtype=torch.float16, device=DEV)
    layer_forward(dev(h), {k: dev(v) for k, v in p.items()}, act, dev(cos), dev(sin), B, s, nh, 1e-5, h_next)
    torch.cuda.synchronize()
    sa = {k: v.cpu().numpy() for k, v in act.attn.items()}
    sm = {k: v.cpu().numpy() for k, v in act.mlp.items()}
    y1, hn = act.y1.cpu().numpy(), h_next.cpu().numpy()
    # attention block
    x64, r64, _ = M.rmsnorm_forward(h, p["w1"], 1e-5)
    ulps_ok(sa["xhat"], O.round_f16(x64), "xhat", worst=1)
    np.testing.assert_allclose(sa["rstd"], r64, rtol=3e-7)
    assert (O.ulp_distance_f16(sa["xn"], O.round_f16(f64(sa["xhat"]) * f64(p["w1"])[None, :])) == 0).all()
    raw = O.round_f16(f64(sa["xn"]) @ f64(p["W_qkv"]).T)
    rot = np.concatenate((A.rope_rotate(raw[:, :H], cos, sin, s, nh), A.rope_rotate(raw[:, H:2 * H], cos, sin, s, nh),
                          f64(raw[:, 2 * H:])), axis=1)
    # an input of the rotation may sit one ulp off the oracle's (the contraction's last bit), which moves the output by up
    # to that ulp times |cos| + |sin|; where the contraction's terms cancel, its fp32 accumulation error (2^-20 of the sum
    # of their magnitudes, as for every contraction here) passes through the rotation as well
    terms = np.abs(f64(sa["xn"])) @ np.abs(f64(p["W_qkv"])).T
    pair = (np.abs(f64(raw)) + 2.0 ** -10 * terms).reshape(T, 3 * nh, 2, 64)
    pair = np.broadcast_to(pair.sum(axis=2, keepdims=True), pair.shape).reshape(T, 3 * H)
    mixed_ok(sa["qkv"], rot, "rotated qkv", mag=pair)
    o64, lse64, mag = attention_reference(sa["qkv"], s, nh)
    np.testing.assert_allclose(sa["lse"], lse64, rtol=1e-5, atol=1e-5)
    mixed_ok(sa["o"], o64, "o", mag=2.0 * mag, frac=0.99)
    ref = f64(h) + f64(sa["o"]) @ f64(p["W_o"]).T
    ulps_ok(y1, O.round_f16(ref), "y1", near=np.abs(f64(y1) - ref) <= 2.0 ** -20 * (np.abs(f64(h)) + np.abs(f64(sa["o"])) @ np.abs(f64(p["W_o"])).T))
    # feed-forward block
    x64, r64, _ = M.rmsnorm_forward(y1, p["w2"], 1e-5)
    ulps_ok(sm["xhat"], O.round_f16(x64), "xhat2", worst=1)
    ref = f64(sm["xn"]) @ f64(p["W_gu"]).T
    ulps_ok(sm["gate_up"], O.round_f16(ref), "gate_up", near=np.abs(f64(sm["gate_up"]) - ref) <= 2.0 ** -20 * (np.abs(f64(sm["xn"])) @ np.abs(f64(p["W_gu"])).T))
    ulps_ok(sm["a"], O.round_f16(M.silu(f64(sm["gate_up"][:, :F])) * f64(sm["gate_up"][:, F:])), "a", worst=1)
    ref = f64(y1) + f64(sm["a"]) @ f64(p["W_d"]).T
    ulps_ok(hn, O.round_f16(ref), "layer output", near=np.abs(f64(hn) - ref) <= 2.0 ** -20 * (np.abs(f64(y1)) + np.abs(f64(sm["a"])) @ np.abs(f64(p["W_d"])).T))
    # the whole layer against the oracle's stored forward
    if T * H <= 1 << 20:
        osa, osm = A.layer_forward_stored(h, p, cos, sin, s, nh, 1e-5)
        want = O.round_f16(f64(osa["y"]) + f64(osm["a"]) @ f64(p["W_d"]).T)
        assert np.linalg.norm(f64(hn) - f64(want)) / np.linalg.norm(f64(want)) < 2.0 ** -10


def problem(rng, B, s, nh, F, V, n_layers):
    H, T = nh * 128, B * s
    m = make_model(rng, V, H, F, n_layers)
    m["W_emb"] = f16(rng, (V, H), 1.0)
    ids = rng.integers(0, V, size=T).astype(np.int32)
    ids[T // 2:T // 2 + 20] = ids[3]
    targets = np.roll(ids, -1).astype(np.int32)
    targets[s - 1::s] = -100                      # no next token at the end of a sequence
    cos, sin = A.rope_tables(s, 128)
    return m, ids, targets, cos, sin


def kept_activation_step(B, s, nh, F, V, n_layers, m, ids, targets, n_counted, cos, sin, lr, scale, max_norm, grouped):
    """The same kernels without checkpointing: every layer's activations kept, then the chained step on them."""
    from paper_2306_09782_amd.chain import (LayerActivations, layer_forward, LomoModelChain, LomoGroupedNormChain)
    import paper_2306_09782_amd as Lb
    H, T = nh * 128, B * s
    dm = to_dev_model(m)
    dcos, dsin, dids = dev(cos), dev(sin), dev(ids)
    hs = [torch.empty(T, H, dtype=torch.float16, device=DEV) for _ in range(n_layers + 1)]
    acts = [LayerActivations(DEV, T, H, F, nh) for _ in range(n_layers)]
    Lb.lomo_embedding_forward(dids, dm["W_emb"], hs[0])
    for li in range(n_layers):
        layer_forward(hs[li], dm["layers"][li], acts[li], dcos, dsin, B, s, nh, 1e-5, hs[li + 1])
    final = {"xhat": torch.empty(T, H, dtype=torch.float16, device=DEV), "rstd": torch.empty(T, dtype=torch.float32, device=DEV),
             "xn": torch.empty(T, H, dtype=torch.float16, device=DEV)}
    Lb.lomo_rmsnorm_forward(hs[n_layers], dm["w_f"], 1e-5, final["xhat"], final["rstd"], final["xn"])
    logits = torch.empty(T, V, dtype=torch.float16, device=DEV)
    Lb.lomo_linear_forward(final["xn"], dm["W_lm"], logits)
    loss = torch.empty(T, dtype=torch.float32, device=DEV)
    raw_logits = logits.clone()
    Lb.lomo_cross_entropy(logits, dev(targets), scale / n_counted, loss, logits)
    saved = {"layers": [(a.attn, a.mlp) for a in acts], "final": final}
    chain = (LomoGroupedNormChain(DEV, B, s, H, F, nh, n_layers, layers_per_group=grouped) if grouped
             else LomoModelChain(DEV, B, s, H, F, nh, n_layers))
    chain.step(dids, logits, saved, dm, dcos, dsin, lr, scale, max_norm)
    torch.cuda.synchronize()
    return dm, chain, raw_logits.cpu().numpy(), loss.cpu().numpy()


@pytest.mark.parametrize("norm,kw", [("global", dict(checkpoint=False)), ("global", dict(checkpoint=False, keep_handons=True)),
                                     ("global", dict(checkpoint=False, keep_handons=True, overlap_norm_pass=True)),
                                     ("grouped", dict(checkpoint=False))])
def test_memory_policies_do_not_change_a_bit(L, norm, kw):
    """Keeping the activations (and the hand-ons) instead of recomputing them gives the checkpointed step's bits."""
    from paper_2306_09782_amd.chain import LomoFineTuneStep
    rng = np.random.default_rng(64)
    B, s, nh, F, V, n_layers, scale = 2, 64, 1, 344, 256, 3, 1024.0
    m, ids, targets, cos, sin = problem(rng, B, s, nh, F, V, n_layers)
    n_counted = int((targets >= 0).sum())
    out = []
    for extra in (dict(), kw):
        step = LomoFineTuneStep(DEV, B, s, nh * 128, F, nh, n_layers, V, norm=norm, **extra)
        dm = to_dev_model(m)
        step.step(dev(ids), dev(targets), dm, dev(cos), dev(sin), 0.05, scale, 1e30)
        torch.cuda.synchronize()
        out.append((dm, step.result()))
    (d1, r1), (d2, r2) = out
    assert r1["loss"] == r2["loss"] and r1["overflow"] is False and r2["overflow"] is False
    if norm == "global":
        assert abs(r1["norm"] / r2["norm"] - 1) < 1e-12 and r1["flags"] == r2["flags"]
    same = lambda a, b: torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert same(d1["W_emb"], d2["W_emb"]) and same(d1["W_lm"], d2["W_lm"]) and same(d1["w_f"], d2["w_f"])
    for p1, p2 in zip(d1["layers"], d2["layers"]):
        for k in p1:
            assert same(p1[k], p2[k]), k


@pytest.mark.parametrize("norm,per", [("global", 1), ("grouped", 1), ("grouped", 2)])
def test_checkpointed_step_equals_kept_activation_step_bit_for_bit(L, norm, per):
    from paper_2306_09782_amd.chain import LomoFineTuneStep
    rng = np.random.default_rng(62)
    B, s, nh, F, V, n_layers, scale = 2, 64, 1, 344, 256, 3, 1024.0
    m, ids, targets, cos, sin = problem(rng, B, s, nh, F, V, n_layers)
    n_counted = int((targets >= 0).sum())
    lr = 0.05
    ref, ref_chain, _, ref_loss = kept_activation_step(B, s, nh, F, V, n_layers, m, ids, targets, n_counted, cos, sin, lr, scale,
                                                       1e30, per if norm == "grouped" else 0)
    step = LomoFineTuneStep(DEV, B, s, nh * 128, F, nh, n_layers, V, norm=norm, layers_per_group=per)
    dm = to_dev_model(m)
    step.step(dev(ids), dev(targets), dm, dev(cos), dev(sin), lr, scale, 1e30)
    torch.cuda.synchronize()
    res = step.result()
    assert res["overflow"] is False and abs(res["loss"] - ref_loss.astype(np.float64).sum() / n_counted) < 1e-9
    same = lambda a, b: torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert same(ref["W_emb"], dm["W_emb"]) and same(ref["W_lm"], dm["W_lm"]) and same(ref["w_f"], dm["w_f"])
    for p1, p2 in zip(ref["layers"], dm["layers"]):
        for k in p1:
            assert same(p1[k], p2[k]), k
    moved = (dm["layers"][0]["W_qkv"].cpu().numpy().view(np.uint16) != m["layers"][0]["W_qkv"].view(np.uint16)).mean()
    assert moved > 0.05, moved


@pytest.mark.parametrize("norm,shape", [("global", (2, 128, 2, 344, 512, 2)), ("grouped", (2, 128, 2, 344, 512, 2)),
                                        ("global", (3, 192, 3, 1032, 1000, 1))])
def test_training_step_from_token_ids_against_the_oracle(L, norm, shape):
    from paper_2306_09782_amd.chain import LomoFineTuneStep
    rng = np.random.default_rng(63)
    B, s, nh, F, V, n_layers = shape
    scale = 4096.0
    m, ids, targets, cos, sin = problem(rng, B, s, nh, F, V, n_layers)
    n_counted = int((targets >= 0).sum())
    saved = A.model_forward_stored(ids, m, cos, sin, s, nh, 1e-5)
    logits = O.round_f16(f64(saved["final"]["xn"]) @ f64(m["W_lm"]).T)
    ce = LS.cross_entropy(logits, targets, scale)
    stepper = A.model_step if norm == "global" else A.model_step_grouped
    probe = A.model_step_grouped(ids, ce["dlogits_f16"], saved, m, cos, sin, s, nh, 1.0, scale, max_norm=1e30)
    norms = sorted(probe["group_norms"])
    max_norm = math.sqrt(norms[-1] * norms[-2])          # clips the largest group (and the global norm)
    k = probe["names"].index("layers.0.W_gu")
    typical = math.sqrt(probe["sqnorms"][k] / m["layers"][0]["W_gu"].size) / scale
    lr = float(np.float32(20 * 2.0 ** -16 / typical))     # the layers' weights move by tens of ulps
    want = stepper(ids, ce["dlogits_f16"], saved, m, cos, sin, s, nh, lr, scale, max_norm=max_norm)
    step = LomoFineTuneStep(DEV, B, s, nh * 128, F, nh, n_layers, V, norm=norm)
    dm = to_dev_model(m)
    step.step(dev(ids), dev(targets), dm, dev(cos), dev(sin), lr, scale, max_norm)
    torch.cuda.synchronize()
    res = step.result()
    assert res["overflow"] is False and res["flags"] == want["flags"]
    assert abs(res["loss"] / ce["loss"] - 1) < 1e-3
    if norm == "global":
        assert abs(res["norm"] / want["norm"] - 1) < 2e-3 and abs(res["clip_coef"] / want["clip_coef"] - 1) < 2e-3
    else:
        for a, b in zip(res["group_norms"], want["group_norms"]):
            assert abs(a / b - 1) < 2e-3
    got, old = model_tensors(dm, n_layers, want["names"]), model_tensors(m, n_layers, want["names"])
    for name in want["names"]:
        w = want["params"][name]
        d = O.ulp_distance_f16(got[name], w)
        wu = f64(w) - f64(old[name])
        # an element whose gradient terms cancel carries the chain's differences relative to the terms, not to itself
        near = np.abs(f64(got[name]) - f64(w)) <= 2.0 ** -6 * np.abs(wu) + 2.0 ** -8 * math.sqrt(float((wu ** 2).mean()))
        assert ((d <= 1) | near).all(), (name, d[~((d <= 1) | near)].max())
        assert (d == 0).mean() >= 0.95, (name, (d == 0).mean())
        if w.ndim == 2 and name != "W_emb":
            assert (w.view(np.uint16) != old[name].view(np.uint16)).mean() > 0.5, name


@pytest.mark.parametrize("norm", ["global", "grouped"])
def test_training_run_with_the_dynamic_scaler_follows_the_oracle(L, norm):
    """Ten steps on a repeated batch: a scale that overflows fp16 in the loss gradient drops the step and halves,
    three clean steps double it again; the losses follow the oracle's run and go down."""
    from paper_2306_09782_amd.chain import LomoFineTuneStep, LomoTrainer
    from oracle import training as TR
    rng = np.random.default_rng(71)
    B, s, nh, F, V, n_layers = 2, 64, 1, 344, 256, 2
    m, ids, targets, cos, sin = problem(rng, B, s, nh, F, V, n_layers)
    n = int((targets >= 0).sum())
    S0 = 2.0 ** 24
    assert S0 / 2 / n > 65504 * 1.01 and S0 / 4 / n < 65504 / 1.9      # inf at S0 and S0 / 2 for certain, far from it at S0 / 4
    steps, lr = 10, 0.05
    _, log = TR.training_steps(ids, targets, m, cos, sin, s, nh, 1e-5, steps, lr, S0, 3, grouped=(norm == "grouped"))
    assert [r["overflow"] for r in log] == [True, True, False, False, False, True, False, False, False, True]
    trainer = LomoTrainer(LomoFineTuneStep(DEV, B, s, nh * 128, F, nh, n_layers, V, norm=norm), lr, S0, 3)
    dm = to_dev_model(m)
    dids, dt, dcos, dsin = dev(ids), dev(targets), dev(cos), dev(sin)
    before = None
    for k, want in enumerate(log):
        if want["overflow"]:
            before = {name: t.clone() for name, t in dm["layers"][0].items()}
        res = trainer.train_step(dids, dt, dm, dcos, dsin)
        assert res["overflow"] is want["overflow"] and res["loss_scale"] == want["loss_scale"], k
        assert abs(res["loss"] / want["loss"] - 1) < 2e-3, (k, res["loss"], want["loss"])
        if want["overflow"]:      # dropped (the loss gradient itself overflowed, so the first group already): nothing moved
            assert all(torch.equal(before[name].view(torch.int16), t.view(torch.int16)) for name, t in dm["layers"][0].items())
    assert log[-1]["loss"] < log[0]["loss"] - 0.01
