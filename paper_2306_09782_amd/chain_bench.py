#!/usr/bin/env python3
"""Timings of the chained backward loop (one decoder layer, a whole model, a whole fine-tuning step from token ids).

These are the steps either side of the hot path that bench.py measures; they are not part of its JSON line.
    python -m paper_2306_09782_amd.chain_bench --chain | --model-chain | --train-step [--train-model 13b ...]
Prints one JSON object.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0     # MI355X dense fp16 MFMA peak, published


def chain_bench(L, torch, np, dev, steps, warmup):
    """Two-pass step through one whole 7B decoder layer (8 x 512 tokens, H = 4096, 32 heads, F = 11008) with the
    hand-on gradients produced by the kernels themselves: 4 GEMMs per linear tensor, as in the paper's two
    backward passes.  Synthetic saved activations (the chain's arithmetic does not care what they hold)."""
    from paper_2306_09782_amd.chain import LomoDecoderLayer
    import lomo_synth as S
    Bt, s, nh, H, F = 8, 512, 32, 4096, 11008
    T = Bt * s
    key = lambda i: S.tensor_key(0, 99, i, 0)
    gen = lambda i, shape, sigma: S.normal_f16_torch(key(i), shape, S.normal_mult(sigma), dev)
    ones = lambda n, dt: torch.ones(n, dtype=dt, device=dev)
    sm = {"a": gen(0, (T, F), 0.3), "xn": gen(1, (T, H), 1.0), "xhat": gen(2, (T, H), 1.0),
          "gate_up": gen(3, (T, 2 * F), 1.0), "rstd": ones(T, torch.float32)}
    sa = {"o": gen(7, (T, H), 0.2), "xn": gen(8, (T, H), 1.0), "xhat": gen(9, (T, H), 1.0), "qkv": gen(10, (T, 3 * H), 1.0),
          "rstd": ones(T, torch.float32), "lse": torch.full((T, nh), 4.0, dtype=torch.float32, device=dev)}
    p = {"w1": ones(H, torch.float16), "w2": ones(H, torch.float16), "W_qkv": gen(11, (3 * H, H), 0.02),
         "W_o": gen(12, (H, H), 0.02), "W_gu": gen(4, (2 * F, H), 0.02), "W_d": gen(5, (H, F), 0.02)}
    ang = torch.arange(s, device=dev, dtype=torch.float64)[:, None] * (10000.0 ** (-torch.arange(64, device=dev, dtype=torch.float64) / 64.0))[None, :]
    cos, sin = torch.cos(ang).float().contiguous(), torch.sin(ang).float().contiguous()
    dy = gen(6, (T, H), 1e-3 * 65536.0)
    dh = torch.empty(T, H, dtype=torch.float16, device=dev)
    layer = LomoDecoderLayer(dev, Bt, s, H, F, nh)
    run = lambda: layer.step(dy, sa, sm, p, cos, sin, dh, 1e-2, 65536.0)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    L.lomo_timing_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    fam = {name: L.lomo_timing_read(i) for i, name in enumerate(L.KERNEL_FAMILIES)}
    L.lomo_timing_enable(False)
    res = layer.result()

    def timed(fn, reps=20):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    m, at = layer.mlp, layer.attn
    sw_ms = timed(lambda: L.lomo_swiglu_backward(m.da, sm["gate_up"], m.dgu))
    rn_ms = timed(lambda: L.lomo_rmsnorm_backward(m.dxn, sm["xhat"], sm["rstd"], p["w2"], dy, dh))
    at_ms = timed(lambda: L.lomo_attention_backward(sa["qkv"], sa["o"], at.do, sa["lse"], cos, sin, at.delta, at.dqkv, Bt, s, nh))
    sw_bytes, rn_bytes = 5 * T * F * 2, 4 * T * H * 2 + 4 * T + 2 * H
    # attention backward: 7 block products of 2 * 64 * 64 * 128 flop per (query block, key block) pair at or below
    # the diagonal (S and dP in both kernels, dv, dk, dq once); bytes: qkv, o, dO read, dqkv written, once each
    nb = s // 64
    at_flops = Bt * nh * (nb * (nb + 1) // 2) * 7 * 2 * 64 * 64 * 128
    at_bytes = (3 * T * H + T * H + T * H + 3 * T * H) * 2
    lin_flops = 2 * T * H * (3 * H + H + 2 * F + F)
    flops = 4 * lin_flops + 2 * at_flops
    return {"workload": "one 7B decoder layer, chained (8 x 512 tokens, H 4096, 32 heads, F 11008)", "ms_per_step": ms,
            "gemms_per_linear": 4, "tflops": flops / (ms * 1e-3) / 1e12, "grad_norm": res["norm"], "overflow": res["overflow"],
            "family_ms_per_step": {k: v[0] / steps for k, v in fam.items() if v[1]},
            "swiglu_backward": {"ms": sw_ms, "algorithmic_bytes": sw_bytes, "gb_per_s": sw_bytes / sw_ms / 1e6,
                                "frac_hbm_peak": sw_bytes / sw_ms / 1e6 / 8000.0},
            "rmsnorm_backward": {"ms": rn_ms, "algorithmic_bytes": rn_bytes, "gb_per_s": rn_bytes / rn_ms / 1e6,
                                 "frac_hbm_peak": rn_bytes / rn_ms / 1e6 / 8000.0},
            "attention_backward": {"ms": at_ms, "flops": at_flops, "tflops": at_flops / (at_ms * 1e-3) / 1e12,
                                   "frac_fp16_mfma_peak": at_flops / (at_ms * 1e-3) / 1e12 / PEAK_FP16_TFLOPS,
                                   "algorithmic_bytes": at_bytes, "gb_per_s": at_bytes / at_ms / 1e6}}


def model_chain_bench(L, torch, np, dev, steps, warmup, n_layers=32, keep_handons=False, grouped=0):
    """Two-pass step through a whole 7B-shaped decoder-only model (32 layers, H = 4096, 32 heads, F = 11008,
    vocabulary 32000, 8 x 512 tokens): output projection, final norm, every layer, embedding table, with every
    hand-on gradient produced by the kernels.  Synthetic saved activations, one set per layer (17 GB), and weight
    scales chosen so that the gradient neither dies nor overflows on its way down 32 random layers."""
    from paper_2306_09782_amd.chain import LomoModelChain, LomoGroupedNormChain
    import lomo_synth as S
    Bt, s, nh, H, F, V = 8, 512, 32, 4096, 11008, 32000
    T = Bt * s
    torch.cuda.reset_peak_memory_stats()
    count = [0]

    def gen(shape, sigma):
        count[0] += 1
        return S.normal_f16_torch(S.tensor_key(0, 98, count[0], 0), shape, S.normal_mult(sigma), dev)
    ones = lambda n, dt: torch.ones(n, dtype=dt, device=dev)
    pos = torch.arange(s, device=dev, dtype=torch.float32).repeat(Bt)
    lse = torch.log(1.65 * (pos + 1.0))[:, None].repeat(1, nh).contiguous()     # rows of P sum to about one
    layers, saved = [], []
    for _ in range(n_layers):
        layers.append({"w1": ones(H, torch.float16), "w2": ones(H, torch.float16), "W_qkv": gen((3 * H, H), 0.005),
                       "W_o": gen((H, H), 0.005), "W_gu": gen((2 * F, H), 0.004), "W_d": gen((H, F), 0.006)})
        sm = {"a": gen((T, F), 0.3), "xn": gen((T, H), 1.0), "xhat": gen((T, H), 1.0), "gate_up": gen((T, 2 * F), 1.0),
              "rstd": ones(T, torch.float32)}
        sa = {"o": gen((T, H), 0.2), "xn": gen((T, H), 1.0), "xhat": gen((T, H), 1.0), "qkv": gen((T, 3 * H), 1.0),
              "rstd": ones(T, torch.float32), "lse": lse}
        saved.append((sa, sm))
    m = {"W_emb": gen((V, H), 1.0), "layers": layers, "w_f": ones(H, torch.float16), "W_lm": gen((V, H), 0.02)}
    final = {"xn": gen((T, H), 1.0), "xhat": gen((T, H), 1.0), "rstd": ones(T, torch.float32)}
    ids = torch.from_numpy(S.zipf_ids(98, T, V).astype(np.int32)).to(dev)
    dlogits = gen((T, V), 1.0)
    ang = torch.arange(s, device=dev, dtype=torch.float64)[:, None] * (10000.0 ** (-torch.arange(64, device=dev, dtype=torch.float64) / 64.0))[None, :]
    cos, sin = torch.cos(ang).float().contiguous(), torch.sin(ang).float().contiguous()
    if grouped:
        chain = LomoGroupedNormChain(dev, Bt, s, H, F, nh, n_layers, layers_per_group=grouped)
    else:
        chain = LomoModelChain(dev, Bt, s, H, F, nh, n_layers, keep_handons=keep_handons)
    sv = {"layers": saved, "final": final}
    run = lambda: chain.step(ids, dlogits, sv, m, cos, sin, 1e-3, 1024.0)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    L.lomo_timing_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    fam = {name: L.lomo_timing_read(i) for i, name in enumerate(L.KERNEL_FAMILIES)}
    L.lomo_timing_enable(False)
    res = chain.result()
    nb = s // 64
    at_flops = Bt * nh * (nb * (nb + 1) // 2) * 7 * 2 * 64 * 64 * 128
    n_lin = n_layers * H * (3 * H + H + 2 * F + F) + V * H
    once = keep_handons or grouped
    gemms = 3 if once else 4
    flops = gemms * 2 * T * n_lin + (1 if once else 2) * n_layers * at_flops
    n_params = n_lin + V * H + (2 * n_layers + 1) * H
    return {"workload": f"7B-shaped model, chained ({n_layers} layers, 8 x 512 tokens, H 4096, 32 heads, F 11008, V 32000)",
            "ms_per_step": ms, "gemms_per_linear": gemms, "hand_ons": (f"kept within a group of {grouped} layer(s), one walk" if grouped else
                                                               "kept from pass 1" if keep_handons else "recomputed in pass 2"),
            "norm": "per group" if grouped else "global", "params": n_params, "tflops": flops / (ms * 1e-3) / 1e12,
            "tokens_per_s_backward_and_update": T / (ms * 1e-3), "params_per_s": n_params / (ms * 1e-3),
            "grad_norm": res["norm"] if not grouped else math.sqrt(sum(v * v for v in res["group_norms"])),
            "clip_coef": res["clip_coef"] if not grouped else [min(res["group_coefs"]), max(res["group_coefs"])],
            "overflow": res["overflow"], "device_memory_gb": torch.cuda.max_memory_allocated() / 1e9,
            "family_ms_per_step": {k: v[0] / steps for k, v in fam.items() if v[1]}}


# layers, hidden width, heads (of width 128), feed-forward width of the LLaMA sizes the paper trains (section 4.2)
TRAIN_MODELS = {"7b": (32, 4096, 32, 11008), "13b": (40, 5120, 40, 13824), "30b": (60, 6656, 52, 17920),
                "65b": (80, 8192, 64, 22016)}


def train_model(torch, dev, name):
    """Random-init weights of a LLaMA-shaped model: sigma 0.02 at H = 4096, scaled with 1 / sqrt(H); gains 1."""
    import lomo_synth as S
    n_layers, H, nh, F = TRAIN_MODELS[name]
    V = 32000
    sig = 0.02 * math.sqrt(4096.0 / H)
    count = [0]

    def gen(shape, sigma):
        count[0] += 1
        return S.normal_f16_torch(S.tensor_key(0, 97, count[0], 0), shape, S.normal_mult(sigma), dev)
    ones = lambda n: torch.ones(n, dtype=torch.float16, device=dev)
    return {"W_emb": gen((V, H), 1.0), "w_f": ones(H), "W_lm": gen((V, H), sig),
            "layers": [{"w1": ones(H), "w2": ones(H), "W_qkv": gen((3 * H, H), sig), "W_o": gen((H, H), sig),
                        "W_gu": gen((2 * F, H), sig), "W_d": gen((H, F), sig)} for _ in range(n_layers)]}


def train_step_bench(L, torch, np, dev, steps, warmup, norm, m, model="7b", batch=8, seq=512, checkpoint=True, keep_handons=False,
                     overlap=False):
    """One whole fine-tuning step of a LLaMA-shaped model from token ids (default 7B: 32 layers, H 4096, 32 heads,
    F 11008, V 32000; 8 x 512 tokens): forward keeping only the layer inputs, cross-entropy, backward loop with every
    layer recomputed from its checkpoint, fused updates.  Random-init weights `m` (updated in place), Zipf token ids;
    the target of a position is the next token."""
    from paper_2306_09782_amd.chain import LomoFineTuneStep
    import lomo_synth as S
    n_layers, H, nh, F = TRAIN_MODELS[model]
    Bt, s, V = batch, seq, 32000
    T = Bt * s
    torch.cuda.reset_peak_memory_stats()
    ids_h = S.zipf_ids(97, T, V).astype(np.int32)
    tg_h = np.roll(ids_h, -1).astype(np.int32)
    tg_h[s - 1::s] = -100
    ids, targets = torch.from_numpy(ids_h).to(dev), torch.from_numpy(tg_h).to(dev)
    ang = torch.arange(s, device=dev, dtype=torch.float64)[:, None] * (10000.0 ** (-torch.arange(64, device=dev, dtype=torch.float64) / 64.0))[None, :]
    cos, sin = torch.cos(ang).float().contiguous(), torch.sin(ang).float().contiguous()
    step = LomoFineTuneStep(dev, Bt, s, H, F, nh, n_layers, V, norm=norm, checkpoint=checkpoint, keep_handons=keep_handons,
                            overlap_norm_pass=overlap)
    run = lambda: step.step(ids, targets, m, cos, sin, 1e-3, 65536.0)
    losses = []
    for _ in range(warmup):
        run()
        torch.cuda.synchronize()
        losses.append(step.result()["loss"])
    L.lomo_timing_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    fam = {name: L.lomo_timing_read(i) for i, name in enumerate(L.KERNEL_FAMILIES)}
    L.lomo_timing_enable(False)
    res = step.result()
    losses.append(res["loss"])
    walks = 2 if (norm == "global" and not keep_handons) else 1
    n_layer_lin = H * (3 * H + H + 2 * F + F)
    n_lin = n_layers * n_layer_lin + V * H
    n_params = n_lin + V * H + (2 * n_layers + 1) * H
    nb = s // 64
    pairs = Bt * nh * (nb * (nb + 1) // 2)
    at_fwd, at_bwd = pairs * 2 * 2 * 64 * 64 * 128, pairs * 7 * 2 * 64 * 64 * 128
    recomputed = n_layers * H * (3 * H + H + 2 * F) * walks - H * (3 * H + H + 2 * F)     # no W_d; last layer once less
    if not checkpoint:
        recomputed = 0
    # forward + recomputation + wgrad (norm pass and update pass: 2 per linear) + dgrad (once per walk)
    gemm_flops = 2 * T * (n_lin + recomputed + 2 * n_lin + walks * n_lin)
    flops = gemm_flops + n_layers * at_fwd * (1 + (walks if checkpoint else 0)) + walks * n_layers * at_bwd
    return {"workload": f"{model.upper()}-shaped model from token ids ({n_layers} layers, H {H}, {nh} heads, F {F}, V 32000; "
                        f"{Bt} x {s} tokens)",
            "activations": "checkpointed and recomputed" if checkpoint else "kept",
            "hand_ons": "kept from pass 1" if keep_handons else "not kept", "norm_pass_on_second_stream": overlap,
            "norm": norm, "backward_walks": walks, "ms_per_step": ms, "tokens_per_s": T / (ms * 1e-3), "params": n_params,
            "executed_tflops": flops / (ms * 1e-3) / 1e12, "model_flops_tflops": 6.0 * n_params * T / (ms * 1e-3) / 1e12,
            "loss_by_step": losses, "grad_norm": res.get("norm", None) if norm == "global" else math.sqrt(sum(v * v for v in res["group_norms"])),
            "overflow": res["overflow"], "device_memory_gb": torch.cuda.max_memory_allocated() / 1e9,
            "family_ms_per_step": {k: v[0] / steps for k, v in fam.items() if v[1]}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=6)
    ap.add_argument("--train-shape", default="8x512", help="batch x sequence length of --train-step (default 8x512)")
    ap.add_argument("--train-model", default="7b", choices=sorted(TRAIN_MODELS), help="model size of --train-step (default 7b)")
    ap.add_argument("--train-policies", default="all", choices=["all", "checkpointed", "kept-activations"],
                    help="--train-step: every memory policy, only the two checkpointed ones, or only the two that keep the "
                         "activations but not the hand-ons (the largest models do not fit the others)")
    ap.add_argument("--train-step", action="store_true", help="a whole fine-tuning step from token ids")
    ap.add_argument("--model-chain", action="store_true", help="the chained two-pass step through a whole 32-layer 7B-shaped model")
    ap.add_argument("--chain", action="store_true", help="the chained two-pass step through one 7B decoder layer")
    args = ap.parse_args()

    import numpy as np
    import torch
    import paper_2306_09782_amd as L
    L.load_library()
    dev = torch.device("cuda:0")
    out = {}
    if args.chain:
        out["chain"] = chain_bench(L, torch, np, dev, max(3, args.steps), 2)
    if args.model_chain:
        torch.cuda.empty_cache()
        out["model_chain"] = model_chain_bench(L, torch, np, dev, 3, 1)
        torch.cuda.empty_cache()
        out["model_chain_kept_handons"] = model_chain_bench(L, torch, np, dev, 3, 1, keep_handons=True)
        torch.cuda.empty_cache()
        out["model_chain_grouped_norm"] = model_chain_bench(L, torch, np, dev, 3, 1, grouped=1)
    if args.train_step:
        torch.cuda.empty_cache()
        tb, ts = (int(v) for v in args.train_shape.split("x"))
        tm = train_model(torch, dev, args.train_model)
        kw = dict(model=args.train_model, batch=tb, seq=ts)
        nst, nwu = (3, 2) if args.train_model == "7b" else (2, 1)
        if args.train_policies != "kept-activations":
            out["train_step_global_norm"] = train_step_bench(L, torch, np, dev, nst, nwu, "global", tm, **kw)
            torch.cuda.empty_cache()
            out["train_step_grouped_norm"] = train_step_bench(L, torch, np, dev, nst, nwu, "grouped", tm, **kw)
        else:
            out["train_step_global_norm_kept_activations"] = train_step_bench(L, torch, np, dev, nst, nwu, "global", tm, checkpoint=False, **kw)
            torch.cuda.empty_cache()
            out["train_step_grouped_norm_kept_activations"] = train_step_bench(L, torch, np, dev, nst, nwu, "grouped", tm,
                                                                               checkpoint=False, **kw)
        if args.train_policies == "all":
            torch.cuda.empty_cache()
            out["train_step_global_norm_kept_activations"] = train_step_bench(L, torch, np, dev, nst, nwu, "global", tm, checkpoint=False, **kw)
            torch.cuda.empty_cache()
            out["train_step_global_norm_kept_activations_and_handons"] = train_step_bench(
                L, torch, np, dev, nst, nwu, "global", tm, checkpoint=False, keep_handons=True, **kw)
            torch.cuda.empty_cache()
            out["train_step_global_norm_kept_activations_and_handons_two_streams"] = train_step_bench(
                L, torch, np, dev, nst, nwu, "global", tm, checkpoint=False, keep_handons=True, overlap=True, **kw)
            torch.cuda.empty_cache()
            out["train_step_grouped_norm_kept_activations"] = train_step_bench(L, torch, np, dev, nst, nwu, "grouped", tm,
                                                                               checkpoint=False, **kw)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
