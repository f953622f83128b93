#!/usr/bin/env python3
"""Benchmark of the two-pass LOMO step (norm pass, clipping coefficient, fused update pass).

A step = pass 1 over every tensor of the workload (squared gradient norm + overflow flags),
the coefficient (a one-thread kernel by default; --host-coefficient reads the norm back and
forms it on the host, one synchronisation per step), pass 2 over every tensor (dgrad from the
pre-update W, then the fused weight-gradient + SGD update) and a copy of the step's scalars to
pinned host memory.  Inputs are synthetic, seeded and resident in HBM before the timed region.  W is not restored between iterations: the clipped updates are far below one
fp16 ulp for these workloads, so the weights drift by at most a few ulps over a run.

Prints ONE JSON line: whole-step throughput, the roofline of the dominant kernel (the fused
wgrad + update GEMM, timed live with HIP events on the launch stream) and the CPU oracle timed
on a bounded sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0     # MI355X dense fp16 MFMA peak, published


def profiled_traffic(workload_name):
    """HBM-side bytes per launch of the fused kernel, from the committed rocprofv3 --pmc summary."""
    path = os.path.join(ROOT, "profiles", f"lomo_contract_{workload_name}_hbm_traffic.txt")
    try:
        for line in open(path):
            if "traffic_bytes_per_launch:" in line:
                return int(line.split("traffic_bytes_per_launch:")[1].split()[0])
    except OSError:
        pass
    return None


def cpu_baseline(wl, max_seconds=25.0):
    """The oracle as it stands, on a bounded sample: the first linear tensors of the workload."""
    import numpy as np
    from oracle import lomo_oracle as O
    budget_flops = 1.2e13          # about 10-20 s of fp64 BLAS on a 16-core host
    sample, flops = [], 0
    for spec in wl.tensors:
        if spec.kind != "linear":
            continue
        f = 2 * spec.gemm_flops                     # gradient + dX
        if sample and flops + f > budget_flops:
            break
        sample.append(spec)
        flops += f
    recs = [dict(kind="linear", X=wl.X_np(s), dY=wl.dY_np(s), W=wl.W_np(s)) for s in sample]
    t0 = time.perf_counter()
    res = O.step_materialised(recs, float(np.float32(wl.lr)), wl.loss_scale, wl.max_norm, wl.eps)
    dt = time.perf_counter() - t0
    params = sum(s.n_params for s in sample)
    try:
        import threadpoolctl
        cores = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{len(sample)} linear tensors of {wl.name} ({', '.join(s.name for s in sample)}), "
                      f"fp64 gradient + dX + update, {flops / 1e12:.2f} TFLOP in {dt:.1f} s",
            "params_per_s": params / dt, "seconds": dt, "norm": res["norm"]}


def hbm_kernels(wl, fam, steps):
    """Achieved GB/s of the bandwidth-bound kernels: algorithmic bytes of both passes / event time."""
    out = {}
    emb = [s for s in wl.tensors if s.kind == "embedding"]
    vec = [s for s in wl.tensors if s.kind == "vector"]
    if emb and fam["embedding"][1]:
        import numpy as np
        by = 0
        for s in emb:
            u = int(np.unique(wl.ids_np(s)).size)
            by += 2 * (4 * s.T + 2 * s.T * s.K) + 4 * u * s.K        # pass 1 + pass 2 (+ row read-modify-write)
        ms = fam["embedding"][0] / steps
        out["embedding"] = {"ms_per_step": ms, "algorithmic_bytes_per_step": by, "gb_per_s": by / ms / 1e6,
                            "frac_hbm_peak": by / ms / 1e6 / 8000.0}
    if vec and fam["vector"][1]:
        by = sum(2 * (4 * s.T * s.K) + 4 * s.K for s in vec)
        ms = fam["vector"][0] / steps
        out["vector"] = {"ms_per_step": ms, "algorithmic_bytes_per_step": by, "gb_per_s": by / ms / 1e6,
                         "frac_hbm_peak": by / ms / 1e6 / 8000.0}
    return out


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
    n_counted = int((tg_h >= 0).sum())
    ids, targets = torch.from_numpy(ids_h).to(dev), torch.from_numpy(tg_h).to(dev)
    ang = torch.arange(s, device=dev, dtype=torch.float64)[:, None] * (10000.0 ** (-torch.arange(64, device=dev, dtype=torch.float64) / 64.0))[None, :]
    cos, sin = torch.cos(ang).float().contiguous(), torch.sin(ang).float().contiguous()
    step = LomoFineTuneStep(dev, Bt, s, H, F, nh, n_layers, V, norm=norm, checkpoint=checkpoint, keep_handons=keep_handons,
                            overlap_norm_pass=overlap)
    run = lambda: step.step(ids, targets, n_counted, m, cos, sin, 1e-3, 65536.0)
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
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama7b_layer",
                    help="llama7b_layer (default), linear1024, llama7b_stack[:layers], llama13b_stack[:n], ...")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dgrad", action="store_true", help="skip dX (diagnostic only; not the metric)")
    ap.add_argument("--per-tensor-calls", action="store_true",
                    help="one C call per tensor instead of the whole-pass calls (same results, more launches)")
    ap.add_argument("--host-coefficient", action="store_true",
                    help="form the clipping coefficient on the host after a read-back between the passes (one "
                         "synchronisation per step) instead of on the device")
    ap.add_argument("--norm-pass", choices=["direct", "auto", "gram"], default="direct",
                    help="route of the norm pass for linear tensors in the timed steps (default: direct, the one the "
                         "metric's flop count describes)")
    ap.add_argument("--no-norm-compare", action="store_true",
                    help="skip the extra timing of pass 1 alone on each route after the timed steps")
    ap.add_argument("--train-shape", default="8x512", help="batch x sequence length of --train-step (default 8x512)")
    ap.add_argument("--train-model", default="7b", choices=sorted(TRAIN_MODELS), help="model size of --train-step (default 7b)")
    ap.add_argument("--train-policies", default="all", choices=["all", "checkpointed", "kept-activations"],
                    help="--train-step: every memory policy, only the two checkpointed ones, or only the two that keep the "
                         "activations but not the hand-ons (the largest models do not fit the others)")
    ap.add_argument("--train-step", action="store_true",
                    help="also time a whole fine-tuning step of a 7B-shaped model from token ids, with activation "
                         "checkpointing (extra keys `train_step_global_norm`, `train_step_grouped_norm`)")
    ap.add_argument("--model-chain", action="store_true",
                    help="also time the chained two-pass step through a whole 32-layer 7B-shaped model (extra key `model_chain`)")
    ap.add_argument("--chain", action="store_true",
                    help="also time the chained two-pass step through one whole 7B decoder layer (extra key `chain`)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy three times (reference for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import lomo_synth as S
    import paper_2306_09782_amd as L
    from paper_2306_09782_amd.step import LomoStep

    if not os.path.exists(L.library_path()):
        from paper_2306_09782_amd.build import build
        build(verbose=False)
    L.load_library()
    dev = torch.device("cuda:0")
    wl = S.workload(args.workload)

    tensors = []
    for spec in wl.tensors:
        t = {"kind": spec.kind, "name": spec.name, "dY": wl.dY_torch(spec, dev), "W": wl.W_torch(spec, dev)}
        if spec.kind == "embedding":
            t["ids"] = torch.from_numpy(wl.ids_np(spec)).to(dev)
        else:
            t["X"] = wl.X_torch(spec, dev)
        if spec.kind == "linear" and not args.no_dgrad:
            t["dX"] = torch.empty(spec.T, spec.K, dtype=torch.float16, device=dev)
        tensors.append(t)
    torch.cuda.synchronize()

    if args.calibrate_copy:      # known traffic: 1 GiB read + 1 GiB written per copy
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    maxH = max(s.K for s in wl.tensors)
    stepper = LomoStep(dev, max_T=wl.T, max_H=maxH, max_tensors=len(tensors), grouped=not args.per_tensor_calls)
    lr = float(np.float32(wl.lr))

    L.lomo_set_norm_algorithm(args.norm_pass)
    device_coef = not args.host_coefficient and not args.per_tensor_calls

    def one_step():
        if device_coef:      # pass 1, coefficient kernel, pass 2, scalars to pinned memory: no host wait
            stepper.run_async(tensors, lr, wl.loss_scale, wl.max_norm, wl.eps)
            return None
        return stepper.run(tensors, lr, wl.loss_scale, wl.max_norm, wl.eps)

    res = None
    for _ in range(args.warmup):
        res = one_step()
    torch.cuda.synchronize()

    L.lomo_timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if device_coef:
        res = stepper.result()
    fam = {name: L.lomo_timing_read(i) for i, name in enumerate(L.KERNEL_FAMILIES)}
    L.lomo_timing_enable(False)

    # Pass 1 alone on each route (same inputs, same result up to rounding): not part of `value`.
    norm_compare = None
    if not args.no_norm_compare:
        norm_compare = {}
        for route in ("direct", "gram", "auto"):
            L.lomo_set_norm_algorithm(route)
            for _ in range(2):
                stepper.norm_pass(tensors)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            reps = max(3, min(10, args.steps))
            for _ in range(reps):
                stepper.norm_pass(tensors)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t1) / reps * 1e3
            norm_compare[route] = {"ms": ms, "total_sqnorm": stepper.read_back(len(tensors))["total_sqnorm"]}
        L.lomo_set_norm_algorithm(args.norm_pass)

    ms_per_step = dt / args.steps * 1e3
    lin = [s for s in wl.tensors if s.kind == "linear"]
    flops_pass = sum(s.gemm_flops for s in lin)
    gemms_per_step = 2 if args.no_dgrad else 3
    step_flops = gemms_per_step * flops_pass
    tflops = step_flops / (ms_per_step * 1e-3) / 1e12

    def fam_rate(name):
        ms, n = fam[name]
        if n == 0 or ms <= 0:
            return None
        per_step_ms = ms / args.steps
        return {"tflops": flops_pass / (per_step_ms * 1e-3) / 1e12, "ms_per_step": per_step_ms,
                "launches": n, "avg_launch_ms": ms / n}

    k1 = fam_rate("wgrad_update")
    roofline = None
    if k1:
        roofline = {"kernel": "fused wgrad + SGD update (lomo_contract_dma_kernel<true, EPI_UPDATE>)", "bound": "mfma",
                    "achieved": k1["tflops"], "peak": PEAK_FP16_TFLOPS, "unit": "TFLOP/s",
                    "frac": k1["tflops"] / PEAK_FP16_TFLOPS, "traffic": profiled_traffic(wl.name),
                    "flops_per_launch": flops_pass * args.steps / k1["launches"], "avg_launch_ms": k1["avg_launch_ms"],
                    "launches_timed": k1["launches"]}

    out = {
        "metric": "fused wgrad+SGD-update TFLOP/s (two-pass LOMO step: norm pass + dgrad + fused update)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "accumulate": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "tokens": wl.T, "tensors": len(wl.tensors), "params": wl.n_params,
                   "loss_scale": wl.loss_scale, "lr": wl.lr, "max_norm": wl.max_norm,
                   "gemms_per_linear": gemms_per_step, "weights_restored_between_steps": False,
                   "calls": "per_tensor" if args.per_tensor_calls else "whole_pass", "norm_pass": args.norm_pass,
                   "coefficient": "device" if device_coef else "host"},
        "params_per_s": wl.n_params / (ms_per_step * 1e-3),
        "frac_fp16_mfma_peak_whole_step": tflops / PEAK_FP16_TFLOPS,
        "kernels": {k: fam_rate(k) for k in ("wgrad_update", "wgrad_sqnorm", "dgrad")},
        "hbm_kernels": hbm_kernels(wl, fam, args.steps),
        "grad_norm": res["norm"], "clip_coef": res["clip_coef"], "overflow": res["overflow"],
        "roofline": roofline,
    }
    if fam["gram_sqnorm"][1]:
        out["kernels"]["gram_sqnorm"] = {"ms_per_step": fam["gram_sqnorm"][0] / args.steps, "launches": fam["gram_sqnorm"][1],
                                         "avg_launch_ms": fam["gram_sqnorm"][0] / fam["gram_sqnorm"][1]}
    if norm_compare:
        out["norm_pass_alone"] = norm_compare
    if args.chain:
        del tensors
        torch.cuda.empty_cache()
        out["chain"] = chain_bench(L, torch, np, dev, max(3, args.steps // 2), 2)
    if args.model_chain:
        tensors = None
        torch.cuda.empty_cache()
        out["model_chain"] = model_chain_bench(L, torch, np, dev, 3, 1)
        torch.cuda.empty_cache()
        out["model_chain_kept_handons"] = model_chain_bench(L, torch, np, dev, 3, 1, keep_handons=True)
        torch.cuda.empty_cache()
        out["model_chain_grouped_norm"] = model_chain_bench(L, torch, np, dev, 3, 1, grouped=1)
    if args.train_step:
        tensors = None
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
        del tm
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
