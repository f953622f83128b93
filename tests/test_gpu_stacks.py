"""Full-size stacks (LLaMA 7B / 13B / 65B shapes) through the launch configuration bench.py times.

The oracle cannot materialise these steps in seconds, so the checks are:
  * every linear tensor: sampled rows x columns of the updated W and sampled rows of dX, computed
    by the oracle from the same input bits (read back from the device), to the 1-ulp / 2-ulp bar,
    for a visible step (clip forced to 1) and for the clipped step that follows it;
  * every embedding and gain tensor: element by element (they are small enough);
  * the norm: one tensor of every shape class in full against the oracle (1e-3, observed 1e-6),
    and the step total against the sum of per-tensor device norms;
  * flags: all clear on the clean run; on the run with one +inf injected exactly that tensor's
    flag, every weight byte unchanged (hash over all W), scale halved.
"""
import math
import os
import sys

import numpy as np
import pytest
import torch

import lomo_synth as S
from oracle import lomo_oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def L():
    import paper_2306_09782_amd as L
    if not os.path.exists(L.library_path()):
        from paper_2306_09782_amd.build import build
        build(verbose=False)
    L.load_library()
    return L


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def build_stack(wl):
    ts = []
    for spec in wl.tensors:
        t = {"kind": spec.kind, "name": spec.name, "spec": spec, "dY": wl.dY_torch(spec, DEV), "W": wl.W_torch(spec, DEV)}
        if spec.kind == "embedding":
            t["ids"] = torch.from_numpy(wl.ids_np(spec)).to(DEV)
        else:
            t["X"] = wl.X_torch(spec, DEV)
        if spec.kind == "linear":
            t["dX"] = torch.empty(spec.T, spec.K, dtype=torch.float16, device=DEV)
        ts.append(t)
    torch.cuda.synchronize()
    return ts


def idx(rng, n, k):
    return torch.from_numpy(np.sort(rng.choice(n, size=min(k, n), replace=False))).to(DEV)


def sample_linear(t, rng, R=8, C=256, RT=4, CX=64):
    """Device-side gathers of what the oracle needs for sampled outputs of one linear tensor."""
    sp = t["spec"]
    rows, cols = idx(rng, sp.N, R), idx(rng, sp.K, C)
    trows, xcols = idx(rng, sp.T, RT), idx(rng, sp.K, CX)
    return {
        "rows": rows, "cols": cols, "trows": trows, "xcols": xcols,
        "dY_rows": t["dY"].index_select(1, rows).cpu().numpy(),              # [T x R]
        "X_cols": t["X"].index_select(1, cols).cpu().numpy(),                # [T x C]
        "W_old": t["W"].index_select(0, rows).index_select(1, cols).cpu().numpy(),
        "dY_trows": t["dY"].index_select(0, trows).cpu().numpy(),            # [RT x N]
        "W_xcols": t["W"].index_select(1, xcols).cpu().numpy(),              # [N x CX]
    }


def check_ulps(got, want, what):
    d = O.ulp_distance_f16(got, want)
    assert d.max() <= 2, f"{what}: {d.max()} ulp"
    assert (d <= 1).mean() >= 0.999, what
    return d


def check_linear(t, smp, lr, coef, S_, what):
    G = O.linear_grad(smp["X_cols"], smp["dY_rows"])                         # [R x C], fp64
    want = O.sgd_update(smp["W_old"], G, lr, coef, S_)
    got = t["W"].index_select(0, smp["rows"]).index_select(1, smp["cols"]).cpu().numpy()
    check_ulps(got, want, f"{what} W")
    ref64 = O.input_grad_f64(smp["dY_trows"], smp["W_xcols"])
    gdx = t["dX"].index_select(0, smp["trows"]).index_select(1, smp["xcols"]).cpu().numpy()
    d = O.ulp_distance_f16(gdx, O.round_f16(ref64))
    guard = 2.0 ** -20 * (np.abs(smp["dY_trows"].astype(np.float64)) @ np.abs(smp["W_xcols"].astype(np.float64)))
    near = np.abs(gdx.astype(np.float64) - ref64) <= guard
    assert ((d <= 2) | near).all() and ((d <= 1) | near).mean() >= 0.999, f"{what} dX"
    return (want.view(np.uint16) != smp["W_old"].view(np.uint16)), (got.view(np.uint16) != smp["W_old"].view(np.uint16))


def small_tensor_host(t):
    return {k: (v.cpu().numpy() if torch.is_tensor(v) else v) for k, v in t.items() if k in ("kind", "X", "dY", "W", "ids")}


def weights_hash(ts):
    h = torch.zeros(1, dtype=torch.int64, device=DEV)
    for t in ts:
        w = t["W"].view(torch.int16).to(torch.int64).view(-1)
        h += (w * (torch.arange(w.numel(), device=DEV, dtype=torch.int64) % 1000003 + 1)).sum()
    return int(h.item())


STACKS = [("llama7b_stack", None), ("llama13b_stack", None), ("llama65b_stack", None)]


@pytest.mark.parametrize("name,layers", STACKS)
def test_stack_step(L, name, layers):
    from paper_2306_09782_amd.step import LomoStep
    import gc
    gc.collect()
    torch.cuda.empty_cache()          # blocks cached from the previous stack count as used otherwise
    free, total = torch.cuda.mem_get_info()
    wl = S.workload(name if layers is None else f"{name}:{layers}")
    need = sum(2 * (s.n_params + s.T * (s.K + (s.N if s.kind == "linear" else s.K)) + (s.T * s.K if s.kind == "linear" else 0))
               for s in wl.tensors)
    if need > 0.92 * free:
        pytest.skip(f"{name} needs {need / 2**30:.0f} GiB of device memory, {free / 2**30:.0f} GiB free")
    say(f"[{name}] generating {wl.n_params / 1e9:.2f} G parameters + activations ({need / 2**30:.0f} GiB)")
    ts = build_stack(wl)
    stepper = LomoStep(DEV, max_T=wl.T, max_H=max(s.K for s in wl.tensors), max_tensors=len(ts))
    lr = float(np.float32(wl.lr))
    Sc = wl.loss_scale
    rng = np.random.default_rng(0)

    # ---- norm: per-tensor device norms; one tensor per shape class in full against the oracle
    say(f"[{name}] per-tensor norms")
    accs = torch.zeros(len(ts), dtype=torch.float64, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    for i, t in enumerate(ts):
        a = accs[i:i + 1]
        if t["kind"] == "linear":
            L.lomo_wgrad_sqnorm(t["X"], t["dY"], a, flag)
        elif t["kind"] == "embedding":
            L.lomo_embedding_sqnorm(t["ids"], t["dY"], t["W"].shape[0], stepper.ws, a, flag)
        else:
            L.lomo_vector_sqnorm(t["X"], t["dY"], stepper.ws, a, flag)
    per = accs.cpu().numpy()
    assert int(flag.item()) == 0
    seen = set()
    for i, t in enumerate(ts):
        sp = t["spec"]
        cls = (sp.kind, sp.N, sp.K)
        if sp.kind == "linear":
            if cls in seen:
                continue
            seen.add(cls)
            want = O.sqnorm(O.linear_grad(t["X"].cpu().numpy(), t["dY"].cpu().numpy()))
        else:
            want = O.sqnorm(O.tensor_grad(small_tensor_host(t)))
        assert abs(per[i] / want - 1) < 1e-3, (t["name"], per[i], want)
        assert abs(per[i] / want - 1) < 2e-5, (t["name"], per[i], want)
    say(f"[{name}] {len(seen)} linear shape classes and all row/vector tensors match the oracle norm")

    # ---- visible step (clip forced to 1), then the clipped step of the workload, sampled
    sig = wl.tensors[0].sigma_dy
    lr_vis = float(np.float32(30 * 2.0 ** -16 / (math.sqrt(wl.T) * sig)))
    for label, step_lr, override in (("visible", lr_vis, 1.0), ("clipped", lr, None)):
        say(f"[{name}] sampling inputs for the {label} step")
        samples = [sample_linear(t, rng) if t["kind"] == "linear" else small_tensor_host(t) for t in ts]
        res = stepper.run(ts, step_lr, Sc, wl.max_norm, wl.eps, clip_override=override)
        torch.cuda.synchronize()
        assert res["overflow"] is False and not any(res["flags"])
        assert abs(res["total_sqnorm"] / float(per.sum()) - 1) < 1e-6
        coef = res["clip_coef"]
        if override is None:
            assert abs(coef / L.lomo_clip_coef(float(per.sum()), Sc, wl.max_norm, wl.eps) - 1) < 1e-6
            assert coef == pytest.approx(O.clip_coef(O.grad_norm(float(per.sum()), Sc), wl.max_norm, wl.eps), rel=1e-12)
        changed_o = changed_g = total_s = 0
        for t, smp in zip(ts, samples):
            if t["kind"] == "linear":
                co, cg = check_linear(t, smp, step_lr, coef, Sc, f"{name}/{t['name']} {label}")
                changed_o += int(co.sum()); changed_g += int((co != cg).sum()); total_s += co.size
            else:
                G = O.tensor_grad(smp)
                want = O.sgd_update(smp["W"], G, step_lr, coef, Sc)
                check_ulps(t["W"].cpu().numpy(), want, f"{name}/{t['name']} {label}")
        if label == "visible":
            assert changed_o / total_s > 0.9 and changed_g / total_s < 1e-3
        say(f"[{name}] {label} step ok: norm {res['norm']:.5g}, clip {coef:.4g}, "
            f"{changed_o}/{total_s} sampled weights changed")

    # ---- overflow run (the 7B stack carries the injection point)
    if wl.inject_inf is not None:
        tname, r, c = wl.inject_inf
        victim = next(t for t in ts if t["name"] == tname)
        before = weights_hash(ts)
        old = victim["dY"][r, c].clone()
        victim["dY"][r, c] = float("inf")
        res = stepper.run(ts, lr, Sc, wl.max_norm, wl.eps)
        torch.cuda.synchronize()
        assert res["overflow"] is True
        assert [t["name"] for t, f in zip(ts, res["flags"]) if f] == [tname]
        assert weights_hash(ts) == before
        assert L.lomo_scaler_step(Sc, 5, 1000, True) == (Sc / 2, 0) == O.scaler_step(Sc, 5, 1000, True)
        # pass 2 launched anyway (asynchronous use): the device flag keeps every W untouched
        stepper.update_pass(ts, lr, 1.0 / Sc, 1.0)
        torch.cuda.synchronize()
        assert weights_hash(ts) == before
        victim["dY"][r, c] = old
        res = stepper.run(ts, lr, Sc / 2, wl.max_norm, wl.eps)   # the retried step is clean
        assert res["overflow"] is False
        say(f"[{name}] overflow run ok: flag on {tname} only, weights untouched, scale {Sc} -> {Sc / 2}")
