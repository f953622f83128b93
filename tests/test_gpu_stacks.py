"""Full-size stacks (LLaMA 7B / 13B / 65B shapes) through the launch configuration bench.py times.

The oracle cannot materialise these steps in seconds, so the checks are:
  * every linear tensor, updated W: the kernels work on 256 x 256 output tiles, so the sample takes at least one
    row of W out of EVERY band of 256 rows and, in the visible step (clip forced to 1), ALL columns of those rows
    -- at least 64 full rows per tensor, every output tile contributes 256 checked elements per sampled row.
    In the clipped step that follows it is 8 columns out of every band of 256 columns, again in every band of
    rows: every tile contributes at least 8 checked elements.  The oracle computes those elements from the
    device's own input bits (read back) to the 1-ulp / 2-ulp bar;
  * every linear tensor, dX: one token row out of every band of 256 tokens x 8 columns out of every band of 256
    columns (every 256 x 256 tile of dX), same bar with the cancellation guard;
  * every embedding and gain tensor: element by element (they are small enough);
  * the norm: one tensor of every shape class in full against the oracle (1e-3, observed 1e-6), and the step
    total against the sum of per-tensor device norms;
  * flags: all clear on the clean run; on the run with one +inf injected exactly that tensor's flag, every weight
    byte unchanged (hash over all W), scale halved;
  * memory: what a step allocates beyond its inputs and outputs (workspace, accumulator, flags, scalars) stays
    below the largest weight tensor of one decoder layer (the paper's table 1 keeps one tensor's gradient; here
    not even that is needed).

The 7B and 13B stacks keep every tensor's X / dY / dX resident.  The 65B stack is run as its description says:
activations regenerated layer by layer from the seed, in both passes, into one layer's buffers; the oracle reads
back the bits of the layer that is in place.
"""
import gc
import math
import os
import sys
import time

import numpy as np
import pytest
import torch

import lomo_synth as S
from oracle import lomo_oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TILE = 256


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


def one_per_band(rng, n, extra_to=0):
    """One index out of every band of TILE consecutive ones (the last band may be short), topped up with further
    distinct indices to at least `extra_to`."""
    picks = [int(rng.integers(b, min(b + TILE, n))) for b in range(0, n, TILE)]
    if extra_to > len(picks):
        rest = np.setdiff1d(np.arange(n), np.asarray(picks))
        picks += rng.choice(rest, size=min(extra_to - len(picks), rest.size), replace=False).tolist()
    return np.sort(np.asarray(picks, dtype=np.int64))


def some_per_band(rng, n, per):
    picks = []
    for b in range(0, n, TILE):
        width = min(TILE, n - b)
        picks += (b + rng.choice(width, size=min(per, width), replace=False)).tolist()
    return np.sort(np.asarray(picks, dtype=np.int64))


class LinearSample:
    """Which elements of one linear tensor are checked, and the old weights they need (taken before the step)."""

    def __init__(self, t, rng, full_rows: bool):
        sp = t["spec"]
        self.full = full_rows
        self.rows = torch.from_numpy(one_per_band(rng, sp.N, 64 if full_rows else 0)).to(DEV)
        self.cols = None if full_rows else torch.from_numpy(some_per_band(rng, sp.K, 8)).to(DEV)
        self.trows = torch.from_numpy(one_per_band(rng, sp.T)).to(DEV)
        self.xcols = torch.from_numpy(some_per_band(rng, sp.K, 8)).to(DEV)
        assert self.rows.numel() >= (64 if full_rows else 1) and len(set((self.rows // TILE).tolist())) == -(-sp.N // TILE)
        assert len(set((self.xcols // TILE).tolist())) == -(-sp.K // TILE) and len(set((self.trows // TILE).tolist())) == -(-sp.T // TILE)
        W = t["W"]
        w_rows = W.index_select(0, self.rows)
        self.W_old = (w_rows if full_rows else w_rows.index_select(1, self.cols)).cpu().numpy()
        self.W_xcols = W.index_select(1, self.xcols).cpu().numpy()            # [N x CX], pre-update

    def check(self, t, lr, coef, S_, what):
        """Reads the inputs that are in place on the device now, and the outputs; returns (changed per the oracle,
        changed on the device) over the sampled weights."""
        X = t["X"] if self.full else t["X"].index_select(1, self.cols)
        G = O.linear_grad(X.cpu().numpy(), t["dY"].index_select(1, self.rows).cpu().numpy())      # [R x C], fp64
        want = O.sgd_update(self.W_old, G, lr, coef, S_)
        got = t["W"].index_select(0, self.rows)
        got = (got if self.full else got.index_select(1, self.cols)).cpu().numpy()
        d = O.ulp_distance_f16(got, want)
        assert d.max() <= 2, f"{what} W: {d.max()} ulp"
        assert (d <= 1).mean() >= 0.999, f"{what} W"
        dY_t = t["dY"].index_select(0, self.trows).cpu().numpy()
        ref64 = O.input_grad_f64(dY_t, self.W_xcols)
        gdx = t["dX"].index_select(0, self.trows).index_select(1, self.xcols).cpu().numpy()
        d = O.ulp_distance_f16(gdx, O.round_f16(ref64))
        guard = 2.0 ** -20 * (np.abs(dY_t.astype(np.float64)) @ np.abs(self.W_xcols.astype(np.float64)))
        near = np.abs(gdx.astype(np.float64) - ref64) <= guard
        assert ((d <= 2) | near).all() and ((d <= 1) | near).mean() >= 0.999, f"{what} dX"
        old = self.W_old.view(np.uint16)
        return (want.view(np.uint16) != old), (got.view(np.uint16) != old)


def check_ulps(got, want, what):
    d = O.ulp_distance_f16(got, want)
    assert d.max() <= 2, f"{what}: {d.max()} ulp"
    assert (d <= 1).mean() >= 0.999, what
    return d


def small_tensor_host(t):
    return {k: (v.cpu().numpy() if torch.is_tensor(v) else v) for k, v in t.items() if k in ("kind", "X", "dY", "W", "ids")}


def weights_hash(ts):
    h = torch.zeros(1, dtype=torch.int64, device=DEV)
    for t in ts:
        w = t["W"].view(torch.int16).to(torch.int64).view(-1)
        h += (w * (torch.arange(w.numel(), device=DEV, dtype=torch.int64) % 1000003 + 1)).sum()
    return int(h.item())


def largest_layer_weight_bytes(wl):
    return 2 * max(s.n_params for s in wl.tensors if s.kind == "linear" and s.name != "lm_head")


def visible_lr(wl):
    sig = wl.tensors[0].sigma_dy
    return float(np.float32(30 * 2.0 ** -16 / (math.sqrt(wl.T) * sig)))


def fresh_device(name, need):
    gc.collect()
    torch.cuda.empty_cache()          # blocks cached from the previous stack count as used otherwise
    free, total = torch.cuda.mem_get_info()
    assert need <= 0.92 * free, (f"{name} needs {need / 2**30:.0f} GiB of device memory and {free / 2**30:.0f} GiB of "
                                 f"{total / 2**30:.0f} GiB are free: an MI355X (288 GB) holds every workload")


RESIDENT = ["llama7b_stack", "llama13b_stack"]


@pytest.mark.parametrize("name", RESIDENT)
def test_stack_step(L, name):
    from paper_2306_09782_amd.step import LomoStep
    wl = S.workload(name)
    need = sum(2 * (s.n_params + s.T * (s.K + (s.N if s.kind == "linear" else s.K)) + (s.T * s.K if s.kind == "linear" else 0))
               for s in wl.tensors)
    fresh_device(name, need)
    say(f"[{name}] generating {wl.n_params / 1e9:.2f} G parameters + activations ({need / 2**30:.0f} GiB)")
    ts = build_stack(wl)
    base_bytes = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    stepper = LomoStep(DEV, max_T=wl.T, max_H=max(s.K for s in wl.tensors if s.kind != "linear"), max_tensors=len(ts))
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

    # ---- visible step (clip forced to 1; full rows), then the clipped step of the workload (column samples)
    for label, step_lr, override in (("visible", visible_lr(wl), 1.0), ("clipped", lr, None)):
        t0 = time.time()
        samples = [LinearSample(t, rng, label == "visible") if t["kind"] == "linear" else small_tensor_host(t) for t in ts]
        res = stepper.run(ts, step_lr, Sc, wl.max_norm, wl.eps, clip_override=override)
        torch.cuda.synchronize()
        assert res["overflow"] is False and not any(res["flags"])
        assert abs(res["total_sqnorm"] / float(per.sum()) - 1) < 1e-6
        coef = res["clip_coef"]
        if override is None:
            assert abs(coef / L.lomo_clip_coef(float(per.sum()), Sc, wl.max_norm, wl.eps) - 1) < 1e-6
            assert coef == pytest.approx(O.clip_coef(O.grad_norm(float(per.sum()), Sc), wl.max_norm, wl.eps), rel=1e-12)
        changed_o = changed_g = total_s = 0
        for k, (t, smp) in enumerate(zip(ts, samples)):
            if t["kind"] == "linear":
                co, cg = smp.check(t, step_lr, coef, Sc, f"{name}/{t['name']} {label}")
                changed_o += int(co.sum()); changed_g += int((co != cg).sum()); total_s += co.size
            else:
                G = O.tensor_grad(smp)
                want = O.sgd_update(smp["W"], G, step_lr, coef, Sc)
                check_ulps(t["W"].cpu().numpy(), want, f"{name}/{t['name']} {label}")
            if k % 64 == 63:
                say(f"[{name}] {label}: {k + 1}/{len(ts)} tensors checked")
        if label == "visible":
            assert changed_o / total_s > 0.9 and changed_g / total_s < 1e-3
        say(f"[{name}] {label} step ok in {time.time() - t0:.0f} s: norm {res['norm']:.5g}, clip {coef:.4g}, "
            f"{changed_o}/{total_s} sampled weights changed")

    # ---- memory: everything the steps allocated beyond inputs and outputs (samples are host-side or freed)
    extra = torch.cuda.max_memory_allocated() - base_bytes
    bound = largest_layer_weight_bytes(wl)
    say(f"[{name}] peak extra device memory {extra / 2**20:.1f} MiB (bound: largest layer tensor {bound / 2**20:.1f} MiB)")
    assert stepper.ws.numel() + 8 + 4 * stepper.flags.numel() + 32 <= bound
    assert extra <= bound + (64 << 20), "test-side gathers are included in the peak: 64 MiB of slack for them"

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


def test_measured_extra_memory_of_a_step(L):
    """Nothing but the step itself between the two memory readings: the extra device memory of the 7B-layer step is
    its workspace and a few scalars, far below one weight tensor."""
    from paper_2306_09782_amd.step import LomoStep
    wl = S.workload("llama7b_stack:2")
    ts = build_stack(wl)
    torch.cuda.synchronize()
    base = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    stepper = LomoStep(DEV, max_T=256, max_H=256, max_tensors=len(ts))
    stepper.run_async(ts, float(np.float32(wl.lr)), wl.loss_scale, wl.max_norm, wl.eps)
    torch.cuda.synchronize()
    extra = torch.cuda.max_memory_allocated() - base
    assert not stepper.result()["overflow"]
    assert 0 < extra <= largest_layer_weight_bytes(wl), (extra, largest_layer_weight_bytes(wl))
    # and no gradient-sized buffer: the workspace is the embedding's partial rows plus four gain vectors' partial sums
    assert extra < 16 << 20, extra


def test_stack_step_with_regenerated_activations(L):
    """The 65B-shaped stack as its description has it: 130 GB of parameters resident, every layer's X / dY
    regenerated from the seed into one layer's buffers just before that layer's turn, in both passes.  A visible
    step (every sampled weight moves), checked layer by layer while that layer's inputs are in place."""
    from paper_2306_09782_amd.step import LomoStreamedStep
    name = "llama65b_stack"
    wl = S.workload(name)
    layer = [s for s in wl.tensors if s.layer == 0]
    per_layer_io = sum(2 * (s.T * (s.K + (s.N if s.kind == "linear" else s.K)) + (s.T * s.K if s.kind == "linear" else 0)) for s in layer)
    need = 2 * wl.n_params + 3 * per_layer_io
    fresh_device(name, need)
    say(f"[{name}] generating {wl.n_params / 1e9:.2f} G parameters; one layer's activations: {per_layer_io / 2**30:.2f} GiB")
    stack = S.StreamedStack(wl, DEV)
    torch.cuda.synchronize()
    base_bytes = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    stepper = LomoStreamedStep(DEV, max_tensors=len(wl.tensors) + len(stack.groups) + 1)
    stepper.bind(stack.groups)
    ws_bytes = stepper.ws.numel()
    Sc = wl.loss_scale
    rng = np.random.default_rng(5)
    n_groups = len(stack.groups)
    assert n_groups == 82 and sum(len(g) for g in stack.groups) == len(wl.tensors)

    # The oracle needs the step's coefficient before it can check a layer, and the layer's inputs are gone once the
    # next layer is prepared.  So the visible step runs with a coefficient of one: max_norm is set above the norm.
    lr = visible_lr(wl)
    samples, seen_pass, stats = {}, {}, {"changed_o": 0, "changed_g": 0, "total": 0, "layers": 0}
    t0 = time.time()
    accs = torch.zeros(len(wl.tensors), dtype=torch.float64, device=DEV)      # per-tensor device norms, in list order
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    first = {}
    for gi, grp in enumerate(stack.groups):
        for ti, t in enumerate(grp):
            first.setdefault((t["kind"], t["spec"].N, t["spec"].K), (gi, ti))     # one tensor per shape class
    offset = np.cumsum([0] + [len(grp) for grp in stack.groups])

    def prepare(g):
        stack.prepare(g)
        if g not in seen_pass:                      # pass 1: the weights are still the old ones
            seen_pass[g] = 1
            samples[g] = [LinearSample(t, rng, True) if t["kind"] == "linear" else
                          {"kind": t["kind"], "W": t["W"].cpu().numpy()} for t in stack.groups[g]]

    def after_update(g):
        torch.cuda.synchronize()
        for ti, (t, smp) in enumerate(zip(stack.groups[g], samples.pop(g))):
            what = f"{name}/{t['name']} visible"
            a = accs[offset[g] + ti:offset[g] + ti + 1]
            if t["kind"] == "linear":
                L.lomo_wgrad_sqnorm(t["X"], t["dY"], a, flag)
            elif t["kind"] == "embedding":
                L.lomo_embedding_sqnorm(t["ids"], t["dY"], t["W"].shape[0], stepper.ws, a, flag)
            else:
                L.lomo_vector_sqnorm(t["X"], t["dY"], stepper.ws, a, flag)
            if first[(t["kind"], t["spec"].N, t["spec"].K)] == (g, ti):       # in full against the oracle
                want = O.sqnorm(O.linear_grad(t["X"].cpu().numpy(), t["dY"].cpu().numpy())) if t["kind"] == "linear" \
                    else O.sqnorm(O.tensor_grad(small_tensor_host(t)))
                got = float(a.item())
                assert abs(got / want - 1) < 1e-3 and abs(got / want - 1) < 2e-5, (t["name"], got, want)
            if t["kind"] == "linear":
                co, cg = smp.check(t, lr, 1.0, Sc, what)
                stats["changed_o"] += int(co.sum()); stats["changed_g"] += int((co != cg).sum()); stats["total"] += co.size
            else:
                host = small_tensor_host(t)
                host["W"] = smp["W"]
                check_ulps(t["W"].cpu().numpy(), O.sgd_update(smp["W"], O.tensor_grad(host), lr, 1.0, Sc), what)
        stats["layers"] += 1
        if stats["layers"] % 10 == 0:
            say(f"[{name}] {stats['layers']}/{n_groups} groups checked ({time.time() - t0:.0f} s)")

    stepper.run_async(prepare, lr, Sc, 1e30, wl.eps, after_update=after_update)
    torch.cuda.synchronize()
    res = stepper.result()
    assert res["overflow"] is False and not any(any(f) for f in res["flags"]) and res["clip_coef"] == 1.0
    assert stats["layers"] == n_groups and not samples
    assert stats["changed_o"] / stats["total"] > 0.9 and stats["changed_g"] / stats["total"] < 1e-3
    # the step's norm: one tensor of every shape class was compared with the oracle in full above; the total against
    # the sum of the per-tensor device norms
    per = accs.cpu().numpy()
    assert int(flag.item()) == 0 and (per > 0).all()
    assert abs((res["norm"] * Sc) ** 2 / float(per.sum()) - 1) < 1e-6
    extra = torch.cuda.max_memory_allocated() - base_bytes
    bound = largest_layer_weight_bytes(wl)
    say(f"[{name}] visible step ok in {time.time() - t0:.0f} s: norm {res['norm']:.5g}; workspace {ws_bytes / 2**20:.1f} MiB, "
        f"peak extra {extra / 2**20:.1f} MiB, bound {bound / 2**20:.1f} MiB; {stats['changed_o']}/{stats['total']} sampled weights changed")
    assert ws_bytes <= bound and extra <= bound + (256 << 20), "test-side gathers (one tensor's X on its way to the host) are in the peak"

    # ---- the clipped step of the workload on the same stack: coefficient from the device, flags clear, finite norm
    stepper.run_async(stack.prepare, float(np.float32(wl.lr)), Sc, wl.max_norm, wl.eps)
    torch.cuda.synchronize()
    res2 = stepper.result()
    assert res2["overflow"] is False and 0 < res2["clip_coef"] < 1
    assert res2["clip_coef"] == pytest.approx(O.clip_coef(res2["norm"], wl.max_norm, wl.eps), rel=1e-9)
    assert abs(res2["norm"] / res["norm"] - 1) < 1e-3          # same inputs, weights moved by a visible step only
    say(f"[{name}] clipped step ok: norm {res2['norm']:.5g}, clip {res2['clip_coef']:.4g}")


def test_streamed_step_equals_resident_step(L):
    """Regenerating the activations group by group changes nothing: on a two-layer 65B-shaped stack the streamed
    step leaves every weight bit-identical to the resident whole-pass step, and the norms agree (the accumulator's
    atomic adds come in another order)."""
    from paper_2306_09782_amd.step import LomoStep, LomoStreamedStep
    wl = S.workload("llama65b_stack:2")
    lr = visible_lr(wl)
    ts = build_stack(wl)
    stepper = LomoStep(DEV, max_T=256, max_H=256, max_tensors=len(ts))
    stepper.run_async(ts, lr, wl.loss_scale, 1e30, wl.eps)
    torch.cuda.synchronize()
    want = stepper.result()
    stack = S.StreamedStack(wl, DEV)
    st2 = LomoStreamedStep(DEV, max_tensors=len(ts) + 8)
    st2.bind(stack.groups)
    st2.run_async(stack.prepare, lr, wl.loss_scale, 1e30, wl.eps)
    torch.cuda.synchronize()
    got = st2.result()
    assert got["overflow"] is False and want["overflow"] is False
    assert abs(got["norm"] / want["norm"] - 1) < 1e-9 and got["clip_coef"] == want["clip_coef"] == 1.0
    flat = [t for g in stack.groups for t in g]
    assert [t["name"] for t in flat] == [t["name"] for t in ts]
    moved = 0
    for a, b in zip(flat, ts):
        assert torch.equal(a["W"].view(torch.int16), b["W"].view(torch.int16)), a["name"]
        moved += int((a["W"].view(torch.int16) != wl.W_torch(a["spec"], DEV).view(torch.int16)).sum())
    assert moved > 0.9 * wl.n_params * 0.5
