"""Whole two-pass steps of the named workloads on the GPU against the materialising oracle.

linear1024 and llama7b_layer are checked element by element on every tensor, in the launch
configuration bench.py times (LomoStep.run).  Inputs come from the counter-based generators
(device twin; the bits the oracle sees are read back from the device).
"""
import math
import os

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


def _device_tensors(wl):
    out = []
    for spec in wl.tensors:
        t = {"kind": spec.kind, "name": spec.name, "dY": wl.dY_torch(spec, DEV), "W": wl.W_torch(spec, DEV)}
        if spec.kind == "embedding":
            t["ids"] = torch.from_numpy(wl.ids_np(spec)).to(DEV)
        else:
            t["X"] = wl.X_torch(spec, DEV)
        if spec.kind == "linear":
            t["dX"] = torch.empty(spec.T, spec.K, dtype=torch.float16, device=DEV)
        out.append(t)
    return out


def _host(t):
    return {k: (v.cpu().numpy() if torch.is_tensor(v) else v) for k, v in t.items() if k != "dX"}


def _check_ulps(got, want, what):
    d = O.ulp_distance_f16(got, want)
    assert d.max() <= 2, f"{what}: {d.max()} ulp"
    assert (d <= 1).mean() >= 0.999, what
    return float((d == 0).mean())


def _check_dx(got, dY, W, what):
    """dX within 1 ulp (2 at most), or within 2^-20 * sum_n |dY||W| where the sum cancels."""
    ref64 = O.input_grad_f64(dY, W)
    d = O.ulp_distance_f16(got, O.round_f16(ref64))
    guard = 2.0 ** -20 * (np.abs(dY.astype(np.float64)) @ np.abs(W.astype(np.float64)))
    near = np.abs(got.astype(np.float64) - ref64) <= guard
    assert ((d <= 2) | near).all(), f"{what}: dX off by {d.max()} ulp"
    assert ((d <= 1) | near).mean() >= 0.999, what


@pytest.mark.parametrize("grouped", [True, False], ids=["grouped", "per_tensor"])
@pytest.mark.parametrize("name", ["linear1024", "llama7b_layer"])
def test_two_pass_step_matches_oracle(L, name, grouped):
    from paper_2306_09782_amd.step import LomoStep
    wl = S.workload(name)
    gpu = _device_tensors(wl)
    cpu = [_host(t) for t in gpu]
    if name == "linear1024":     # the CPU generator yields the same bits
        np.testing.assert_array_equal(cpu[0]["X"].view(np.uint16), wl.X_np(wl.tensors[0]).view(np.uint16))
    lr = float(np.float32(wl.lr))
    stepper = LomoStep(DEV, max_T=wl.T, max_H=max(s.K for s in wl.tensors), max_tensors=len(gpu), grouped=grouped)

    # oracle, materialised: every gradient of the step is held at once
    grads = [O.tensor_grad(t) for t in cpu]
    flags = [O.has_overflow(g) for g in grads]
    total = math.fsum(O.sqnorm(g) for g in grads)
    norm = O.grad_norm(total, wl.loss_scale)
    coef = O.clip_coef(norm, wl.max_norm, wl.eps)

    # 1) the step as the workload states it (clipped: most updates are below one ulp)
    res = stepper.run(gpu, lr, wl.loss_scale, wl.max_norm, wl.eps)
    assert res["flags"] == flags and res["overflow"] is False
    assert abs(res["norm"] / norm - 1) < 1e-3
    assert abs(res["norm"] / norm - 1) < 1e-5           # what the fp32/fp64 accumulation really gives
    assert abs(res["clip_coef"] / coef - 1) < 1e-3
    for g, t, G in zip(gpu, cpu, grads):
        want = O.sgd_update(t["W"], G, lr, res["clip_coef"], wl.loss_scale)
        _check_ulps(g["W"].cpu().numpy(), want, f"{name}/{g['name']} clipped")
        _check_dx(g["dX"].cpu().numpy(), t["dY"], t["W"], g["name"])

    # 2) a visible step from the same start: clip forced to 1, typical update about 30 ulp
    for g, t in zip(gpu, cpu):
        g["W"].copy_(torch.from_numpy(t["W"]))
    sig = wl.tensors[0].sigma_dy
    lr_vis = float(np.float32(30 * 2.0 ** -16 / (math.sqrt(wl.T) * sig)))
    stepper.run(gpu, lr_vis, wl.loss_scale, wl.max_norm, wl.eps, clip_override=1.0)
    for g, t, G in zip(gpu, cpu, grads):
        want = O.sgd_update(t["W"], G, lr_vis, 1.0, wl.loss_scale)
        got = g["W"].cpu().numpy()
        exact = _check_ulps(got, want, f"{name}/{g['name']} visible")
        assert exact > 0.98
        changed_o = want.view(np.uint16) != t["W"].view(np.uint16)
        changed_g = got.view(np.uint16) != t["W"].view(np.uint16)
        assert changed_o.mean() > 0.9 and (changed_o != changed_g).mean() < 1e-3


@pytest.mark.parametrize("name", ["linear1024", "llama7b_layer"])
def test_device_coefficient_step_matches_oracle(L, name):
    """Norm pass, coefficient kernel and update pass queued without a host wait (LomoStep.run_async)."""
    from paper_2306_09782_amd.step import LomoStep
    wl = S.workload(name)
    gpu = _device_tensors(wl)
    cpu = [_host(t) for t in gpu]
    stepper = LomoStep(DEV, max_T=wl.T, max_H=max(s.K for s in wl.tensors), max_tensors=len(gpu))
    grads = [O.tensor_grad(t) for t in cpu]
    total = math.fsum(O.sqnorm(g) for g in grads)
    norm = O.grad_norm(total, wl.loss_scale)
    coef = O.clip_coef(norm, wl.max_norm, wl.eps)
    sig = wl.tensors[0].sigma_dy
    lr_vis = 30 * 2.0 ** -16 / (math.sqrt(wl.T) * sig)

    # clipped step made visible: lr such that lr * coef is the visible step size
    lr = float(np.float32(lr_vis / coef))
    stepper.run_async(gpu, lr, wl.loss_scale, wl.max_norm, wl.eps)
    torch.cuda.synchronize()
    res = stepper.result()
    assert res["overflow"] is False
    assert abs(res["norm"] / norm - 1) < 1e-5 and abs(res["clip_coef"] / coef - 1) < 1e-5
    assert abs(res["step"] / (lr * coef / wl.loss_scale) - 1) < 1e-5
    assert res["clip_coef"] == pytest.approx(L.lomo_clip_coef(stepper.read_back(len(gpu))["total_sqnorm"], wl.loss_scale,
                                                              wl.max_norm, wl.eps), rel=1e-14)
    for g, t, G in zip(gpu, cpu, grads):
        want = O.sgd_update(t["W"], G, lr, res["clip_coef"], wl.loss_scale)
        got = g["W"].cpu().numpy()
        exact = _check_ulps(got, want, f"{name}/{g['name']} device coefficient")
        assert exact > 0.98
        changed_o = want.view(np.uint16) != t["W"].view(np.uint16)
        assert changed_o.mean() > 0.9 and (changed_o != (got.view(np.uint16) != t["W"].view(np.uint16))).mean() < 1e-3
        _check_dx(g["dX"].cpu().numpy(), t["dY"], t["W"], g["name"])

    # overflow: pass 2 is queued anyway and must leave every weight alone; the scalars say why
    before = [g["W"].clone() for g in gpu]
    gpu[-1]["dY"][0, 0] = float("inf")
    stepper.run_async(gpu, lr, wl.loss_scale, wl.max_norm, wl.eps)
    torch.cuda.synchronize()
    res = stepper.result()
    assert res["overflow"] is True and res["clip_coef"] == 0.0 and res["step"] == 0.0
    for g, b in zip(gpu, before):
        assert torch.equal(g["W"].view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("mode", ["host_coefficient", "device_coefficient"])
def test_step_on_a_stream_that_is_not_current(L, mode):
    """Every part of the step -- zeroing the accumulator and the flags, the kernels, the read-back -- goes to the
    stream that is passed in.  The current stream is kept busy meanwhile and the accumulator starts dirty, so a
    fill or a read-back that went to the current stream would come too late (wrong norm) or too early."""
    from paper_2306_09782_amd.step import LomoStep
    T, V, H, N = 320, 700, 264, 392
    Sc = 1024.0
    mk = lambda i, shape, sig, sc=1.0: S.normal_f16_np(S.tensor_key(3, 0, i, 0), shape, S.normal_mult(sig, sc))
    cpu = [
        dict(kind="linear", X=mk(0, (T, H), 1.0), dY=mk(1, (T, N), 0.01, Sc), W=mk(2, (N, H), 0.02)),
        dict(kind="vector", X=mk(3, (T, H), 1.0), dY=mk(4, (T, H), 0.01, Sc), W=np.ones(H, np.float16)),
        dict(kind="embedding", ids=S.zipf_ids(3, T, V), dY=mk(5, (T, H), 0.01, Sc), W=mk(6, (V, H), 0.02)),
    ]
    gpu = [{k: (torch.from_numpy(v).to(DEV) if isinstance(v, np.ndarray) else v) for k, v in t.items()} for t in cpu]
    gpu[0]["dX"] = torch.empty(T, H, dtype=torch.float16, device=DEV)
    ref = O.step_materialised(cpu, 4.0, Sc)
    stepper = LomoStep(DEV, max_T=T, max_H=H)
    stepper.acc.fill_(1e30)                       # stale contents from "a previous step"
    stepper.flags.fill_(1)
    torch.cuda.synchronize()
    side = torch.cuda.Stream(DEV)                 # default priority
    busy_a = torch.randn(4096, 4096, device=DEV)
    for _ in range(20):                           # tens of milliseconds of work queued on the current stream
        busy_a = busy_a @ busy_a * 1e-3
    if mode == "host_coefficient":
        res = stepper.run(gpu, 4.0, Sc, stream=side)
    else:
        stepper.run_async(gpu, 4.0, Sc, stream=side)
        side.synchronize()
        res = stepper.result()
        res["flags"] = stepper.read_back(len(gpu), side)["flags"]
    side.synchronize()
    assert res["overflow"] is False and res["flags"] == ref["flags"]
    assert abs(res["norm"] / ref["norm"] - 1) < 1e-5
    for g, t, w in zip(gpu, cpu, ref["W"]):
        got = g["W"].cpu().numpy()
        _check_ulps(got, w, t["kind"])
        assert (got.view(np.uint16) != t["W"].view(np.uint16)).any()
    _check_dx(gpu[0]["dX"].cpu().numpy(), cpu[0]["dY"], cpu[0]["W"], "dX")
    torch.cuda.synchronize()


def test_captured_step_replays_like_the_eager_step(L):
    """The whole step recorded as a HIP graph: every replay (three of them, with eager steps and synchronisations in
    between) must leave the weights the eager step leaves from the same start, and report the same scalars."""
    from paper_2306_09782_amd.step import LomoStep, CapturedStep
    T, V, H, N = 320, 700, 264, 392
    Sc = 1024.0
    mk = lambda i, shape, sig, sc=1.0: S.normal_f16_np(S.tensor_key(4, 0, i, 0), shape, S.normal_mult(sig, sc))
    cpu = [
        dict(kind="linear", X=mk(0, (T, H), 1.0), dY=mk(1, (T, N), 0.01, Sc), W=mk(2, (N, H), 0.02)),
        dict(kind="linear", X=mk(7, (512, 1024), 1.0), dY=mk(8, (512, 1024), 0.01, Sc), W=mk(9, (1024, 1024), 0.02)),
        dict(kind="vector", X=mk(3, (T, H), 1.0), dY=mk(4, (T, H), 0.01, Sc), W=np.ones(H, np.float16)),
        dict(kind="embedding", ids=S.zipf_ids(4, T, V), dY=mk(5, (T, H), 0.01, Sc), W=mk(6, (V, H), 0.02)),
    ]
    lr = 4.0
    ref = O.step_materialised(cpu, lr, Sc)
    gpu = [{k: (torch.from_numpy(v).to(DEV) if isinstance(v, np.ndarray) else v) for k, v in t.items()} for t in cpu]
    gpu[0]["dX"] = torch.empty(T, H, dtype=torch.float16, device=DEV)
    gpu[1]["dX"] = torch.empty(512, 1024, dtype=torch.float16, device=DEV)
    start = [t["W"].clone() for t in gpu]

    def reset():
        for t, w in zip(gpu, start):
            t["W"].copy_(w)

    stepper = LomoStep(DEV, max_T=512, max_H=1024)
    captured = CapturedStep(stepper, gpu, lr, Sc)          # its warm-up and its recording do not count as steps here ...
    reset()                                                # ... but the warm-up has moved the weights
    stepper.run_async(gpu, lr, Sc)
    torch.cuda.synchronize()
    eager = [t["W"].clone() for t in gpu]
    eager_res = stepper.result()
    eager_dx = gpu[0]["dX"].clone()
    for rep in range(3):
        reset()
        gpu[0]["dX"].zero_()
        captured.replay()
        torch.cuda.synchronize()
        res = captured.result()
        assert res["overflow"] is False and abs(res["norm"] / eager_res["norm"] - 1) < 1e-9, rep
        assert abs(res["norm"] / ref["norm"] - 1) < 1e-5
        for t, e, w, c in zip(gpu, eager, ref["W"], cpu):
            got = t["W"]
            same = (got.view(torch.int16) == e.view(torch.int16)).float().mean().item()
            assert same > 0.9999, (rep, c["kind"], same)      # the step size may differ in its last bit (atomic order)
            _check_ulps(got.cpu().numpy(), w, f"replay {rep} {c['kind']}")
        assert torch.equal(gpu[0]["dX"].view(torch.int16), eager_dx.view(torch.int16))
        # the program's own eager work between replays
        reset()
        stepper.run_async(gpu, lr, Sc)
        torch.cuda.synchronize()
        for t, e in zip(gpu, eager):
            assert (t["W"].view(torch.int16) == e.view(torch.int16)).float().mean().item() > 0.9999
