"""Pins for the CPU oracle: everything here checks oracle/ against something other than itself.

Sources of truth used: central finite differences of a scalar loss (the definition of a
gradient), hand-computed fixtures under tests/golden/ (each cites the passage it follows),
exact rational arithmetic for rounding, brute-force Python loops on tiny inputs, closed forms
and the Gram identity for norms, and numbers printed in the paper.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import lomo_oracle as O
from golden_io import read_golden

RNG = np.random.default_rng(1234)


def f16(a):
    return np.asarray(a, dtype=np.float64).astype(np.float16)


# ----------------------------------------------------------------------------- P1 finite differences


class TinyModel:
    """embedding -> RMSNorm gain -> linear -> tanh -> linear -> scalar loss, all fp64."""

    def __init__(self, rng, T=5, V=6, H=4, D=3, Oo=2):
        self.ids = np.array([2, 0, 2, 5, 0][:T])
        self.V = V
        self.p = {
            "E": rng.normal(size=(V, H)),
            "g": 1.0 + 0.1 * rng.normal(size=(H,)),
            "W1": rng.normal(size=(D, H)) * 0.7,
            "W2": rng.normal(size=(Oo, D)) * 0.7,
        }
        self.C = rng.normal(size=(T, Oo))

    def forward(self, p):
        e = p["E"][self.ids]
        r = np.sqrt((e * e).mean(axis=1, keepdims=True) + 1e-5)
        xhat = e / r
        y = xhat * p["g"]
        h1 = y @ p["W1"].T
        a = np.tanh(h1)
        h2 = a @ p["W2"].T
        loss = 0.5 * (h2 * h2).sum() + (self.C * h2).sum()
        return loss, dict(e=e, r=r, xhat=xhat, y=y, a=a, h2=h2)

    def grads_via_oracle(self, lin=None, inp=None, vec=None, emb=None):
        lin = lin or O.linear_grad
        inp = inp or O.input_grad_f64
        vec = vec or O.vector_grad
        emb = emb or O.embedding_grad
        p = self.p
        _, c = self.forward(p)
        dh2 = c["h2"] + self.C
        gW2 = lin(c["a"], dh2)
        da = inp(dh2, p["W2"])
        dh1 = da * (1.0 - c["a"] ** 2)
        gW1 = lin(c["y"], dh1)
        dy = inp(dh1, p["W1"])
        gg = vec(c["xhat"], dy)
        dxhat = dy * p["g"]
        de = (dxhat - c["xhat"] * (dxhat * c["xhat"]).mean(axis=1, keepdims=True)) / c["r"]
        gE = emb(self.ids, de, self.V)
        return {"E": gE, "g": gg, "W1": gW1, "W2": gW2}

    def grads_fd(self, h=1e-6):
        out = {}
        for name, arr in self.p.items():
            g = np.zeros_like(arr)
            it = np.nditer(arr, flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = arr[idx]
                arr[idx] = old + h
                lp, _ = self.forward(self.p)
                arr[idx] = old - h
                lm, _ = self.forward(self.p)
                arr[idx] = old
                g[idx] = (lp - lm) / (2 * h)
            out[name] = g
        return out


def _fd_check(model, **mut):
    an = model.grads_via_oracle(**mut)
    fd = model.grads_fd()
    for k in fd:
        assert an[k].shape == fd[k].shape, k
        np.testing.assert_allclose(an[k], fd[k], rtol=2e-6, atol=2e-8, err_msg=k)


def test_p1_finite_differences_two_layer_model():
    _fd_check(TinyModel(np.random.default_rng(7)))


@pytest.mark.parametrize("mut", [
    dict(lin=lambda X, dY: O.as_f64(X).T @ O.as_f64(dY)),                 # transposed layout
    dict(lin=lambda X, dY: -O.linear_grad(X, dY)),                        # sign
    dict(inp=lambda dY, W: O.as_f64(dY) @ O.as_f64(W)[:, ::-1]),          # wrong index
    dict(vec=lambda xh, dY: O.as_f64(dY).sum(axis=0)),                    # dropped factor
    dict(emb=lambda ids, dY, V: O.embedding_grad(ids[::-1], dY, V)),      # wrong position order
])
def test_p1_is_sensitive_to_planted_mistakes(mut):
    with pytest.raises((AssertionError, ValueError)):
        _fd_check(TinyModel(np.random.default_rng(7)), **mut)


# ----------------------------------------------------------------------------- P2 hand examples


def test_p2_hand_linear_2x3(golden_dir):
    g = read_golden(os.path.join(golden_dir, "hand_linear_2x3.txt"))
    X, dY, W = f16(g["X"]), f16(g["dY"]), f16(g["W"])
    G = O.linear_grad(X, dY)
    np.testing.assert_array_equal(G, g["G"])
    assert O.sqnorm(G) == g["sqnorm"]
    Wn = O.sgd_update(W, G, g["lr"], 1.0, g["loss_scale"])
    np.testing.assert_array_equal(Wn.astype(np.float64), g["W_new"])
    np.testing.assert_array_equal(O.input_grad(dY, W).astype(np.float64), g["dX"])
    # the whole-step driver with clipping: coef = 1/(sqrt(335)+eps)
    res = O.step_materialised([dict(kind="linear", X=X, dY=dY, W=W)], g["lr"], 1.0, 1.0, 1e-6)
    coef = 1.0 / (math.sqrt(335.0) + 1e-6)
    assert res["clip_coef"] == pytest.approx(coef, rel=1e-15)
    expect = f16(g["W"] - g["lr"] * coef * g["G"])
    np.testing.assert_array_equal(res["W"][0], expect)


def test_p2_hand_sgd_4x4_with_loss_scale(golden_dir):
    g = read_golden(os.path.join(golden_dir, "hand_sgd_4x4.txt"))
    X, dY, W = f16(g["X"]), f16(g["dY"]), f16(g["W"])
    G = O.linear_grad(X, dY)
    np.testing.assert_array_equal(G, g["G"])
    Wn = O.sgd_update(W, G, g["lr"], 1.0, g["loss_scale"])
    assert Wn.dtype == np.float16
    np.testing.assert_array_equal(Wn.astype(np.float64), g["W_new"])
    # textbook SGD typed out independently: W - lr * (dY^T / S)
    np.testing.assert_array_equal(Wn.astype(np.float64), g["W"] - g["lr"] * (g["dY"].T / g["loss_scale"]))


def test_hand_embedding_and_vector(golden_dir):
    g = read_golden(os.path.join(golden_dir, "hand_embedding_vector.txt"))
    ids = g["ids"][0].astype(np.int32)
    G = O.embedding_grad(ids, f16(g["emb_dY"]), 4)
    np.testing.assert_array_equal(G, g["emb_G"])
    u, off, perm = O.embedding_grouping(ids)
    np.testing.assert_array_equal(perm, g["perm"][0])
    np.testing.assert_array_equal(u, g["unique_ids"][0])
    np.testing.assert_array_equal(off, g["seg_offsets"][0])
    np.testing.assert_array_equal(O.vector_grad(f16(g["xhat"]), f16(g["vec_dY"])), g["vec_g"][0])


# ----------------------------------------------------------------------------- P3 LOMO order == SGD


def _random_step_tensors(rng, S=64.0, with_inf=False):
    def h(*s, sd=1.0):
        return (rng.normal(size=s) * sd).astype(np.float16)
    T, V, H = 12, 9, 8
    ts = [
        dict(kind="linear", X=h(T, 8), dY=h(T, 6, sd=0.05 * S), W=h(6, 8, sd=0.3)),
        dict(kind="vector", X=h(T, H), dY=h(T, H, sd=0.05 * S), W=np.ones(H, np.float16)),
        dict(kind="linear", X=h(T, 10), dY=h(T, 8, sd=0.05 * S), W=h(8, 10, sd=0.3)),
        dict(kind="embedding", ids=rng.integers(0, V, size=T).astype(np.int32), dY=h(T, H, sd=0.05 * S),
             W=h(V, H, sd=0.3)),
    ]
    if with_inf:
        ts[2]["dY"][3, 1] = np.inf
    return ts


def _assert_same_step(a, b):
    assert a["overflow"] == b["overflow"] and a["flags"] == b["flags"]
    for x, y in zip(a["W"], b["W"]):
        np.testing.assert_array_equal(x.view(np.uint16), y.view(np.uint16))
    for x, y in zip(a["dX"], b["dX"]):
        assert (x is None) == (y is None)
        if x is not None:
            np.testing.assert_array_equal(x.view(np.uint16), y.view(np.uint16))


def test_p3_fused_order_equals_materialised_sgd():
    ts = _random_step_tensors(np.random.default_rng(3))
    a = O.step_materialised(ts, 0.25, 64.0)
    b = O.step_fused_order(ts, 0.25, 64.0)
    _assert_same_step(a, b)
    assert a["clip_coef"] == b["clip_coef"] < 1.0
    # and the update is visible: most weights moved
    moved = sum(int((x.view(np.uint16) != t["W"].view(np.uint16)).sum()) for x, t in zip(a["W"], ts))
    assert moved > 100


def test_p3_dx_uses_pre_update_weights():
    ts = _random_step_tensors(np.random.default_rng(4))
    res = O.step_fused_order(ts, 0.25, 64.0)
    lin = ts[0]
    brute = np.zeros((lin["dY"].shape[0], lin["W"].shape[1]))
    for t in range(brute.shape[0]):
        for k in range(brute.shape[1]):
            brute[t, k] = math.fsum(float(lin["dY"][t, n]) * float(lin["W"][n, k]) for n in range(lin["W"].shape[0]))
    np.testing.assert_array_equal(res["dX"][0], f16(brute))
    post = O.input_grad(lin["dY"], res["W"][0])
    assert (post.view(np.uint16) != res["dX"][0].view(np.uint16)).any()


# ----------------------------------------------------------------------------- P4 norms


def test_p4_bruteforce_gradient_and_norm():
    rng = np.random.default_rng(5)
    X = rng.normal(size=(7, 5)).astype(np.float16)
    dY = rng.normal(size=(7, 3)).astype(np.float16)
    G = O.linear_grad(X, dY)
    assert G.shape == (3, 5)
    tot = []
    for n in range(3):
        for k in range(5):
            v = math.fsum(float(dY[t, n]) * float(X[t, k]) for t in range(7))
            assert G[n, k] == pytest.approx(v, rel=1e-14, abs=1e-15)
            tot.append(v * v)
    assert O.sqnorm(G) == pytest.approx(math.fsum(tot), rel=1e-13)


def test_p4_closed_forms():
    rng = np.random.default_rng(6)
    x = rng.normal(size=(1, 9)).astype(np.float16)
    dy = rng.normal(size=(1, 4)).astype(np.float16)
    nx = math.sqrt(math.fsum(float(v) ** 2 for v in x[0]))
    ny = math.sqrt(math.fsum(float(v) ** 2 for v in dy[0]))
    assert math.sqrt(O.sqnorm(O.linear_grad(x, dy))) == pytest.approx(nx * ny, rel=1e-13)   # rank one
    eye = np.eye(6, dtype=np.float16)
    dY = rng.normal(size=(6, 4)).astype(np.float16)
    assert O.sqnorm(O.linear_grad(eye, dY)) == pytest.approx(
        math.fsum(float(v) ** 2 for v in dY.ravel()), rel=1e-13)


def test_p4_gram_identity():
    rng = np.random.default_rng(8)
    X = rng.normal(size=(11, 13)).astype(np.float16).astype(np.float64)
    dY = rng.normal(size=(11, 6)).astype(np.float16).astype(np.float64)
    gram = 0.0
    for t in range(11):
        for u in range(11):
            gram += float(X[t] @ X[u]) * float(dY[t] @ dY[u])
    assert O.sqnorm(O.linear_grad(X.astype(np.float16), dY.astype(np.float16))) == pytest.approx(gram, rel=1e-12)


def test_global_norm_is_over_all_tensors_and_unscaled():
    ts = _random_step_tensors(np.random.default_rng(9), S=64.0)
    res = O.step_materialised(ts, 0.1, 64.0)
    per = [O.sqnorm(O.tensor_grad(t)) for t in ts]
    assert res["norm"] == pytest.approx(math.sqrt(math.fsum(per)) / 64.0, rel=1e-14)
    assert res["norm"] > max(math.sqrt(p) / 64.0 for p in per)     # not a per-tensor norm


# ----------------------------------------------------------------------------- P5 printed numbers


def test_p5_table1_parameter_and_gradient_memory(golden_dir):
    from lomo_synth import llama_tensor_list, count_params
    g = read_golden(os.path.join(golden_dir, "paper_printed_values.txt"))
    ts = llama_tensor_list(4096, 4096, 11008, 32, 32000, final_norm=True)
    n = count_params(ts)
    assert n == 6_738_415_616
    assert round(n * 2 / 2 ** 30, 2) == g["params_gb"]
    largest = max(t.n_params for t in ts)
    assert largest == 32000 * 4096
    assert round(largest * 2 / 2 ** 30, 2) == g["lomo_grad_gb"]
    assert g["max_grad_norm"] == 1.0


# ----------------------------------------------------------------------------- P6..P8 invariants


def test_p6_loss_scale_invariance_is_bit_exact():
    rng = np.random.default_rng(10)
    ts = _random_step_tensors(rng, S=64.0)
    ts2 = [dict(t) for t in ts]
    for t, t0 in zip(ts2, ts):
        t["dY"] = (t0["dY"].astype(np.float64) * 2).astype(np.float16)
        assert np.array_equal(t["dY"].astype(np.float64), t0["dY"].astype(np.float64) * 2)
    a = O.step_materialised(ts, 0.25, 64.0)
    b = O.step_materialised(ts2, 0.25, 128.0)
    assert a["norm"] == b["norm"] and a["flags"] == b["flags"]
    for x, y in zip(a["W"], b["W"]):
        np.testing.assert_array_equal(x.view(np.uint16), y.view(np.uint16))
    for x, y in zip(a["dX"], b["dX"]):       # dX carries the scale: it doubles exactly
        if x is not None:
            np.testing.assert_array_equal(x.astype(np.float64) * 2, y.astype(np.float64))


def test_p7_clip_invariants():
    assert O.clip_coef(0.5, 1.0, 1e-6) == 1.0                 # below the threshold: plain SGD
    assert O.clip_coef(1.0 - 2e-6, 1.0, 1e-6) == 1.0
    c = O.clip_coef(20.0, 1.0, 1e-6)
    assert c == pytest.approx(1 / 20.000001, rel=1e-15)
    assert c * 20.0 == pytest.approx(20.0 / 20.000001, rel=1e-15)   # post-clip norm = c*norm/(norm+eps)
    assert O.clip_coef(4.0, 2.0, 0.0) == 0.5
    assert O.grad_norm(3.0 ** 2 * 8.0 ** 2, 8.0) == 3.0
    # small gradient => unclipped step equals plain SGD
    X = np.eye(4, dtype=np.float16)
    dY = (np.full((4, 4), 0.125)).astype(np.float16)
    W = np.zeros((4, 4), np.float16)
    res = O.step_materialised([dict(kind="linear", X=X, dY=dY, W=W)], 0.5, 1.0)
    assert res["clip_coef"] == 1.0
    np.testing.assert_array_equal(res["W"][0].astype(np.float64), -0.0625 * np.ones((4, 4)))


def test_p8_overflow_skips_every_tensor_and_halves_scale():
    ts = _random_step_tensors(np.random.default_rng(11), with_inf=True)
    for fn in (O.step_materialised, O.step_fused_order):
        res = fn(ts, 0.25, 64.0)
        assert res["overflow"] and res["flags"] == [False, False, True, False]
        for w, t in zip(res["W"], ts):
            np.testing.assert_array_equal(w.view(np.uint16), t["W"].view(np.uint16))
    nan_ts = _random_step_tensors(np.random.default_rng(11))
    nan_ts[1]["X"][0, 0] = np.nan
    assert O.step_materialised(nan_ts, 0.25, 64.0)["flags"] == [False, True, False, False]
    emb_ts = _random_step_tensors(np.random.default_rng(11))
    emb_ts[3]["dY"][2, 2] = -np.inf
    assert O.step_materialised(emb_ts, 0.25, 64.0)["flags"] == [False, False, False, True]


def test_p8_lr_zero_leaves_weights_and_dx_correct():
    ts = _random_step_tensors(np.random.default_rng(12))
    res = O.step_materialised(ts, 0.0, 64.0)
    for w, t in zip(res["W"], ts):
        np.testing.assert_array_equal(w.view(np.uint16), t["W"].view(np.uint16))
    assert res["dX"][0] is not None and np.isfinite(res["dX"][0].astype(np.float64)).all()


def test_scaler_state_machine():
    S, c = 65536.0, 0
    S, c = O.scaler_step(S, c, 2, True);  assert (S, c) == (32768.0, 0)
    S, c = O.scaler_step(S, c, 2, False); assert (S, c) == (32768.0, 1)
    S, c = O.scaler_step(S, c, 2, False); assert (S, c) == (65536.0, 0)
    S, c = O.scaler_step(S, c, 2, False); assert (S, c) == (65536.0, 1)
    S, c = O.scaler_step(S, c, 2, True);  assert (S, c) == (32768.0, 0)
    assert O.scaler_step(1.0, 5, 2, True) == (1.0, 0)
    assert O.scaler_step(2.0 ** 24, 1, 2, False) == (2.0 ** 24, 0)


# ----------------------------------------------------------------------------- P9, P10 reductions


def test_p9_embedding_is_onehot_linear():
    rng = np.random.default_rng(13)
    T, V, H = 17, 7, 5
    ids = rng.integers(0, V, size=T).astype(np.int32)
    dY = rng.normal(size=(T, H)).astype(np.float16)
    onehot = np.zeros((T, V), np.float16)
    onehot[np.arange(T), ids] = 1
    # G_emb [V x H] = onehot^T dY = linear_grad(X=dY, dY=onehot)
    np.testing.assert_allclose(O.embedding_grad(ids, dY, V), O.linear_grad(dY, onehot), rtol=1e-14, atol=1e-14)
    same = np.full(T, 3, np.int32)
    G = O.embedding_grad(same, dY, V)
    np.testing.assert_allclose(G[3], dY.astype(np.float64).sum(axis=0), rtol=1e-14)
    assert not G[[0, 1, 2, 4, 5, 6]].any()
    distinct = rng.permutation(V)[:5].astype(np.int32)
    G = O.embedding_grad(distinct, dY[:5], V)
    np.testing.assert_array_equal(G[distinct], dY[:5].astype(np.float64))


def test_p9_grouping_bruteforce():
    rng = np.random.default_rng(14)
    for T in (0, 1, 2, 33):
        ids = rng.integers(0, 6, size=T).astype(np.int32)
        u, off, perm = O.embedding_grouping(ids)
        pairs = sorted((int(v), t) for t, v in enumerate(ids))
        assert [t for _, t in pairs] == perm.tolist()
        uniq = sorted(set(int(v) for v in ids))
        assert u.tolist() == uniq
        assert off.tolist() == [sum(1 for v, _ in pairs if v < x) for x in uniq] + [T]


def test_untouched_embedding_rows_are_bit_identical():
    ts = _random_step_tensors(np.random.default_rng(15))
    res = O.step_materialised(ts, 0.25, 64.0)
    emb, new = ts[3], res["W"][3]
    absent = sorted(set(range(9)) - set(int(v) for v in emb["ids"]))
    assert absent
    np.testing.assert_array_equal(new[absent].view(np.uint16), emb["W"][absent].view(np.uint16))


def test_p10_vector_grad_is_diagonal_of_linear():
    rng = np.random.default_rng(16)
    xh = rng.normal(size=(9, 6)).astype(np.float16)
    dY = rng.normal(size=(9, 6)).astype(np.float16)
    np.testing.assert_allclose(O.vector_grad(xh, dY), np.diag(O.linear_grad(xh, dY)), rtol=1e-14)


def test_p11_clip_by_value_printed_example(golden_dir):
    g = read_golden(os.path.join(golden_dir, "paper_printed_values.txt"))
    W = np.zeros(2, np.float16)
    out = O.sgd_update_clip_value(W, g["clip_value_in"][0], 1.0, 1.0, 1.0)
    np.testing.assert_array_equal(out, f16(-g["clip_value_out"][0]))
    out = O.sgd_update_clip_value(W, -4.0 * g["clip_value_in"][0], 1.0, 1.0, 4.0)   # scaled, other sign
    np.testing.assert_array_equal(out, f16(g["clip_value_out"][0]))


def test_clip_by_value_hand_cases():
    """Hand-worked: W = [1, 1, 1, 1], scaled G = [8, -8, 1, inf], S = 4, c = 1, lr = 0.5.
    g = [2, -2, 0.25, inf] -> clamp [1, -1, 0.25, (left alone)] -> W' = [0.5, 1.5, 0.875, 1]."""
    W = np.ones(4, np.float16)
    G = np.array([8.0, -8.0, 1.0, np.inf])
    out = O.sgd_update_clip_value(W, G, 0.5, 1.0, 4.0)
    np.testing.assert_array_equal(out.astype(np.float64), [0.5, 1.5, 0.875, 1.0])
    assert O.has_overflow(G)
    out = O.sgd_update_clip_value(W, np.array([np.nan, 2.0, -0.5, 0.0]), 1.0, 0.25, 1.0)
    np.testing.assert_array_equal(out.astype(np.float64), [1.0, 0.75, 1.25, 1.0])
    # below the threshold it is plain SGD
    G = np.array([0.5, -0.25, 0.125, 0.0])
    np.testing.assert_array_equal(O.sgd_update_clip_value(W, G, 0.5, 1.0, 1.0), O.sgd_update(W, G, 0.5, 1.0, 1.0))


# ----------------------------------------------------------------------------- rounding


def _all_finite_f16():
    bits = np.arange(0, 0x7C00, dtype=np.uint16)
    return bits.view(np.float16).astype(np.float64)        # non-negative finite values, ascending


_POS = _all_finite_f16()


def _rne_exact(v: float) -> float:
    """Nearest fp16 to an fp64 value by exact rational comparison; ties to even mantissa."""
    s = -1.0 if v < 0 or (v == 0 and math.copysign(1, v) < 0) else 1.0
    a = Fraction(abs(v))
    if a >= Fraction(65520):
        return s * math.inf
    hi = int(np.searchsorted(_POS, float(abs(v)), side="left"))
    hi = min(hi, len(_POS) - 1)
    lo = max(hi - 1, 0)
    dl, dh = a - Fraction(_POS[lo]), Fraction(_POS[hi]) - a
    if dh < 0:
        return s * _POS[hi]
    if dl < dh:
        return s * _POS[lo]
    if dh < dl:
        return s * _POS[hi]
    return s * (_POS[lo] if lo % 2 == 0 else _POS[hi])


def test_round_f16_is_direct_rne():
    rng = np.random.default_rng(17)
    vals = np.concatenate([
        rng.normal(size=400) * 0.02, rng.normal(size=200) * 100, rng.normal(size=200) * 1e-6,
        [1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 1 + 2.0 ** -11 + 2.0 ** -40, 1 + 2.0 ** -11 - 2.0 ** -40,
         65504.0, 65519.999, 65520.0, -65520.0, 2.0 ** -25, 2.0 ** -25 + 2.0 ** -60, 3 * 2.0 ** -25, 0.0, -0.0],
    ])
    got = O.round_f16(vals).astype(np.float64)
    for v, g in zip(vals, got):
        assert g == _rne_exact(float(v)), v
    # the double-rounding hazard: via fp32 this value would become a tie and round down to 1.0
    hazard = 1 + 2.0 ** -11 + 2.0 ** -40
    assert float(O.round_f16(np.array([hazard]))[0]) == 1 + 2.0 ** -10
    assert float(np.float32(hazard).astype(np.float16)) == 1.0


def test_update_is_full_precision_rounded_once():
    """Section 3.3.2: the update runs in full precision; an fp16-arithmetic update differs."""
    rng = np.random.default_rng(18)
    W = (rng.normal(size=(32, 32)) * 0.02).astype(np.float16)
    G = rng.normal(size=(32, 32)) * 40.0
    lr, coef, S = 1e-2, 0.05, 64.0
    got = O.sgd_update(W, G, lr, coef, S).astype(np.float64)
    for idx in [(0, 0), (3, 7), (31, 31), (10, 20)]:
        exact = Fraction(float(W[idx])) - Fraction(lr) * Fraction(coef) * Fraction(float(G[idx])) / Fraction(S)
        assert got[idx] == _rne_exact(float(exact))
    straw = (W - (np.float16(lr) * (G / S * coef).astype(np.float16)).astype(np.float16)).astype(np.float16)
    assert (straw.view(np.uint16) != O.sgd_update(W, G, lr, coef, S).view(np.uint16)).any()


def test_ulp_distance():
    one = np.array([1.0], np.float16)
    nxt = (one.view(np.uint16) + 1).view(np.float16)
    assert O.ulp_distance_f16(one, nxt)[0] == 1
    assert O.ulp_distance_f16(np.array([0.0], np.float16), np.array([-0.0], np.float16))[0] == 0
    tiny = np.array([1], np.uint16).view(np.float16)
    assert O.ulp_distance_f16(tiny, -tiny)[0] == 2
    assert O.ulp_distance_f16(np.array([2.0], np.float16), np.array([1.0], np.float16))[0] == 1024


def test_oracle_does_not_import_the_hip_path():
    import ast
    import oracle.lomo_oracle as mod
    import oracle.mlp_chain as chain
    import oracle.attn_chain as attn
    for m in (mod, chain, attn):
        tree = ast.parse(open(m.__file__).read())
        names = set()
        for node in ast.walk(tree):
            if isinstance(node, ast.Import):
                names |= {a.name.split(".")[0] for a in node.names}
            elif isinstance(node, ast.ImportFrom):
                names.add((node.module or "").split(".")[0] if node.level == 0 else "oracle")
        assert names <= {"__future__", "math", "typing", "numpy", "oracle"}, names


# --------------------------------------------------------------------------- feed-forward block chain

from oracle import mlp_chain as M


def _block_inputs(rng, T=3, H=4, F=5):
    h = rng.normal(size=(T, H))
    w = 1.0 + 0.3 * rng.normal(size=H)
    W_gu = 0.7 * rng.normal(size=(2 * F, H))
    W_d = 0.7 * rng.normal(size=(H, F))
    R = rng.normal(size=(T, H))
    return h, w, W_gu, W_d, R


def _block_grads_f64(h, w, W_gu, W_d, dy, eps):
    """The chain's formulas composed in fp64 without any storage rounding."""
    F = W_d.shape[1]
    xhat, r, xn = M.rmsnorm_forward(h, w, eps)
    gu = xn @ W_gu.T
    a = M.silu(gu[:, :F]) * gu[:, F:]
    da = O.input_grad_f64(dy, W_d)
    dgu = M.swiglu_backward(da, gu)
    dxn = O.input_grad_f64(dgu, W_gu)
    return {"G_d": O.linear_grad(a, dy), "G_gu": O.linear_grad(xn, dgu), "g_w": O.vector_grad(xhat, dxn),
            "dh": M.rmsnorm_backward(dxn, xhat, r, w, dres=dy)}


def test_block_chain_finite_differences():
    rng = np.random.default_rng(5)
    eps = 1e-3
    h, w, W_gu, W_d, R = _block_inputs(rng)
    got = _block_grads_f64(h, w, W_gu, W_d, R, eps)          # loss = sum(y * R)  =>  dy = R
    loss = lambda h_, w_, Wgu_, Wd_: float((M.block_forward_f64(h_, w_, Wgu_, Wd_, eps) * R).sum())
    d = 1e-6

    def fd(arr, idx, which):
        p, m = arr.copy(), arr.copy()
        p[idx] += d
        m[idx] -= d
        args_p = {"h": h, "w": w, "W_gu": W_gu, "W_d": W_d}
        args_m = dict(args_p)
        args_p[which], args_m[which] = p, m
        return (loss(args_p["h"], args_p["w"], args_p["W_gu"], args_p["W_d"]) -
                loss(args_m["h"], args_m["w"], args_m["W_gu"], args_m["W_d"])) / (2 * d)

    for which, arr, grad in (("W_d", W_d, got["G_d"]), ("W_gu", W_gu, got["G_gu"]), ("w", w, got["g_w"]),
                             ("h", h, got["dh"])):
        for idx in np.ndindex(arr.shape):
            assert fd(arr, idx, which) == pytest.approx(grad[idx], rel=2e-6, abs=2e-7), (which, idx)


@pytest.mark.parametrize("mut", ["silu_prime_without_product_term", "rms_without_projection", "gain_uses_xn",
                                 "dup_uses_sigmoid_only"])
def test_block_chain_finite_differences_catch_planted_mistakes(mut):
    """The same check must fail for plausible wrong formulas (planted here, in CPU code only)."""
    rng = np.random.default_rng(6)
    eps = 1e-3
    h, w, W_gu, W_d, R = _block_inputs(rng)
    F = W_d.shape[1]
    xhat, r, xn = M.rmsnorm_forward(h, w, eps)
    gu = xn @ W_gu.T
    g, u = gu[:, :F], gu[:, F:]
    s = M.sigmoid(g)
    da = R @ W_d
    good = _block_grads_f64(h, w, W_gu, W_d, R, eps)
    if mut == "silu_prime_without_product_term":
        dgu = np.concatenate((da * u * s, da * g * s), axis=1)
        bad, ref = O.linear_grad(xn, dgu), good["G_gu"]
    elif mut == "dup_uses_sigmoid_only":
        dgu = np.concatenate((da * u * (s * (1 + g * (1 - s))), da * s), axis=1)
        bad, ref = O.linear_grad(xn, dgu), good["G_gu"]
    elif mut == "rms_without_projection":
        dxn = M.swiglu_backward(da, gu) @ W_gu
        bad, ref = r[:, None] * (dxn * w) + R, good["dh"]
    else:
        dxn = M.swiglu_backward(da, gu) @ W_gu
        bad, ref = (dxn * xn).sum(0), good["g_w"]
    assert np.abs(bad - ref).max() > 1e-3 * np.abs(ref).max()


def test_block_hand_example(golden_dir):
    g = read_golden(os.path.join(golden_dir, "hand_mlp_block.txt"))
    h, w, W_gu, W_d, dy = g["h"], g["w"][0], g["W_gu"], g["W_d"], g["dy"]
    np.testing.assert_allclose(M.block_forward_f64(h, w, W_gu, W_d, g["eps"]), g["y"], rtol=1e-14)
    xhat, r, xn = M.rmsnorm_forward(h, w, g["eps"])
    gu = xn @ W_gu.T
    a = M.silu(gu[:, :1]) * gu[:, 1:]
    da = O.input_grad_f64(dy, W_d)
    np.testing.assert_allclose(da, g["da"], rtol=1e-14)
    dgu = M.swiglu_backward(da, gu)
    np.testing.assert_allclose(dgu, g["dgu"], rtol=1e-14)
    dxn = O.input_grad_f64(dgu, W_gu)
    np.testing.assert_allclose(dxn, g["dxn"], rtol=1e-14)
    np.testing.assert_allclose(O.linear_grad(a, dy), g["G_d"], rtol=1e-14)
    np.testing.assert_allclose(O.linear_grad(xn, dgu), g["G_gu"], rtol=1e-14)
    np.testing.assert_allclose(O.vector_grad(xhat, dxn), g["g_w"][0], rtol=1e-14)
    np.testing.assert_allclose(M.rmsnorm_backward(dxn, xhat, r, w, dres=dy), g["dh"], rtol=1e-14)


def test_swiglu_backward_closed_forms():
    one = np.ones((1, 1))
    for gate, dgate_want, dup_want in ((0.0, 0.5, 0.0), (40.0, 1.0, 40.0), (-40.0, 0.0, 0.0)):
        out = M.swiglu_backward(one, np.array([[gate, 1.0]]))
        assert out[0, 0] == pytest.approx(dgate_want, abs=1e-12) and out[0, 1] == pytest.approx(dup_want, abs=1e-12)
    # silu'(g) against a difference quotient of silu itself
    for gate in (-3.0, -0.5, 0.3, 2.0):
        fdq = (M.silu(np.array(gate + 1e-6)) - M.silu(np.array(gate - 1e-6))) / 2e-6
        assert M.swiglu_backward(one, np.array([[gate, 1.0]]))[0, 0] == pytest.approx(float(fdq), rel=1e-8)


def test_rmsnorm_backward_is_orthogonal_to_its_input():
    """RMSNorm ignores the scale of h (eps = 0), so the gradient through it has no component along h."""
    rng = np.random.default_rng(7)
    h = rng.normal(size=(5, 16))
    w = rng.normal(size=16)
    xhat, r, _ = M.rmsnorm_forward(h, w, 0.0)
    dxn = rng.normal(size=(5, 16))
    dh = M.rmsnorm_backward(dxn, xhat, r, w)
    assert np.abs((dh * h).sum(1)).max() < 1e-12 * np.abs(dh).max() * np.abs(h).max() * 16
    assert np.allclose((xhat * xhat).mean(1), 1.0)
    # all-equal row, unit gain: xhat = 1, any dxn is projected onto the zero-mean subspace
    dh1 = M.rmsnorm_backward(np.array([[1.0, 2.0, 3.0, 6.0]]), np.ones((1, 4)), np.array([0.5]), np.ones(4))
    np.testing.assert_allclose(dh1, 0.5 * (np.array([[1.0, 2.0, 3.0, 6.0]]) - 3.0))


def _stored_block(seed, T=24, H=16, F=24, scale=256.0):
    rng = np.random.default_rng(seed)
    h = rng.normal(size=(T, H)).astype(np.float16)
    w = (1.0 + 0.1 * rng.normal(size=H)).astype(np.float16)
    W_gu = (0.3 * rng.normal(size=(2 * F, H))).astype(np.float16)
    W_d = (0.3 * rng.normal(size=(H, F))).astype(np.float16)
    dy = (0.01 * scale * rng.normal(size=(T, H))).astype(np.float16)
    return h, w, W_gu, W_d, dy, M.block_forward_stored(h, w, W_gu, W_d, 1e-5)


def test_block_step_fused_order_equals_materialised():
    h, w, W_gu, W_d, dy, saved = _stored_block(8)
    a = M.block_step(dy, saved, w, W_gu, W_d, 0.5, 256.0, max_norm=1e9)
    b = M.block_step_fused_order(dy, saved, w, W_gu, W_d, 0.5, 256.0, max_norm=1e9)
    for k in ("W_d", "W_gu", "w", "dh"):
        np.testing.assert_array_equal(a[k].view(np.uint16), b[k].view(np.uint16))
    assert (a["W_gu"].view(np.uint16) != W_gu.view(np.uint16)).mean() > 0.5       # the step is visible
    assert a["clip_coef"] == 1.0 and a["overflow"] is False


def test_block_step_matches_generic_step_on_its_three_tensors():
    """The block step is the generic materialised step applied to (W_d, W_gu, w) with the chain's hand-ons."""
    h, w, W_gu, W_d, dy, saved = _stored_block(9)
    a = M.block_step(dy, saved, w, W_gu, W_d, 0.05, 256.0)
    recs = [dict(kind="linear", X=saved["a"], dY=dy, W=W_d), dict(kind="linear", X=saved["xn"], dY=a["dgu"], W=W_gu),
            dict(kind="vector", X=saved["xhat"], dY=a["dxn"], W=w)]
    b = O.step_materialised(recs, 0.05, 256.0)
    assert a["clip_coef"] == b["clip_coef"] and a["norm"] == b["norm"] and a["clip_coef"] < 1.0
    for got, want in zip((a["W_d"], a["W_gu"], a["w"]), b["W"]):
        np.testing.assert_array_equal(got.view(np.uint16), want.view(np.uint16))
    np.testing.assert_array_equal(a["da"].view(np.uint16), b["dX"][0].view(np.uint16))


def test_block_step_overflow_and_scale_invariance():
    h, w, W_gu, W_d, dy, saved = _stored_block(10)
    bad = dy.copy()
    bad[3, 2] = np.inf
    r = M.block_step(bad, saved, w, W_gu, W_d, 0.05, 256.0)
    assert r["overflow"] is True
    for k, p in (("W_d", W_d), ("W_gu", W_gu), ("w", w)):
        np.testing.assert_array_equal(r[k].view(np.uint16), p.view(np.uint16))
    # doubling the loss scale doubles dy exactly and changes no parameter bit
    a = M.block_step(dy, saved, w, W_gu, W_d, 0.05, 256.0)
    b = M.block_step((dy.astype(np.float32) * 2).astype(np.float16), saved, w, W_gu, W_d, 0.05, 512.0)
    for k in ("W_d", "W_gu", "w"):
        np.testing.assert_array_equal(a[k].view(np.uint16), b[k].view(np.uint16))


# --------------------------------------------------------------------------- attention block chain

from oracle import attn_chain as A


def test_attention_hand_example(golden_dir):
    g = read_golden(os.path.join(golden_dir, "hand_attention_2tok.txt"))
    o, lse = A.attention_forward_f64(g["q"], g["k"], g["v"], 2, 1)
    np.testing.assert_allclose(o, g["o"], rtol=1e-14)
    np.testing.assert_allclose(lse, g["lse"], rtol=1e-14)
    qkv = np.concatenate((g["q"], g["k"], g["v"]), axis=1)
    d = A.attention_backward(qkv, o, g["do"], lse, 2, 1, round_probabilities=False)
    np.testing.assert_allclose(d[:, 0:2], g["dq"], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(d[:, 2:4], g["dk"], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(d[:, 4:6], g["dv"], rtol=1e-13, atol=1e-15)


def test_attention_backward_finite_differences():
    rng = np.random.default_rng(11)
    s, nh, dd, B = 5, 2, 4, 2
    T, H = B * s, nh * dd
    q, k, v, R = (rng.normal(size=(T, H)) for _ in range(4))
    o, lse = A.attention_forward_f64(q, k, v, s, nh)
    got = A.attention_backward(np.concatenate((q, k, v), axis=1), o, R, lse, s, nh, round_probabilities=False)
    loss = lambda q_, k_, v_: float((A.attention_forward_f64(q_, k_, v_, s, nh)[0] * R).sum())
    e = 1e-6
    for part, arr in enumerate((q, k, v)):
        for idx in np.ndindex(arr.shape):
            p, m = arr.copy(), arr.copy()
            p[idx] += e
            m[idx] -= e
            args_p, args_m = [q, k, v], [q, k, v]
            args_p[part], args_m[part] = p, m
            fd = (loss(*args_p) - loss(*args_m)) / (2 * e)
            assert fd == pytest.approx(got[idx[0], part * H + idx[1]], rel=1e-6, abs=1e-8), (part, idx)
    # structure: rows of P sum to one; delta equals sum_j P dP; the last key hears the last query only
    for b in range(B):
        sl = slice(b * s, (b + 1) * s)
        for n in range(nh):
            hs = slice(n * dd, (n + 1) * dd)
            S = (q[sl, hs] @ k[sl, hs].T) / math.sqrt(dd)
            S[np.triu_indices(s, 1)] = -np.inf
            P = np.exp(S - lse[sl, n][:, None])
            np.testing.assert_allclose(P.sum(1), 1.0, rtol=1e-13)
            dP = R[sl, hs] @ v[sl, hs].T
            np.testing.assert_allclose((P * dP).sum(1), (R[sl, hs] * o[sl, hs]).sum(1), rtol=1e-12)
            np.testing.assert_allclose(got[sl, 2 * H + n * dd:2 * H + (n + 1) * dd][-1], P[-1, -1] * R[sl, hs][-1], rtol=1e-12)


def test_rope_is_a_rotation():
    rng = np.random.default_rng(12)
    s, nh, dd = 7, 3, 8
    cos, sin = A.rope_tables(s, dd)
    x = rng.normal(size=(2 * s, nh * dd))
    y = A.rope_rotate(x, cos, sin, s, nh)
    np.testing.assert_allclose(A.rope_rotate(y, cos, sin, s, nh, inverse=True), x, atol=1e-6)   # fp32 table
    np.testing.assert_allclose((y.reshape(2 * s, nh, dd) ** 2).sum(-1), (x.reshape(2 * s, nh, dd) ** 2).sum(-1), rtol=1e-6)
    np.testing.assert_array_equal(y[0], x[0])                      # position 0: angle 0
    np.testing.assert_array_equal(y[s], x[s])                      # first token of the second sequence
    # d = 2, position 1, theta_0 = 1: the textbook plane rotation by one radian
    c1, s1 = A.rope_tables(2, 2)
    r = A.rope_rotate(np.array([[0.0, 0.0], [3.0, 4.0]]), c1, s1, 2, 1)
    np.testing.assert_allclose(r[1], [3 * math.cos(1) - 4 * math.sin(1), 4 * math.cos(1) + 3 * math.sin(1)], rtol=1e-6)
    # the backward step is the transpose of the forward one: <rotate(x), g> == <x, rotate^-1(g)>
    gq = rng.normal(size=x.shape)
    assert float((y * gq).sum()) == pytest.approx(float((x * A.rope_rotate(gq, cos, sin, s, nh, inverse=True)).sum()), rel=1e-12)


def _attn_block_inputs(rng, B=2, s=4, nh=2, dd=4):
    T, H = B * s, nh * dd
    h = rng.normal(size=(T, H))
    w = 1.0 + 0.3 * rng.normal(size=H)
    W_qkv = 0.6 * rng.normal(size=(3 * H, H))
    W_o = 0.6 * rng.normal(size=(H, H))
    R = rng.normal(size=(T, H))
    return h, w, W_qkv, W_o, R, s, nh


def test_attention_block_chain_finite_differences():
    rng = np.random.default_rng(13)
    eps = 1e-3
    h, w, W_qkv, W_o, R, s, nh = _attn_block_inputs(rng)
    T, H = h.shape
    cos, sin = A.rope_tables(s, H // nh)
    # the chain's formulas composed in fp64 without storage rounding
    xhat, r, xn = M.rmsnorm_forward(h, w, eps)
    qkv = xn @ W_qkv.T
    q = A.rope_rotate(qkv[:, :H], cos, sin, s, nh)
    k = A.rope_rotate(qkv[:, H:2 * H], cos, sin, s, nh)
    o, lse = A.attention_forward_f64(q, k, qkv[:, 2 * H:], s, nh)
    do = O.input_grad_f64(R, W_o)
    g = A.attention_backward(np.concatenate((q, k, qkv[:, 2 * H:]), axis=1), o, do, lse, s, nh, round_probabilities=False)
    dqkv = np.concatenate((A.rope_rotate(g[:, :H], cos, sin, s, nh, inverse=True),
                           A.rope_rotate(g[:, H:2 * H], cos, sin, s, nh, inverse=True), g[:, 2 * H:]), axis=1)
    dxn = O.input_grad_f64(dqkv, W_qkv)
    got = {"W_o": O.linear_grad(o, R), "W_qkv": O.linear_grad(xn, dqkv), "w": O.vector_grad(xhat, dxn),
           "h": M.rmsnorm_backward(dxn, xhat, r, w, dres=R)}
    base = {"h": h, "w": w, "W_qkv": W_qkv, "W_o": W_o}
    loss = lambda a: float((A.block_forward_f64(a["h"], a["w"], a["W_qkv"], a["W_o"], cos, sin, s, nh, eps) * R).sum())
    e = 1e-6
    for which in ("W_o", "W_qkv", "w", "h"):
        arr = base[which]
        for idx in list(np.ndindex(arr.shape))[::3]:
            p, m = dict(base), dict(base)
            p[which], m[which] = arr.copy(), arr.copy()
            p[which][idx] += e
            m[which][idx] -= e
            fd = (loss(p) - loss(m)) / (2 * e)
            assert fd == pytest.approx(got[which][idx], rel=5e-6, abs=1e-7), (which, idx)


def test_attention_block_step_is_the_generic_step_on_its_tensors():
    rng = np.random.default_rng(14)
    B, s, nh, dd = 2, 8, 2, 8
    T, H = B * s, nh * dd
    f16 = lambda shape, sig: (sig * rng.normal(size=shape)).astype(np.float16)
    h, w = f16((T, H), 1.0), (1.0 + 0.1 * rng.normal(size=H)).astype(np.float16)
    W_qkv, W_o, dy = f16((3 * H, H), 0.3), f16((H, H), 0.3), f16((T, H), 2.0)
    cos, sin = A.rope_tables(s, dd)
    saved = A.block_forward_stored(h, w, W_qkv, W_o, cos, sin, s, nh, 1e-5)
    a = A.block_step(dy, saved, w, W_qkv, W_o, cos, sin, s, nh, 0.05, 256.0)
    recs = [dict(kind="linear", X=saved["o"], dY=dy, W=W_o), dict(kind="linear", X=saved["xn"], dY=a["dqkv"], W=W_qkv),
            dict(kind="vector", X=saved["xhat"], dY=a["dxn"], W=w)]
    b = O.step_materialised(recs, 0.05, 256.0)
    assert a["clip_coef"] == b["clip_coef"] and a["overflow"] is False
    for got, want in zip((a["W_o"], a["W_qkv"], a["w"]), b["W"]):
        np.testing.assert_array_equal(got.view(np.uint16), want.view(np.uint16))
    # storage rounding of P and dS matters little but is there: the unrounded route differs slightly
    g16 = A.attention_backward(saved["qkv"], saved["o"], a["do"], saved["lse"], s, nh)
    g64 = A.attention_backward(saved["qkv"], saved["o"], a["do"], saved["lse"], s, nh, round_probabilities=False)
    rel = np.abs(g16 - g64).max() / np.abs(g64).max()
    assert 0 < rel < 2e-3
    bad = dy.copy()
    bad[5, 1] = np.nan
    r = A.block_step(bad, saved, w, W_qkv, W_o, cos, sin, s, nh, 0.05, 256.0)
    assert r["overflow"] is True
    np.testing.assert_array_equal(r["W_qkv"].view(np.uint16), W_qkv.view(np.uint16))


@pytest.mark.parametrize("mut", ["no_delta", "no_scale", "rope_forward_instead_of_inverse", "no_causal_mask"])
def test_attention_finite_differences_catch_planted_mistakes(mut):
    """Wrong formulas planted in CPU code must disagree with the difference quotients."""
    rng = np.random.default_rng(15)
    s, nh, dd = 4, 1, 4
    cos, sin = A.rope_tables(s, dd)
    qp, kp, v, R = (rng.normal(size=(s, dd)) for _ in range(4))          # before the rotary step

    def fwd(q_, k_, v_):
        return A.attention_forward_f64(A.rope_rotate(q_, cos, sin, s, nh), A.rope_rotate(k_, cos, sin, s, nh), v_, s, nh)

    loss = lambda q_, k_, v_: float((fwd(q_, k_, v_)[0] * R).sum())
    e = 1e-6
    fd = np.zeros((s, dd))
    for idx in np.ndindex(qp.shape):
        p, m = qp.copy(), qp.copy()
        p[idx] += e
        m[idx] -= e
        fd[idx] = (loss(p, kp, v) - loss(m, kp, v)) / (2 * e)
    q, k = A.rope_rotate(qp, cos, sin, s, nh), A.rope_rotate(kp, cos, sin, s, nh)
    o, lse = fwd(qp, kp, v)
    S = (q @ k.T) / math.sqrt(dd)
    if mut != "no_causal_mask":
        S[np.triu_indices(s, 1)] = -np.inf
    P = np.exp(S - lse[:, 0][:, None])
    dP = R @ v.T
    delta = 0.0 if mut == "no_delta" else (R * o).sum(1, keepdims=True)
    dS = P * (dP - delta) / (1.0 if mut == "no_scale" else math.sqrt(dd))
    dq_rot = dS @ k
    bad = A.rope_rotate(dq_rot, cos, sin, s, nh, inverse=(mut != "rope_forward_instead_of_inverse"))
    good = A.rope_rotate(A.attention_backward(np.concatenate((q, k, v), 1), o, R, lse, s, nh, False)[:, :dd], cos, sin, s, nh, True)
    np.testing.assert_allclose(good, fd, rtol=1e-5, atol=1e-8)
    assert np.abs(bad - fd).max() > 1e-3 * np.abs(fd).max()


def _layer_params(rng, H, F, sig=0.5, dtype=np.float64):
    mk = lambda shape, s_: (s_ * rng.normal(size=shape)).astype(dtype)
    return {"w1": (1.0 + 0.2 * rng.normal(size=H)).astype(dtype), "W_qkv": mk((3 * H, H), sig), "W_o": mk((H, H), sig),
            "w2": (1.0 + 0.2 * rng.normal(size=H)).astype(dtype), "W_gu": mk((2 * F, H), sig), "W_d": mk((H, F), sig)}


def test_layer_chain_finite_differences_across_both_blocks():
    """The hand-on between the blocks (residuals included): gradients of attention-block parameters taken
    through the feed-forward block must match difference quotients of the whole layer."""
    rng = np.random.default_rng(21)
    B, s, nh, dd, F, eps = 1, 4, 1, 4, 6, 1e-3
    T, H = B * s, nh * dd
    p = _layer_params(rng, H, F)
    h, R = rng.normal(size=(T, H)), rng.normal(size=(T, H))
    cos, sin = A.rope_tables(s, dd)
    # unrounded chain, composed from the pieces
    y1 = A.block_forward_f64(h, p["w1"], p["W_qkv"], p["W_o"], cos, sin, s, nh, eps)
    mg = _block_grads_f64(y1, p["w2"], p["W_gu"], p["W_d"], R, eps)
    dmid = mg["dh"]
    xhat, r, xn = M.rmsnorm_forward(h, p["w1"], eps)
    qkv = xn @ p["W_qkv"].T
    q, k = A.rope_rotate(qkv[:, :H], cos, sin, s, nh), A.rope_rotate(qkv[:, H:2 * H], cos, sin, s, nh)
    o, lse = A.attention_forward_f64(q, k, qkv[:, 2 * H:], s, nh)
    do = O.input_grad_f64(dmid, p["W_o"])
    g = A.attention_backward(np.concatenate((q, k, qkv[:, 2 * H:]), 1), o, do, lse, s, nh, round_probabilities=False)
    dqkv = np.concatenate((A.rope_rotate(g[:, :H], cos, sin, s, nh, True), A.rope_rotate(g[:, H:2 * H], cos, sin, s, nh, True),
                           g[:, 2 * H:]), 1)
    dxn = O.input_grad_f64(dqkv, p["W_qkv"])
    got = {"W_o": O.linear_grad(o, dmid), "W_qkv": O.linear_grad(xn, dqkv), "w1": O.vector_grad(xhat, dxn),
           "h": M.rmsnorm_backward(dxn, xhat, r, p["w1"], dres=dmid), "W_d": mg["G_d"], "w2": mg["g_w"]}
    loss = lambda h_, p_: float((A.layer_forward_f64(h_, p_, cos, sin, s, nh, eps) * R).sum())
    e = 1e-6
    for which in ("W_o", "W_qkv", "w1", "W_d", "w2"):
        for idx in list(np.ndindex(p[which].shape))[::2]:
            pp, pm = dict(p), dict(p)
            pp[which], pm[which] = p[which].copy(), p[which].copy()
            pp[which][idx] += e
            pm[which][idx] -= e
            assert (loss(h, pp) - loss(h, pm)) / (2 * e) == pytest.approx(got[which][idx], rel=1e-5, abs=1e-7), (which, idx)
    for idx in np.ndindex(h.shape):
        hp, hm = h.copy(), h.copy()
        hp[idx] += e
        hm[idx] -= e
        assert (loss(hp, p) - loss(hm, p)) / (2 * e) == pytest.approx(got["h"][idx], rel=1e-5, abs=1e-7), idx


def test_layer_step_is_the_generic_step_on_six_tensors():
    rng = np.random.default_rng(22)
    B, s, nh, dd, F = 2, 8, 2, 8, 24
    T, H = B * s, nh * dd
    p = _layer_params(rng, H, F, sig=0.3, dtype=np.float16)
    h = rng.normal(size=(T, H)).astype(np.float16)
    dy = (2.0 * rng.normal(size=(T, H))).astype(np.float16)
    cos, sin = A.rope_tables(s, dd)
    sa, sm = A.layer_forward_stored(h, p, cos, sin, s, nh, 1e-5)
    a = A.layer_step(dy, sa, sm, p, cos, sin, s, nh, 0.05, 256.0)
    recs = [dict(kind="linear", X=sm["a"], dY=dy, W=p["W_d"]), dict(kind="linear", X=sm["xn"], dY=a["mlp"]["dgu"], W=p["W_gu"]),
            dict(kind="vector", X=sm["xhat"], dY=a["mlp"]["dxn"], W=p["w2"]),
            dict(kind="linear", X=sa["o"], dY=a["dh_mid"], W=p["W_o"]), dict(kind="linear", X=sa["xn"], dY=a["attn"]["dqkv"], W=p["W_qkv"]),
            dict(kind="vector", X=sa["xhat"], dY=a["attn"]["dxn"], W=p["w1"])]
    b = O.step_materialised(recs, 0.05, 256.0)
    assert a["clip_coef"] == b["clip_coef"] and a["clip_coef"] < 1.0 and a["flags"] == b["flags"]
    for name, want in zip(A.LAYER_ORDER, b["W"]):
        np.testing.assert_array_equal(a["params"][name].view(np.uint16), want.view(np.uint16))
    # the feed-forward block saw the stored output of the attention block
    np.testing.assert_array_equal(sm["xhat"].shape, sa["y"].shape)


def test_attention_rounding_sensitivity_bounds_a_single_flip():
    """Moving one entry of dS or P by one fp16 ulp moves no output by more than the stated sensitivity."""
    rng = np.random.default_rng(16)
    s, nh, dd = 16, 1, 8
    f16 = lambda shape, sig: (sig * rng.normal(size=shape)).astype(np.float16)
    qkv = np.concatenate((f16((s, dd), 1.0), f16((s, dd), 1.0), f16((s, dd), 1.0)), axis=1)
    att = A.attention_forward_stored(qkv, s, nh)
    do = f16((s, dd), 3.0)
    bound = A.attention_rounding_sensitivity(qkv, att["o"], do, att["lse"], s, nh)
    q, k, v = (O.as_f64(qkv[:, i * dd:(i + 1) * dd]) for i in range(3))
    S = (q @ k.T) / math.sqrt(dd)
    S[np.triu_indices(s, 1)] = -np.inf
    P = np.exp(S - att["lse"].astype(np.float64))
    dS = P * (O.as_f64(do) @ v.T - (O.as_f64(do) * O.as_f64(att["o"])).sum(1, keepdims=True)) / math.sqrt(dd)
    for (i, j) in ((5, 2), (15, 15), (9, 0)):
        bump = np.zeros_like(dS)
        bump[i, j] = abs(dS[i, j]) * 2.0 ** -11                 # at most one ulp of that entry
        assert (np.abs(bump @ k) <= bound[:, :dd] + 1e-300).all() and (np.abs(bump.T @ q) <= bound[:, dd:2 * dd] + 1e-300).all()
        bumpP = np.zeros_like(P)
        bumpP[i, j] = P[i, j] * 2.0 ** -11
        assert (np.abs(bumpP.T @ O.as_f64(do)) <= bound[:, 2 * dd:] + 1e-300).all()


def _small_model(rng, n_layers=2):
    B, s, nh, dd, F, V = 2, 8, 2, 8, 24, 50
    T, H = B * s, nh * dd
    f16 = lambda shape, sig: (sig * rng.normal(size=shape)).astype(np.float16)
    m = {"W_emb": f16((V, H), 1.0), "layers": [_layer_params(rng, H, F, sig=0.3, dtype=np.float16) for _ in range(n_layers)],
         "w_f": (1.0 + 0.1 * rng.normal(size=H)).astype(np.float16), "W_lm": f16((V, H), 0.3)}
    ids = rng.integers(0, V, size=T).astype(np.int32)
    ids[3] = ids[11]                                    # a repeated token: its embedding rows add up
    dlogits = f16((T, V), 2.0)
    cos, sin = A.rope_tables(s, dd)
    saved = A.model_forward_stored(ids, m, cos, sin, s, nh, 1e-5)
    return m, ids, dlogits, cos, sin, saved, s, nh


def _model_records(a, saved, m, ids, dlogits):
    """The model's tensors as records of the generic step, with the hand-on gradients of the walk `a`."""
    f = saved["final"]
    recs = [dict(kind="linear", X=f["xn"], dY=dlogits, W=m["W_lm"]), dict(kind="vector", X=f["xhat"], dY=a["handons"]["dxn_f"], W=m["w_f"])]
    dy = a["handons"]["dy_top"]
    for li, cm, ca in a["per_layer"]:
        p = m["layers"][li]
        sa, sm = saved["layers"][li]
        recs += [dict(kind="linear", X=sm["a"], dY=dy, W=p["W_d"]), dict(kind="linear", X=sm["xn"], dY=cm["dgu"], W=p["W_gu"]),
                 dict(kind="vector", X=sm["xhat"], dY=cm["dxn"], W=p["w2"]), dict(kind="linear", X=sa["o"], dY=cm["dh"], W=p["W_o"]),
                 dict(kind="linear", X=sa["xn"], dY=ca["dqkv"], W=p["W_qkv"]), dict(kind="vector", X=sa["xhat"], dY=ca["dxn"], W=p["w1"])]
        dy = ca["dh"]
    recs.append(dict(kind="embedding", ids=ids, dY=dy, W=m["W_emb"]))
    return recs


def test_model_step_is_the_generic_step_on_all_its_tensors():
    """Two layers, embedding, final norm, output projection: the whole-model oracle equals the generic
    materialised step applied to its tensors with the hand-on gradients of its own walk."""
    m, ids, dlogits, cos, sin, saved, s, nh = _small_model(np.random.default_rng(23))
    a = A.model_step(ids, dlogits, saved, m, cos, sin, s, nh, 0.05, 256.0)
    assert a["names"][0] == "W_lm" and a["names"][-1] == "W_emb" and len(a["names"]) == 2 + 6 * 2 + 1
    b = O.step_materialised(_model_records(a, saved, m, ids, dlogits), 0.05, 256.0)
    assert a["clip_coef"] == b["clip_coef"] and a["flags"] == b["flags"] and a["clip_coef"] < 1.0
    for name, want in zip(a["names"], b["W"]):
        np.testing.assert_array_equal(a["params"][name].view(np.uint16), want.view(np.uint16))
    # the walk really goes from the top to the bottom: the layer-0 hand-on depends on the top gradient
    d2 = dlogits.copy()
    d2[0, 0] = np.float16(float(d2[0, 0]) + 4.0)
    assert (A.model_step(ids, d2, saved, m, cos, sin, s, nh, 0.05, 256.0)["dh0"].view(np.uint16) != a["dh0"].view(np.uint16)).any()


def test_grouped_norm_step_is_the_generic_step_on_each_group():
    """Section 3.3.1, grouped norm: every group is clipped by its own norm.  Each group's parameters must equal
    the generic step applied to that group's tensors alone; the group norms add up (in squares) to the global
    one, so no group's coefficient is below the global coefficient; without clipping nothing differs."""
    m, ids, dlogits, cos, sin, saved, s, nh = _small_model(np.random.default_rng(24), n_layers=3)
    lr, S = 0.05, 256.0
    two = A.model_step(ids, dlogits, saved, m, cos, sin, s, nh, lr, S)
    recs = _model_records(two, saved, m, ids, dlogits)
    for per in (1, 2, 3):
        g = A.model_step_grouped(ids, dlogits, saved, m, cos, sin, s, nh, lr, S, layers_per_group=per)
        want_groups = {1: [[0, 1], [2, 3, 4, 5, 6, 7], [8, 9, 10, 11, 12, 13], [14, 15, 16, 17, 18, 19], [20]],
                       2: [[0, 1], list(range(2, 14)), list(range(14, 20)), [20]],
                       3: [[0, 1], list(range(2, 20)), [20]]}[per]
        assert g["groups"] == want_groups and g["overflow"] is False
        assert abs(math.fsum(n * n for n in g["group_norms"]) / two["norm"] ** 2 - 1) < 1e-12
        assert all(c >= two["clip_coef"] for c in g["group_coefs"]) and len(set(g["group_coefs"])) > 1
        for idx, coef in zip(g["groups"], g["group_coefs"]):
            alone = O.step_materialised([recs[i] for i in idx], lr, S)
            assert alone["clip_coef"] == coef
            for i, want in zip(idx, alone["W"]):
                np.testing.assert_array_equal(g["params"][g["names"][i]].view(np.uint16), want.view(np.uint16))
    free = A.model_step_grouped(ids, dlogits, saved, m, cos, sin, s, nh, lr, S, max_norm=1e30)
    free2 = A.model_step(ids, dlogits, saved, m, cos, sin, s, nh, lr, S, max_norm=1e30)
    for name in free["names"]:
        np.testing.assert_array_equal(free["params"][name].view(np.uint16), free2["params"][name].view(np.uint16))


def test_grouped_norm_overflow_stops_the_walk_updates_from_that_group_on():
    """A non-finite gradient in the middle of the walk: the groups above were updated before it could be known,
    the group itself and every group below keep their bits, and the step reports overflow."""
    m, ids, dlogits, cos, sin, saved, s, nh = _small_model(np.random.default_rng(25), n_layers=3)
    saved["layers"][1][1]["a"][2, 5] = np.inf          # only the gradient of layer 1's W_d sees this activation
    g = A.model_step_grouped(ids, dlogits, saved, m, cos, sin, s, nh, 0.05, 256.0)
    k = g["names"].index("layers.1.W_d")
    assert [i for i, f in enumerate(g["flags"]) if f] == [k]
    assert g["group_overflow"] == [False, False, True, True, True] and g["overflow"] is True
    moved = lambda name, old: (g["params"][name].view(np.uint16) != old.view(np.uint16)).any()
    assert moved("W_lm", m["W_lm"]) and moved("layers.2.W_gu", m["layers"][2]["W_gu"])
    for li in (1, 0):
        for key, old in m["layers"][li].items():
            assert not moved(f"layers.{li}.{key}", old)
    assert not moved("W_emb", m["W_emb"])
    assert A.model_step(ids, dlogits, saved, m, cos, sin, s, nh, 0.05, 256.0)["overflow"] is True


# --------------------------------------------------------------------------- loss (oracle/loss.py)


def test_cross_entropy_against_finite_differences_and_library():
    from oracle import loss as LS
    from scipy.special import log_softmax
    rng = np.random.default_rng(31)
    T, V, S = 7, 24, 512.0
    z = rng.normal(size=(T, V)) * 3.0
    tg = rng.integers(0, V, size=T)
    tg[2] = -100                                       # not counted
    c = LS.cross_entropy(z, tg, S)
    assert c["n"] == T - 1 and c["token_losses"][2] == 0.0 and not c["dlogits"][2].any()
    ls = log_softmax(z, axis=1)
    want = np.array([-ls[t, tg[t]] if tg[t] >= 0 else 0.0 for t in range(T)])
    np.testing.assert_allclose(c["token_losses"], want, rtol=1e-12, atol=1e-12)
    assert abs(c["loss"] - want.sum() / (T - 1)) < 1e-12
    f = lambda zz: S * LS.cross_entropy(zz, tg, S)["loss"]
    for (t, v) in ((0, int(tg[0])), (3, 5), (6, 0), (2, 1)):
        d = np.zeros_like(z)
        d[t, v] = 1e-5
        fd = (f(z + d) - f(z - d)) / 2e-5
        assert abs(fd - c["dlogits"][t, v]) < 1e-5 * S, (t, v)
    np.testing.assert_allclose(c["dlogits"].sum(axis=1), 0.0, atol=1e-9)
    assert all(c["dlogits"][t, tg[t]] < 0 for t in range(T) if tg[t] >= 0)
    u = LS.cross_entropy(np.zeros((3, 16)), [1, 2, 3], 1.0)
    assert abs(u["loss"] - math.log(16)) < 1e-12
    np.testing.assert_allclose(u["dlogits"][0, 0], 1.0 / 16 / 3)
    # a planted mistake (sign of the one-hot term) must fail the finite-difference check
    bad = c["dlogits"].copy()
    bad[0, tg[0]] += 2 * S / (T - 1)
    d = np.zeros_like(z); d[0, tg[0]] = 1e-5
    assert abs((f(z + d) - f(z - d)) / 2e-5 - bad[0, tg[0]]) > 1.0


# --------------------------------------------------------------------------- forward passes (recomputation)


def test_forward_definitions_against_closed_forms_and_brute_force():
    """The forward functions are what a recomputing implementation is compared with, so they are pinned on their
    own: RMSNorm leaves unit mean square (eps = 0); the rotary step makes q . k depend on the distance only;
    attention against a per-token loop with scipy's logsumexp; silu at 0 and far from 0."""
    from scipy.special import logsumexp
    rng = np.random.default_rng(32)
    h = rng.normal(size=(5, 16)) * 3
    xhat, r, xn = M.rmsnorm_forward(h, np.full(16, 2.0), 0.0)
    np.testing.assert_allclose((xhat ** 2).mean(axis=1), 1.0, rtol=1e-12)
    np.testing.assert_allclose(xn, 2 * xhat)
    np.testing.assert_allclose(r, 1 / np.sqrt((h ** 2).mean(axis=1)))
    assert M.silu(np.array([0.0]))[0] == 0.0 and abs(M.silu(np.array([30.0]))[0] - 30.0) < 1e-10
    assert abs(M.silu(np.array([-30.0]))[0]) < 1e-10 and abs(M.silu(np.array([1.0]))[0] - 1 / (1 + math.exp(-1.0))) < 1e-15
    # rotary: the same q and k vector placed at positions (2, 5) and (4, 7) give the same product
    s, d, nh = 8, 8, 1
    cos, sin = A.rope_tables(s, d)
    qv, kv = rng.normal(size=d), rng.normal(size=d)
    q = np.tile(qv, (s, 1)); k = np.tile(kv, (s, 1))
    qr, kr = A.rope_rotate(q, cos, sin, s, nh), A.rope_rotate(k, cos, sin, s, nh)
    assert abs(qr[5] @ kr[2] - qr[7] @ kr[4]) < 1e-6 and abs(qr[5] @ kr[2] - qr[5] @ kr[3]) > 1e-3   # fp32 tables
    np.testing.assert_allclose(qr[0], qv)                       # position 0: no rotation
    # attention: brute force per token
    T, nh, d = 12, 2, 4
    s = 6
    q, k, v = (rng.normal(size=(T, nh * d)) for _ in range(3))
    o, lse = A.attention_forward_f64(q, k, v, s, nh)
    for t in range(T):
        b, i = divmod(t, s)
        for n in range(nh):
            sl = slice(n * d, (n + 1) * d)
            sc = np.array([q[t, sl] @ k[b * s + j, sl] / math.sqrt(d) for j in range(i + 1)])
            assert abs(lse[t, n] - logsumexp(sc)) < 1e-12
            p = np.exp(sc - logsumexp(sc))
            np.testing.assert_allclose(o[t, sl], sum(p[j] * v[b * s + j, sl] for j in range(i + 1)), atol=1e-12)


def test_stored_forward_is_the_definition_up_to_fp16_storage():
    """What the stored (fp16) forward leaves behind differs from the fp64 definition by storage rounding only."""
    rng = np.random.default_rng(33)
    B, s, nh, dd, F = 2, 8, 2, 8, 24
    T, H = B * s, nh * dd
    p = _layer_params(rng, H, F, sig=0.3, dtype=np.float16)
    h = (rng.normal(size=(T, H))).astype(np.float16)
    cos, sin = A.rope_tables(s, dd)
    sa, sm = A.layer_forward_stored(h, p, cos, sin, s, nh, 1e-5)
    y1 = A.block_forward_f64(h, p["w1"], p["W_qkv"], p["W_o"], cos, sin, s, nh, 1e-5)
    assert np.abs(sa["y"].astype(np.float64) - y1).max() < 2.0 ** -8 * np.abs(y1).max()
    y2 = M.block_forward_f64(sa["y"], p["w2"], p["W_gu"], p["W_d"], 1e-5)
    got = sa["y"].astype(np.float64) + sm["a"].astype(np.float64) @ p["W_d"].astype(np.float64).T
    assert np.abs(got - y2).max() < 2.0 ** -8 * np.abs(y2).max()
    # saved pieces against their definitions on the stored inputs
    xhat, r, _ = M.rmsnorm_forward(h, p["w1"], 1e-5)
    assert (O.ulp_distance_f16(sa["xhat"], O.round_f16(xhat)) == 0).all() and np.allclose(sa["r"], r, rtol=1e-6)
    o64, lse64 = A.attention_forward_f64(sa["qkv"][:, :H].astype(np.float64), sa["qkv"][:, H:2 * H].astype(np.float64),
                                         sa["qkv"][:, 2 * H:].astype(np.float64), s, nh)
    assert np.abs(sa["lse"] - lse64).max() < 1e-5 and np.abs(sa["o"].astype(np.float64) - o64).max() < 2.0 ** -9 * np.abs(o64).max()


def test_training_steps_learn_a_repeated_batch_and_follow_the_scaler_protocol():
    """Section 3.3.2's protocol around Algorithm 1: overflow -> step dropped, scale halved; growth_interval clean
    steps -> scale doubled; and the method as a whole trains (the loss on a repeated batch goes down)."""
    from oracle import training as TR
    m, ids, dlogits, cos, sin, saved, s, nh = _small_model(np.random.default_rng(35))
    targets = np.roll(ids, -1).astype(np.int32)
    targets[s - 1::s] = -100
    n = int((targets >= 0).sum())
    S0 = 2.0 ** 20                      # S0 / n > 65504: the target entries of the fp16 loss gradient overflow
    assert S0 / n > 65504
    final, log = TR.training_steps(ids, targets, m, cos, sin, s, nh, 1e-5, 12, 0.05, S0, 2)
    assert log[0]["overflow"] and sum(r["overflow"] for r in log) >= 3 and sum(not r["overflow"] for r in log) >= 6
    clean = 0
    for a, b in zip(log, log[1:]):
        if a["overflow"]:
            assert b["loss_scale"] == a["loss_scale"] / 2 and b["loss"] == a["loss"]        # dropped: nothing moved
            clean = 0
        else:
            clean += 1
            assert b["loss"] < a["loss"]                                                     # a step that counts learns
            assert b["loss_scale"] == (a["loss_scale"] * 2 if clean == 2 else a["loss_scale"])
            clean %= 2
    assert log[-1]["loss"] < 0.85 * log[0]["loss"]
    assert any((final["layers"][0][k].view(np.uint16) != m["layers"][0][k].view(np.uint16)).any() for k in m["layers"][0])
    # the loss of a step does not depend on the scale: the same run at a safe constant scale gives the same losses
    # on its clean steps, up to the rounding of differently scaled fp16 gradients
    _, calm = TR.training_steps(ids, targets, m, cos, sin, s, nh, 1e-5, 4, 0.05, 1024.0, 1000)
    assert not any(r["overflow"] for r in calm)
    kept = [r["loss"] for r in log if not r["overflow"]]
    for a, b in zip(kept, [r["loss"] for r in calm]):
        assert abs(a - b) < 2e-3 * abs(b)
    # grouped norm: different step sizes (never smaller than the global one's), still learning
    _, g = TR.training_steps(ids, targets, m, cos, sin, s, nh, 1e-5, 3, 0.05, 1024.0, 1000, grouped=True)
    assert g[2]["loss"] < g[1]["loss"] < g[0]["loss"] and g[1]["loss"] <= calm[1]["loss"] + 1e-9
