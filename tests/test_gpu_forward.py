"""Forward steps (activation recomputation) and the loss on the GPU against the oracle's forward definitions.

Bars.  Element-wise steps and contractions: within 1 fp16 ulp on >= 99.9 %, none beyond 2 ulp (a contraction may
instead sit within 2^-20 of the sum of its terms' magnitudes where the terms cancel).  Attention output: the kernel
rounds its probabilities to fp16 relative to the running maximum, the oracle relative to the final normaliser,
so an element may move by 2^-11 of the probability-weighted sum of |v|: within 1 ulp on >= 99 %, and everywhere
within 2 ulp or 2^-10 * sum_j P_ij |v_jc|.  lse: 1e-5.  Loss gradient: 1 ulp / 2 ulp bar; token losses 1e-5.
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

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T,K,N,acc", [(256, 256, 768, False), (200, 136, 344, False), (64, 344, 256, True),
                                       (2048, 512, 4096, False), (4096, 1024, 2048, True), (1, 8, 8, False),
                                       (4096, 256, 3072, False), (4096, 128, 3072, True)])
def test_linear_forward(L, T, K, N, acc):
    rng = np.random.default_rng(T + K + N)
    X, W = f16(rng, (T, K), 1.0), f16(rng, (N, K), 0.05)
    R = f16(rng, (T, N), 1.0)
    Y = dev(R) if acc else torch.full((T, N), 7.0, dtype=torch.float16, device=DEV)
    L.lomo_linear_forward(dev(X), dev(W), Y, accumulate=acc)
    ref = f64(X) @ f64(W).T + (f64(R) if acc else 0.0)
    mag = np.abs(f64(X)) @ np.abs(f64(W)).T + (np.abs(f64(R)) if acc else 0.0)
    got = Y.cpu().numpy()
    ulps_ok(got, O.round_f16(ref), f"Y {T}x{K}x{N}", near=np.abs(f64(got) - ref) <= 2.0 ** -20 * mag)


@pytest.mark.parametrize("T,K,N", [(64, 344, 256), (4096, 128, 3072)])
def test_linear_forward_residual_from_its_own_buffer(L, T, K, N):
    rng = np.random.default_rng(T + K + N + 1)
    X, W, R = f16(rng, (T, K), 1.0), f16(rng, (N, K), 0.05), f16(rng, (T, N), 1.0)
    dR = dev(R)
    Y = torch.full((T, N), 7.0, dtype=torch.float16, device=DEV)
    L.lomo_linear_forward_residual(dev(X), dev(W), dR, Y)
    Y2 = dev(R)
    L.lomo_linear_forward(dev(X), dev(W), Y2, accumulate=True)
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16)) and torch.equal(dR.view(torch.int16), dev(R).view(torch.int16))
    ref = f64(X) @ f64(W).T + f64(R)
    got = Y.cpu().numpy()
    ulps_ok(got, O.round_f16(ref), "Y", near=np.abs(f64(got) - ref) <= 2.0 ** -20 * (np.abs(f64(X)) @ np.abs(f64(W)).T + np.abs(f64(R))))


def test_linear_forward_rejects_bad_arguments(L):
    import ctypes
    lib = L.load_library()
    z = ctypes.c_void_p(0)
    assert lib.lomo_linear_forward(z, z, z, 8, 12, 8, 0, z) == 2          # K % 8
    assert lib.lomo_linear_forward(z, z, z, 8, 8, 8, 0, z) == 1           # null
    assert lib.lomo_linear_forward(z, z, z, 0, 8, 8, 0, z) == 0           # empty


@pytest.mark.parametrize("T,H", [(64, 256), (37, 4096), (5, 8)])
def test_rmsnorm_forward(L, T, H):
    rng = np.random.default_rng(T + H)
    h = f16(rng, (T, H), 2.0)
    w = (1.0 + 0.1 * rng.standard_normal(H)).astype(np.float16)
    xhat = torch.empty(T, H, dtype=torch.float16, device=DEV)
    xn = torch.empty_like(xhat)
    rstd = torch.empty(T, dtype=torch.float32, device=DEV)
    L.lomo_rmsnorm_forward(dev(h), dev(w), 1e-5, xhat, rstd, xn)
    x64, r64, _ = M.rmsnorm_forward(h, w, 1e-5)
    np.testing.assert_allclose(rstd.cpu().numpy(), r64, rtol=3e-7)
    got = xhat.cpu().numpy()
    ulps_ok(got, O.round_f16(x64), "xhat", worst=1)
    # xn is defined on the stored xhat: exact on the device's own bits
    want_xn = O.round_f16(f64(got) * f64(w)[None, :])
    assert (O.ulp_distance_f16(xn.cpu().numpy(), want_xn) == 0).all()


def test_swiglu_forward(L):
    rng = np.random.default_rng(3)
    T, F = 50, 344
    gu = f16(rng, (T, 2 * F), 2.0)
    gu[0, :4] = [0.0, 30.0, -30.0, -11.0]
    a = torch.empty(T, F, dtype=torch.float16, device=DEV)
    L.lomo_swiglu_forward(dev(gu), a)
    want = M.silu(f64(gu[:, :F])) * f64(gu[:, F:])
    ulps_ok(a.cpu().numpy(), O.round_f16(want), "a", worst=1)


def test_rope_forward(L):
    rng = np.random.default_rng(4)
    B, s, nh = 3, 64, 2
    T, H = B * s, nh * 128
    qkv = f16(rng, (T, 3 * H), 1.0)
    cos, sin = A.rope_tables(s, 128)
    d = dev(qkv)
    L.lomo_rope_forward(d, dev(cos), dev(sin), s, nh)
    got = d.cpu().numpy()
    for part in (0, 1):
        want = A.rope_rotate(qkv[:, part * H:(part + 1) * H], cos, sin, s, nh)
        ulps_ok(got[:, part * H:(part + 1) * H], O.round_f16(want), "q" if part == 0 else "k", worst=1)
    np.testing.assert_array_equal(got[:, 2 * H:].view(np.uint16), qkv[:, 2 * H:].view(np.uint16))


def attention_reference(qkv, s, nh):
    """o (fp64, from unrounded probabilities), lse, and sum_j P_ij |v_jc| for the error bar."""
    T, H3 = qkv.shape
    H = H3 // 3
    q, k, v = (f64(qkv[:, i * H:(i + 1) * H]) for i in range(3))
    o, lse = A.attention_forward_f64(q, k, v, s, nh)
    mag, _ = A.attention_forward_f64(q, k, np.abs(v), s, nh)
    return o, lse, mag


@pytest.mark.parametrize("B,s,nh,sharp", [(1, 64, 1, 1.0), (2, 128, 2, 1.0), (1, 256, 1, 3.0), (3, 192, 2, 0.3), (1, 512, 2, 1.0)])
def test_attention_forward(L, B, s, nh, sharp):
    rng = np.random.default_rng(B * 1000 + s + nh)
    T, H = B * s, nh * 128
    qkv = np.concatenate((f16(rng, (T, H), sharp), f16(rng, (T, H), 1.0), f16(rng, (T, H), 1.0)), axis=1)
    o = torch.full((T, H), 9.0, dtype=torch.float16, device=DEV)
    lse = torch.empty(T, nh, dtype=torch.float32, device=DEV)
    L.lomo_attention_forward(dev(qkv), o, lse, B, s, nh)
    torch.cuda.synchronize()
    want, want_lse, mag = attention_reference(qkv, s, nh)
    np.testing.assert_allclose(lse.cpu().numpy(), want_lse, rtol=1e-5, atol=1e-5)
    got = o.cpu().numpy()
    d = O.ulp_distance_f16(got, O.round_f16(want))
    near = np.abs(f64(got) - want) <= 2.0 ** -10 * mag
    assert ((d <= 2) | near).all(), d[~((d <= 2) | near)].max()
    assert ((d <= 1) | (np.abs(f64(got) - want) <= 2.0 ** -12 * mag)).mean() >= 0.99
    # and against the oracle's stored forward (fp16 probabilities relative to the final normaliser)
    st = A.attention_forward_stored(qkv, s, nh)
    both = (O.ulp_distance_f16(got, st["o"]) <= 2) | (np.abs(f64(got) - f64(st["o"])) <= 2.0 ** -9 * mag)
    assert both.all()          # two sets of fp16 probability roundings apart


def test_attention_forward_feeds_the_backward(L):
    """o and lse from the forward kernel, handed to the backward kernel, give the gradients of the oracle's chain."""
    rng = np.random.default_rng(8)
    B, s, nh = 2, 128, 2
    T, H = B * s, nh * 128
    qkv = np.concatenate((f16(rng, (T, H), 1.0), f16(rng, (T, H), 1.0), f16(rng, (T, H), 1.0)), axis=1)
    do = f16(rng, (T, H), 3.0)
    o = torch.empty(T, H, dtype=torch.float16, device=DEV)
    lse = torch.empty(T, nh, dtype=torch.float32, device=DEV)
    dq = dev(qkv)
    L.lomo_attention_forward(dq, o, lse, B, s, nh)
    delta = torch.empty(T * nh, dtype=torch.float32, device=DEV)
    out = torch.empty(T, 3 * H, dtype=torch.float16, device=DEV)
    L.lomo_attention_backward(dq, o, dev(do), lse, None, None, delta, out, B, s, nh)
    st = A.attention_forward_stored(qkv, s, nh)
    g = A.attention_backward(qkv, st["o"], do, st["lse"], s, nh)
    rel = np.linalg.norm(f64(out.cpu().numpy()) - g) / np.linalg.norm(g)
    assert rel < 2.0 ** -10, rel


@pytest.mark.parametrize("T,V", [(64, 512), (33, 32000), (4, 8)])
def test_cross_entropy(L, T, V):
    rng = np.random.default_rng(T + V)
    z = f16(rng, (T, V), 3.0)
    tg = rng.integers(0, V, size=T).astype(np.int32)
    tg[1] = -100
    if T > 2:
        tg[2] = V                                   # out of range on the other side: not counted either
    S = 4096.0
    want = LS.cross_entropy(z, tg, S)
    loss = torch.empty(T, dtype=torch.float32, device=DEV)
    dz = torch.full((T, V), 5.0, dtype=torch.float16, device=DEV)
    L.lomo_cross_entropy(dev(z), dev(tg), S / want["n"], loss, dz)
    np.testing.assert_allclose(loss.cpu().numpy(), want["token_losses"], rtol=1e-5, atol=1e-5)
    got = dz.cpu().numpy()
    ulps_ok(got, want["dlogits_f16"], "dlogits", near=np.abs(f64(got) - want["dlogits"]) <= 2.0 ** -24 * S / want["n"])
    assert not got[1].any()
    # in place: the gradient may overwrite the logits
    zz = dev(z)
    L.lomo_cross_entropy(zz, dev(tg), S / want["n"], loss, zz)
    np.testing.assert_array_equal(zz.cpu().numpy().view(np.uint16), got.view(np.uint16))


def test_forward_entry_points_check_their_arguments(L):
    """Empty problems succeed without touching memory; wrong shapes and null pointers are refused before any launch."""
    import ctypes
    lib = L.load_library()
    z = ctypes.c_void_p(0)
    f = ctypes.c_float
    assert lib.lomo_rmsnorm_forward(z, z, f(1e-5), z, z, z, 0, 256, z) == 0
    assert lib.lomo_rmsnorm_forward(z, z, f(1e-5), z, z, z, 4, 12, z) == 2            # H % 8
    assert lib.lomo_rmsnorm_forward(z, z, f(-1.0), z, z, z, 4, 16, z) == 2            # negative eps
    assert lib.lomo_rmsnorm_forward(z, z, f(1e-5), z, z, z, 4, 16, z) == 1            # null
    assert lib.lomo_swiglu_forward(z, z, 0, 64, z) == 0 and lib.lomo_swiglu_forward(z, z, 4, 12, z) == 2
    assert lib.lomo_swiglu_forward(z, z, 4, 16, z) == 1
    assert lib.lomo_rope_forward(z, z, z, 0, 64, 2, 128, z) == 0
    assert lib.lomo_rope_forward(z, z, z, 64, 64, 2, 64, z) == 2                      # head width
    assert lib.lomo_rope_forward(z, z, z, 64, 64, 2, 128, z) == 1
    assert lib.lomo_attention_forward(z, z, z, 0, 64, 2, 128, z) == 0
    assert lib.lomo_attention_forward(z, z, z, 1, 100, 2, 128, z) == 2                # s % 64
    assert lib.lomo_attention_forward(z, z, z, 1, 64, 2, 64, z) == 2
    assert lib.lomo_attention_forward(z, z, z, 1, 64, 2, 128, z) == 1
    assert lib.lomo_cross_entropy(z, z, f(1.0), z, z, 0, 512, z) == 0
    assert lib.lomo_cross_entropy(z, z, f(1.0), z, z, 4, 12, z) == 2 and lib.lomo_cross_entropy(z, z, f(1.0), z, z, 4, 0, z) == 2
    assert lib.lomo_cross_entropy(z, z, f(1.0), z, z, 4, 16, z) == 1
    assert lib.lomo_embedding_forward(z, z, z, 0, 64, 100, z) == 0 and lib.lomo_embedding_forward(z, z, z, 4, 12, 100, z) == 2
    assert lib.lomo_embedding_forward(z, z, z, 4, 16, 100, z) == 1
    assert lib.lomo_linear_forward_residual(z, z, z, z, 4, 16, 16, z) == 1 and lib.lomo_linear_forward_residual(z, z, z, z, 4, 12, 16, z) == 2
    # misaligned pointers
    buf = torch.zeros(4096, dtype=torch.float16, device=DEV)
    p, q = ctypes.c_void_p(buf.data_ptr()), ctypes.c_void_p(buf.data_ptr() + 2)
    assert lib.lomo_swiglu_forward(q, p, 4, 16, z) == 3
    assert lib.lomo_linear_forward(p, p, q, 4, 16, 16, 0, z) == 3


def test_embedding_forward(L):
    rng = np.random.default_rng(9)
    T, H, V = 70, 136, 50
    W = f16(rng, (V, H), 1.0)
    ids = rng.integers(0, V, size=T).astype(np.int32)
    ids[5], ids[6] = -1, V                      # out of range: zero rows
    h = torch.full((T, H), 3.0, dtype=torch.float16, device=DEV)
    L.lomo_embedding_forward(dev(ids), dev(W), h)
    want = np.where(((ids >= 0) & (ids < V))[:, None], W[np.clip(ids, 0, V - 1)], np.float16(0))
    np.testing.assert_array_equal(h.cpu().numpy().view(np.uint16), want.view(np.uint16))
