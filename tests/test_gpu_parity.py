"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Tolerances (written here, as the workload statement fixes them):
  * overflow flags and embedding grouping: bit exact;
  * squared norm / gradient norm: relative error <= 1e-3 (observed ~1e-6);
  * updated fp16 weights: within 1 fp16 ulp of the oracle on >= 99.9 % of elements, none beyond 2;
  * dX: same bar, plus a cancellation guard of 2^-20 * sum_n |dY||W|.
Because clipped updates are mostly far below one ulp, every shape is also run with a "visible"
step (clip = 1, lr chosen so the typical update is tens of ulps) and the set of changed
elements is compared with the oracle's.
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


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def gen(seed, shape, sigma):
    return S.normal_f16_np(S.tensor_key(seed, 7, 3, len(shape) + int(sigma * 1000) % 97), shape, S.normal_mult(sigma))


def assert_weights_close(got16, want16, what=""):
    d = O.ulp_distance_f16(got16, want16)
    assert np.isfinite(got16.astype(np.float32)).all(), what
    frac1 = float((d <= 1).mean())
    assert d.max() <= 2, f"{what}: max ulp distance {d.max()}"
    assert frac1 >= 0.999, f"{what}: only {frac1:.5f} within 1 ulp"
    return float((d == 0).mean())


def assert_dx_close(got16, dY, W, what=""):
    ref64 = O.input_grad_f64(dY, W)
    want16 = O.round_f16(ref64)
    d = O.ulp_distance_f16(got16, want16)
    guard = 2.0 ** -20 * (np.abs(dY.astype(np.float64)) @ np.abs(W.astype(np.float64)))
    ok = (d <= 2) | (np.abs(got16.astype(np.float64) - ref64) <= guard)
    assert ok.all(), f"{what}: dX off by {d.max()} ulp"
    assert float(((d <= 1) | (np.abs(got16.astype(np.float64) - ref64) <= guard)).mean()) >= 0.999, what


LINEAR_SHAPES = [
    (512, 1024, 1024),     # the single-layer workload: 64 tiles of 128 x 128
    (100, 264, 136),       # ragged in every dimension
    (33, 8, 8),            # one partial tile
    (1, 520, 1032),        # a single token: rank-one gradient
    (300, 776, 392),
    (70, 3600, 3320),      # 15 x 13 tiles of 256 x 256, ragged tails
    (64, 4096, 4096),      # 256 full 256 x 256 tiles
    # edges of the persistent 256 x 256 x 32 kernels: the shortest contraction they take (one round of their four
    # stages) and an odd number of rounds, the smallest tile count they take (192), for the weight gradient ...
    (128, 4096, 4096),
    (384, 3072, 4096),
    # ... and for dgrad (tokens are the tile rows there, N is contracted)
    (3328, 3840, 128),
    (3328, 3840, 384),
]


@pytest.mark.parametrize("T,K,N", LINEAR_SHAPES)
def test_linear_sqnorm_update_dgrad(L, T, K, N):
    Sc = 1024.0
    sig_dy = 0.01
    X = gen(1, (T, K), 1.0)
    dY = S.normal_f16_np(S.tensor_key(2, T, K, N), (T, N), S.normal_mult(sig_dy, Sc))
    W = S.normal_f16_np(S.tensor_key(3, T, K, N), (N, K), S.normal_mult(0.02))
    G = O.linear_grad(X, dY)

    # pass 1
    acc = torch.zeros(1, dtype=torch.float64, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    dXd, dYd = dev(X), dev(dY)
    L.lomo_wgrad_sqnorm(dXd, dYd, acc, flag)
    L.lomo_wgrad_sqnorm(dXd, dYd, acc, flag)           # accumulates: twice the norm
    want = O.sqnorm(G)
    assert float(acc.item()) == pytest.approx(2 * want, rel=1e-3)
    assert abs(float(acc.item()) / (2 * want) - 1) < 2e-5
    assert int(flag.item()) == 0

    # pass 2, visible step: typical |delta| about 30 ulp of a 0.02-sized weight
    lr = float(np.float32(30 * 2.0 ** -16 / (math.sqrt(T) * sig_dy)))
    Wd = dev(W)
    dX = torch.empty(T, K, dtype=torch.float16, device=DEV)
    L.lomo_linear_backward_update(dXd, dYd, Wd, dX, lr, 1.0 / Sc, 1.0, flag)
    got = host(Wd)
    wantW = O.sgd_update(W, G, lr, 1.0, Sc)
    exact = assert_weights_close(got, wantW, f"W {T}x{K}x{N}")
    assert exact > 0.98
    changed_o = wantW.view(np.uint16) != W.view(np.uint16)
    changed_g = got.view(np.uint16) != W.view(np.uint16)
    assert changed_o.mean() > 0.9 and (changed_o != changed_g).mean() < 1e-3
    assert_dx_close(host(dX), dY, W, f"dX {T}x{K}x{N}")

    # clipped step of the workload description (tiny update) from the same start
    coef = O.clip_coef(O.grad_norm(want, Sc))
    Wd2 = dev(W)
    L.lomo_linear_backward_update(dXd, dYd, Wd2, None, 1e-2, 1.0 / Sc, float(np.float32(coef)), None)
    assert_weights_close(host(Wd2), O.sgd_update(W, G, float(np.float32(1e-2)), float(np.float32(coef)), Sc), "clipped")


def _random_linear_shapes():
    """Seeded shapes around the boundaries between the three contraction kernels: ragged ones for the guarded kernel,
    multiples of 128 for the whole-tile kernel, and a few with 256-multiples and token counts next to a multiple of 64."""
    rng = np.random.default_rng(20240611)
    shapes = []
    for _ in range(10):
        shapes.append((int(rng.integers(1, 400)), 8 * int(rng.integers(1, 130)), 8 * int(rng.integers(1, 130))))
    for _ in range(6):
        shapes.append((64 * int(rng.integers(1, 6)), 128 * int(rng.integers(1, 9)), 128 * int(rng.integers(1, 9))))
    for _ in range(4):
        shapes.append((64 * int(rng.integers(2, 5)) + int(rng.integers(-1, 2)), 256 * int(rng.integers(1, 5)), 256 * int(rng.integers(1, 5))))
    return shapes


@pytest.mark.parametrize("T,K,N", _random_linear_shapes())
def test_linear_random_shapes(L, T, K, N):
    """Norm, visible update and dX on seeded random shapes, element by element against the oracle."""
    Sc = 256.0
    X = S.normal_f16_np(S.tensor_key(71, T, K, N), (T, K), S.normal_mult(1.0))
    dY = S.normal_f16_np(S.tensor_key(72, T, K, N), (T, N), S.normal_mult(0.01, Sc))
    W = S.normal_f16_np(S.tensor_key(73, T, K, N), (N, K), S.normal_mult(0.02))
    G = O.linear_grad(X, dY)
    acc = torch.zeros(1, dtype=torch.float64, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    Xd, dYd, Wd = dev(X), dev(dY), dev(W)
    L.lomo_wgrad_sqnorm(Xd, dYd, acc, flag)
    assert abs(float(acc.item()) / O.sqnorm(G) - 1) < 2e-5 and int(flag.item()) == 0
    lr = float(np.float32(30 * 2.0 ** -16 / (math.sqrt(T) * 0.01)))
    dX = torch.empty(T, K, dtype=torch.float16, device=DEV)
    L.lomo_linear_backward_update(Xd, dYd, Wd, dX, lr, 1.0 / Sc, 1.0, flag)
    assert_weights_close(host(Wd), O.sgd_update(W, G, lr, 1.0, Sc), f"W {T}x{K}x{N}")
    assert_dx_close(host(dX), dY, W, f"dX {T}x{K}x{N}")


def test_dgrad_reads_weights_before_the_update(L):
    T, K, N = 96, 512, 256
    X, dY, W = gen(4, (T, K), 1.0), gen(5, (T, N), 0.5), gen(6, (N, K), 0.02)
    Wd, dX = dev(W), torch.empty(T, K, dtype=torch.float16, device=DEV)
    L.lomo_linear_backward_update(dev(X), dev(dY), Wd, dX, 0.5, 1.0, 1.0, None)    # a huge step
    assert_dx_close(host(dX), dY, W, "dX before update")
    after = O.input_grad(dY, host(Wd))
    assert (O.ulp_distance_f16(host(dX), after) > 4).mean() > 0.5


@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
@pytest.mark.parametrize("where", ["X", "dY"])
def test_overflow_flag_and_skip(L, bad, where):
    T, K, N = 130, 264, 520
    X, dY, W = gen(7, (T, K), 1.0), gen(8, (T, N), 1.0), gen(9, (N, K), 0.02)
    (X if where == "X" else dY)[T - 1, 5] = bad
    assert O.has_overflow(O.linear_grad(X, dY))
    acc = torch.zeros(1, dtype=torch.float64, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    L.lomo_wgrad_sqnorm(dev(X), dev(dY), acc, flag)
    assert int(flag.item()) == 1
    Wd, dX = dev(W), torch.zeros(T, K, dtype=torch.float16, device=DEV)
    L.lomo_linear_backward_update(dev(X), dev(dY), Wd, dX, 0.1, 1.0, 1.0, flag)
    np.testing.assert_array_equal(host(Wd).view(np.uint16), W.view(np.uint16))     # step dropped
    assert host(dX).any()                                                           # dgrad still ran


def test_loss_scale_invariance_on_device(L):
    T, K, N = 200, 520, 264
    X, W = gen(10, (T, K), 1.0), gen(11, (N, K), 0.02)
    dY = S.normal_f16_np(S.tensor_key(12, 0, 0, 0), (T, N), S.normal_mult(0.01, 256.0))
    dY2 = (dY.astype(np.float32) * 2).astype(np.float16)
    outs = []
    for d, Sc in ((dY, 256.0), (dY2, 512.0)):
        Wd = dev(W)
        L.lomo_linear_backward_update(dev(X), dev(d), Wd, None, 0.02, 1.0 / Sc, 1.0, None)
        outs.append(host(Wd).view(np.uint16))
    np.testing.assert_array_equal(outs[0], outs[1])
    assert (outs[0] != W.view(np.uint16)).mean() > 0.5


def test_lr_zero_keeps_weights(L):
    T, K, N = 64, 136, 72
    X, dY, W = gen(13, (T, K), 1.0), gen(14, (T, N), 1.0), gen(15, (N, K), 0.02)
    Wd = dev(W)
    L.lomo_linear_backward_update(dev(X), dev(dY), Wd, None, 0.0, 1.0, 1.0, None)
    np.testing.assert_array_equal(host(Wd).view(np.uint16), W.view(np.uint16))


# ------------------------------------------------------------------------------- embedding


def _emb_case(T, V, H, mode, seed=0):
    rng = np.random.default_rng(seed)
    if mode == "zipf":
        ids = S.zipf_ids(seed, T, V)
    elif mode == "same":
        ids = np.full(T, V // 3, np.int32)
    elif mode == "distinct":
        ids = rng.permutation(V)[:T].astype(np.int32)
    else:
        ids = rng.integers(0, V, size=T).astype(np.int32)
    dY = S.normal_f16_np(S.tensor_key(seed, T, V, H), (T, H), S.normal_mult(0.05, 64.0))
    W = S.normal_f16_np(S.tensor_key(seed + 1, T, V, H), (V, H), S.normal_mult(0.02))
    return ids, dY, W


EMB_CASES = [(4096, 32000, 512, "zipf"), (0, 50, 64, "uniform"), (1, 50, 64, "uniform"), (2, 50, 64, "same"),
             (777, 100, 72, "uniform"), (300, 1000, 2056, "distinct"), (513, 40, 4096, "same"),
             (20000, 5000, 64, "zipf"), (8192, 32000, 128, "zipf"), (8193, 300, 8, "uniform"),
             # above 8192 positions: sorted chunks + merge rounds (one, two and three rounds; a last chunk of one
             # position; heavy ties), and ids too wide for 32-bit keys (the bitonic route, below and above 8192)
             (65536, 32000, 64, "zipf"), (30000, 200000, 8, "uniform"), (24577, 3, 8, "uniform"),
             (16384, 1000, 8, "same"), (5000, 1500000, 8, "uniform"), (9000, 1500000, 8, "uniform")]


@pytest.mark.parametrize("T,V,H,mode", EMB_CASES)
def test_embedding_grouping_norm_update(L, T, V, H, mode):
    ids, dY, W = _emb_case(T, V, H, mode)
    wsb = L.lomo_embedding_workspace_bytes(T, H)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device=DEV)
    idd = dev(ids) if T else torch.empty(0, dtype=torch.int32, device=DEV)
    dYd = dev(dY) if T else torch.empty(0, H, dtype=torch.float16, device=DEV)

    u = torch.full((max(T, 1),), -1, dtype=torch.int32, device=DEV)
    off = torch.full((T + 1,), -1, dtype=torch.int32, device=DEV)
    perm = torch.full((max(T, 1),), -1, dtype=torch.int32, device=DEV)
    nu = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    L.lomo_embedding_grouping(idd, V, ws, u, off, perm, nu)
    ou, ooff, operm = O.embedding_grouping(ids)
    n = int(nu.item())
    assert n == ou.size
    np.testing.assert_array_equal(host(u)[:n], ou)
    np.testing.assert_array_equal(host(off)[:n + 1], ooff)
    np.testing.assert_array_equal(host(perm)[:T], operm)

    G = O.embedding_grad(ids, dY, V)
    acc = torch.zeros(1, dtype=torch.float64, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    L.lomo_embedding_sqnorm(idd, dYd, V, ws, acc, flag)
    want = O.sqnorm(G)
    assert float(acc.item()) == pytest.approx(want, rel=2e-5, abs=1e-30)
    assert int(flag.item()) == 0

    Wd = dev(W)
    lr, Sc = 0.01, 64.0
    L.lomo_embedding_update(idd, dYd, Wd, lr, 1.0 / Sc, 1.0, ws, flag)
    got = host(Wd)
    wantW = O.sgd_update(W, G, float(np.float32(lr)), 1.0, Sc)
    assert_weights_close(got, wantW, "embedding rows")
    absent = np.setdiff1d(np.arange(V), ids)
    np.testing.assert_array_equal(got[absent].view(np.uint16), W[absent].view(np.uint16))
    if T:
        assert (got[ids[0]].view(np.uint16) != W[ids[0]].view(np.uint16)).any()

    # run-to-run determinism: bit-identical rows
    Wd2 = dev(W)
    L.lomo_embedding_update(idd, dYd, Wd2, lr, 1.0 / Sc, 1.0, ws, flag)
    np.testing.assert_array_equal(host(Wd2).view(np.uint16), got.view(np.uint16))


def test_embedding_overflow(L):
    ids, dY, W = _emb_case(300, 64, 136, "uniform", seed=3)
    dY[17, 9] = np.inf
    dY[18, 9] = -np.inf
    ws = torch.empty(L.lomo_embedding_workspace_bytes(300, 136), dtype=torch.uint8, device=DEV)
    acc = torch.zeros(1, dtype=torch.float64, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    L.lomo_embedding_sqnorm(dev(ids), dev(dY), 64, ws, acc, flag)
    assert int(flag.item()) == 1 and O.has_overflow(O.embedding_grad(ids, dY, 64))
    Wd = dev(W)
    L.lomo_embedding_update(dev(ids), dev(dY), Wd, 0.1, 1.0, 1.0, ws, flag)
    np.testing.assert_array_equal(host(Wd).view(np.uint16), W.view(np.uint16))


# ------------------------------------------------------------------------------- gain vectors


@pytest.mark.parametrize("T,H", [(4096, 4096), (1, 64), (257, 72), (1000, 5120), (0, 64), (20000, 136)])
def test_vector_norm_update(L, T, H):
    Sc = 64.0
    xh = S.normal_f16_np(S.tensor_key(20, T, H, 0), (T, H), S.normal_mult(1.0))
    dY = S.normal_f16_np(S.tensor_key(21, T, H, 0), (T, H), S.normal_mult(1e-3, Sc))
    w = np.ones(H, np.float16)
    g = O.vector_grad(xh, dY) if T else np.zeros(H)
    ws = torch.empty(max(L.lomo_vector_workspace_bytes(T, H), 256), dtype=torch.uint8, device=DEV)
    acc = torch.zeros(1, dtype=torch.float64, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    xd = dev(xh) if T else torch.empty(0, H, dtype=torch.float16, device=DEV)
    dd = dev(dY) if T else torch.empty(0, H, dtype=torch.float16, device=DEV)
    L.lomo_vector_sqnorm(xd, dd, ws, acc, flag)
    assert float(acc.item()) == pytest.approx(O.sqnorm(g), rel=2e-5, abs=1e-30)
    assert int(flag.item()) == 0
    wd = dev(w)
    lr = 30.0 / max(1.0, math.sqrt(T))       # typical |delta| about 30 ulp of 1.0
    L.lomo_vector_update(xd, dd, wd, lr, 1.0 / Sc, 1.0, ws, flag)
    got = host(wd)
    assert_weights_close(got, O.sgd_update(w, g, float(np.float32(lr)), 1.0, Sc), "gain")
    if T:
        assert (got.view(np.uint16) != w.view(np.uint16)).mean() > 0.5


def test_vector_overflow(L):
    T, H = 300, 264
    xh, dY = gen(22, (T, H), 1.0), gen(23, (T, H), 1.0)
    xh[299, 263] = np.nan
    ws = torch.empty(L.lomo_vector_workspace_bytes(T, H), dtype=torch.uint8, device=DEV)
    acc = torch.zeros(1, dtype=torch.float64, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    L.lomo_vector_sqnorm(dev(xh), dev(dY), ws, acc, flag)
    assert int(flag.item()) == 1
    wd = torch.ones(H, dtype=torch.float16, device=DEV)
    L.lomo_vector_update(dev(xh), dev(dY), wd, 0.1, 1.0, 1.0, ws, flag)
    assert (host(wd) == 1.0).all()


# ------------------------------------------------------------------------------- clip by value


@pytest.mark.parametrize("T,K,N", [(512, 1024, 1024), (100, 264, 136), (70, 3600, 3320), (128, 4096, 4096)])
def test_linear_clip_by_value(L, T, K, N):
    Sc, sig_dy = 1024.0, 0.01
    X = gen(31, (T, K), 1.0)
    dY = S.normal_f16_np(S.tensor_key(32, T, K, N), (T, N), S.normal_mult(sig_dy, Sc))
    W = S.normal_f16_np(S.tensor_key(33, T, K, N), (N, K), S.normal_mult(0.02))
    G = O.linear_grad(X, dY)
    gstd = math.sqrt(T) * sig_dy
    clipv = float(np.float32(0.7 * gstd))                     # about half of the elements are clamped
    lr = float(np.float32(30 * 2.0 ** -16 / gstd))
    Wd = dev(W)
    dX = torch.empty(T, K, dtype=torch.float16, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    L.lomo_linear_backward_update_clip_value(dev(X), dev(dY), Wd, dX, lr, 1.0 / Sc, clipv, flag)
    got = host(Wd)
    want = O.sgd_update_clip_value(W, G, lr, clipv, Sc)
    assert_weights_close(got, want, "clip by value")
    clamped = np.abs(G / Sc) > clipv
    assert 0.3 < clamped.mean() < 0.7
    assert (O.ulp_distance_f16(want, O.sgd_update(W, G, lr, 1.0, Sc)) > 2).mean() > 0.2   # clamping matters
    assert int(flag.item()) == 0
    assert_dx_close(host(dX), dY, W, "dX")


def test_clip_by_value_overflow_elements_keep_their_weight(L):
    T, K, N = 130, 264, 520
    X, dY, W = gen(34, (T, K), 1.0), gen(35, (T, N), 1.0), gen(36, (N, K), 0.02)
    dY[7, 33] = np.inf                                         # poisons row 33 of the gradient
    G = O.linear_grad(X, dY)
    Wd = dev(W)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    L.lomo_linear_backward_update_clip_value(dev(X), dev(dY), Wd, None, 0.01, 1.0, 5.0, flag)
    got = host(Wd)
    assert int(flag.item()) == 1
    np.testing.assert_array_equal(got[33].view(np.uint16), W[33].view(np.uint16))
    assert_weights_close(got, O.sgd_update_clip_value(W, G, float(np.float32(0.01)), 5.0, 1.0), "clip by value + inf")


def test_step_clip_by_value_all_kinds(L):
    T, V, H, N = 256, 500, 264, 512
    Sc = 64.0
    cpu = [
        dict(kind="linear", X=gen(40, (T, H), 1.0), dY=S.normal_f16_np(41, (T, N), S.normal_mult(0.01, Sc)), W=gen(42, (N, H), 0.02)),
        dict(kind="linear", X=gen(43, (T, 4096), 1.0), dY=S.normal_f16_np(44, (T, 4096), S.normal_mult(0.01, Sc)),
             W=gen(45, (4096, 4096), 0.02)),                                  # persistent-kernel path
        dict(kind="vector", X=gen(46, (T, H), 1.0), dY=S.normal_f16_np(47, (T, H), S.normal_mult(0.01, Sc)), W=np.ones(H, np.float16)),
        dict(kind="embedding", ids=S.zipf_ids(3, T, V), dY=S.normal_f16_np(48, (T, H), S.normal_mult(0.01, Sc)), W=gen(49, (V, H), 0.02)),
    ]
    cpu[2]["dY"][5, 9] = np.nan
    gpu = [{k: (dev(v) if isinstance(v, np.ndarray) else v) for k, v in t.items()} for t in cpu]
    lst = L.make_tensor_list(gpu)
    ws = torch.empty(max(L.lomo_step_workspace_bytes(lst), 256), dtype=torch.uint8, device=DEV)
    flags = torch.zeros(len(gpu) + 1, dtype=torch.int32, device=DEV)
    lr, clipv = 0.02, 0.05
    L.lomo_step_update_pass_clip_value(lst, lr, 1.0 / Sc, clipv, flags, ws)
    assert flags.cpu().tolist() == [0, 0, 1, 0, 1]
    for g_, t in zip(gpu, cpu):
        want = O.sgd_update_clip_value(t["W"], O.tensor_grad(t), float(np.float32(lr)), float(np.float32(clipv)), Sc)
        assert_weights_close(host(g_["W"]), want, t["kind"])
    assert host(gpu[2]["W"])[9] == 1.0
    # the same pass through the stepper (its own flags and workspace), from the same start
    from paper_2306_09782_amd.step import LomoStep
    gpu2 = [{k: (dev(v) if isinstance(v, np.ndarray) else v) for k, v in t.items()} for t in cpu]
    stepper = LomoStep(DEV, max_T=T, max_H=H, max_tensors=len(gpu2))
    stepper.clip_value_pass(gpu2, lr, 1.0 / Sc, clipv)
    assert stepper.flags[:len(gpu2) + 1].cpu().tolist() == [0, 0, 1, 0, 1]
    for a, b in zip(gpu, gpu2):
        np.testing.assert_array_equal(host(a["W"]).view(np.uint16), host(b["W"]).view(np.uint16))


def test_reduce_flags(L):
    f = torch.zeros(700, dtype=torch.int32, device=DEV)
    out = torch.full((1,), 7, dtype=torch.int32, device=DEV)
    L.lomo_reduce_flags(f, out)
    assert int(out.item()) == 0
    f[613] = 1
    L.lomo_reduce_flags(f, out)
    assert int(out.item()) == 1


def test_generators_agree_on_device():
    key = S.tensor_key(0, 5, 1, 2)
    for mult in (S.normal_mult(0.02), S.normal_mult(1e-3, 65536.0)):
        a = S.normal_f16_np(key, (300, 520), mult)
        b = S.normal_f16_torch(key, (300, 520), mult, DEV).cpu().numpy()
        np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16))
        c = S.normal_f16_torch(key, (300, 520), mult, DEV, force_torch_ops=True).cpu().numpy()
        np.testing.assert_array_equal(a.view(np.uint16), c.view(np.uint16))


def _mixed_step_tensors(seed=0):
    """70 gain vectors of one shape (more than one launch holds), 3 of another, 2 of a third with T = 1, an embedding
    and a small linear tensor, against the oracle's materialised step."""
    Sc = 256.0
    recs = []
    k = [0]

    def g(shape, sig, sc=1.0):
        k[0] += 1
        return S.normal_f16_np(S.tensor_key(seed, 31, k[0], 0), shape, S.normal_mult(sig, sc))
    for (T, H, n) in ((96, 264, 70), (200, 1032, 3), (1, 72, 2)):
        for _ in range(n):
            recs.append(dict(kind="vector", X=g((T, H), 1.0), dY=g((T, H), 0.02, Sc), W=g((H,), 1.0)))
    recs.insert(5, dict(kind="embedding", ids=S.zipf_ids(seed, 300, 400), dY=g((300, 264), 0.02, Sc), W=g((400, 264), 0.05)))
    recs.insert(40, dict(kind="linear", X=g((96, 264), 1.0), dY=g((96, 136), 0.02, Sc), W=g((136, 264), 0.05)))
    return recs, Sc


@pytest.mark.parametrize("workspace", ["recommended", "minimum"])
def test_step_with_many_gain_vectors_of_mixed_shapes(L, workspace):
    """Gain vectors are batched per shape as far as the workspace holds their partial sums: with the recommended size
    64 of the 70 share a launch, with the minimum every vector gets its own; the results are the per-tensor calls' bit
    for bit, and the oracle's to the usual bar."""
    from paper_2306_09782_amd.step import LomoStep
    cpu, Sc = _mixed_step_tensors()
    lr = 0.5
    ref = O.step_materialised(cpu, lr, Sc)
    assert not ref["overflow"]
    results = []
    for grouped in (True, False):
        gpu = [{k: (dev(v) if isinstance(v, np.ndarray) else v) for k, v in t.items()} for t in cpu]
        gpu[40]["dX"] = torch.empty(96, 264, dtype=torch.float16, device=DEV)
        stepper = LomoStep(DEV, max_T=300, max_H=1032, max_tensors=len(gpu), grouped=grouped)
        if grouped:
            arr = L.make_tensor_list(gpu)
            need, least = L.lomo_step_workspace_bytes(arr), L.lomo_step_workspace_min_bytes(arr)
            one = L.lomo_vector_workspace_bytes(96, 264)
            assert least < need and need >= 64 * one
            stepper._list(gpu)                       # binds the list and sizes the workspace
            if workspace == "minimum":
                stepper.ws = torch.empty(least, dtype=torch.uint8, device=DEV)
                with pytest.raises(L.LomoError, match="workspace"):
                    L.lomo_step_norm_pass(arr, stepper.acc, stepper.flags, stepper.ws[:least - 256])
        res = stepper.run(gpu, lr, Sc)
        torch.cuda.synchronize()
        assert res["flags"] == ref["flags"] and res["overflow"] is False
        assert abs(res["norm"] / ref["norm"] - 1) < 1e-5
        results.append([host(t["W"]) for t in gpu])
    moved = 0
    for a, b, t, w in zip(results[0], results[1], cpu, ref["W"]):
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), t["kind"]
        assert_weights_close(a, w, t["kind"])
        moved += int((a.view(np.uint16) != t["W"].view(np.uint16)).sum())
    assert moved > 1000


def test_update_pass_reuses_the_grouping_of_the_norm_pass(L):
    """reuse_grouping = the workspace still holds pass 1's token grouping: same bits as grouping again; a stale
    workspace must not be trusted without the promise; two embeddings in one list never reuse."""
    cpu, Sc = _mixed_step_tensors(seed=3)
    cpu = cpu[:12]                                   # 11 gain vectors + the embedding at position 5
    lr, coef = 0.5, 0.25
    outs = []
    for reuse in (False, True):
        gpu = [{k: (dev(v) if isinstance(v, np.ndarray) else v) for k, v in t.items()} for t in cpu]
        arr = L.make_tensor_list(gpu)
        ws = torch.empty(L.lomo_step_workspace_bytes(arr), dtype=torch.uint8, device=DEV)
        acc = torch.zeros(1, dtype=torch.float64, device=DEV)
        flags = torch.zeros(len(gpu) + 1, dtype=torch.int32, device=DEV)
        L.lomo_step_norm_pass(arr, acc, flags, ws)
        if not reuse:
            ws[:4096].fill_(0xAB)                    # the head of the workspace is the grouping: spoil it, then regroup
        L.lomo_step_update_pass(arr, lr, 1.0 / Sc, coef, flags[len(gpu):], ws, reuse_grouping=reuse)
        torch.cuda.synchronize()
        outs.append([host(t["W"]) for t in gpu])
    for a, b, t in zip(outs[0], outs[1], cpu):
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), t["kind"]
        G = O.tensor_grad(t)
        assert_weights_close(a, O.sgd_update(t["W"], G, lr, coef, Sc), t["kind"])
    # two embedding tensors share the one grouping slot: the flag is ignored and both are grouped again
    two = [cpu[5], dict(cpu[5], ids=S.zipf_ids(9, 300, 400))]
    gpu = [{k: (dev(v) if isinstance(v, np.ndarray) else v) for k, v in t.items()} for t in two]
    arr = L.make_tensor_list(gpu)
    ws = torch.empty(L.lomo_step_workspace_bytes(arr), dtype=torch.uint8, device=DEV)
    acc = torch.zeros(1, dtype=torch.float64, device=DEV)
    flags = torch.zeros(3, dtype=torch.int32, device=DEV)
    L.lomo_step_norm_pass(arr, acc, flags, ws)
    L.lomo_step_update_pass(arr, lr, 1.0 / Sc, coef, flags[2:], ws, reuse_grouping=True)
    torch.cuda.synchronize()
    for g_, t in zip(gpu, two):
        assert_weights_close(host(g_["W"]), O.sgd_update(t["W"], O.tensor_grad(t), lr, coef, Sc), "embedding pair")
