"""Gram route of the norm pass on the GPU against the oracle's materialised gradient norm.

||dY^T X||^2 computed from X X^T and dY dY^T (lower triangle, weights 2 / 1) must equal the oracle's
sum of squares of the fp64 gradient within the norm tolerance (1e-3; observed ~1e-6), and must raise
the same overflow flag.  Inputs with strongly correlated rows make the off-diagonal token pairs carry
almost all of the sum, so a wrong triangle weight or a misplaced tile cannot hide inside the tolerance.
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


@pytest.fixture()
def gram(L):
    return L


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gen(seed, shape, sigma, role=0):
    return S.normal_f16_np(S.tensor_key(seed, 11, role, 5), shape, S.normal_mult(sigma))


def correlated(seed, T, C, sigma, role):
    """Rows = one common row + a tenth of independent noise: every token pair has a large dot product."""
    base = gen(seed, (1, C), sigma, role).astype(np.float32)
    noise = gen(seed + 1, (T, C), sigma * 0.1, role).astype(np.float32)
    return (base + noise).astype(np.float16)


def device_sqnorm(L, X, dY, route="gram"):
    acc = torch.zeros(1, dtype=torch.float64, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    L.lomo_wgrad_sqnorm_route(dev(X), dev(dY), acc, flag, route)
    torch.cuda.synchronize()
    return float(acc.item()), int(flag.item())


GRAM_SHAPES = [
    (256, 128, 128),       # one tile row: both tiles straddle the diagonal
    (512, 256, 384),
    (768, 128, 640),       # three tile rows: a partial band
    (1024, 1024, 512),     # exactly one band
    (1280, 384, 256),      # one band + a one-row band
    (2048, 1024, 4096),    # 72 tiles
    (4096, 256, 128),      # 272 tiles: more than one per CU
]


@pytest.mark.parametrize("kind", ["independent", "correlated"])
@pytest.mark.parametrize("T,K,N", GRAM_SHAPES)
def test_gram_norm_matches_oracle(gram, T, K, N, kind):
    L = gram
    if kind == "independent":
        X, dY = gen(1, (T, K), 1.0, 0), gen(2, (T, N), 0.5, 1)
    else:
        X, dY = correlated(3, T, K, 1.0, 0), correlated(5, T, N, 0.5, 1)
    want = O.sqnorm(O.linear_grad(X, dY))
    got, flag = device_sqnorm(L, X, dY)
    assert flag == 0
    assert abs(got / want - 1) < 1e-3, (got, want)
    assert abs(got / want - 1) < 2e-5, (got, want)       # what fp32 accumulation actually delivers
    # the direct route on the same bits
    direct, _ = device_sqnorm(L, X, dY, "direct")
    assert abs(direct / want - 1) < 2e-5
    if kind == "correlated":
        # the diagonal pairs alone are a small part of the sum here: the triangle weights matter
        diag = float(((X.astype(np.float64) ** 2).sum(1) * (dY.astype(np.float64) ** 2).sum(1)).sum())
        assert diag < 0.05 * want


def test_gram_is_used_and_falls_back(gram):
    L = gram
    L.lomo_timing_enable(True)
    fam = L.KERNEL_FAMILIES.index("gram_sqnorm")
    X, dY = gen(7, (512, 256), 1.0, 0), gen(8, (512, 384), 1.0, 1)
    device_sqnorm(L, X, dY)
    assert L.lomo_timing_read(fam)[1] == 1
    # T not a multiple of 256, K not a multiple of 128: the direct kernels take over, same answer
    for (T, K, N) in [(300, 256, 384), (512, 264, 384), (512, 256, 8)]:
        X, dY = gen(9, (T, K), 1.0, 0), gen(10, (T, N), 1.0, 1)
        got, flag = device_sqnorm(L, X, dY)
        assert flag == 0 and abs(got / O.sqnorm(O.linear_grad(X, dY)) - 1) < 2e-5
    assert L.lomo_timing_read(fam)[1] == 1
    L.lomo_timing_enable(False)


@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
@pytest.mark.parametrize("where,row,col", [("X", 0, 0), ("X", 700, 129), ("dY", 255, 383), ("dY", 767, 1)])
def test_gram_overflow_flag(gram, bad, where, row, col):
    L = gram
    X, dY = gen(11, (768, 256), 1.0, 0), gen(12, (768, 384), 1.0, 1)
    (X if where == "X" else dY)[row, col] = bad
    assert O.has_overflow(O.linear_grad(X, dY))
    _, flag = device_sqnorm(L, X, dY)
    assert flag == 1


def test_gram_zero_rows_and_zero_inputs(gram):
    L = gram
    X, dY = gen(13, (512, 128), 1.0, 0), gen(14, (512, 256), 1.0, 1)
    X[100:300] = 0
    got, flag = device_sqnorm(L, X, dY)
    assert flag == 0 and abs(got / O.sqnorm(O.linear_grad(X, dY)) - 1) < 2e-5
    got, flag = device_sqnorm(L, np.zeros_like(X), dY)
    assert flag == 0 and got == 0.0


@pytest.mark.parametrize("mode", ["gram", "auto"])
def test_norm_pass_routes(L, mode):
    """A whole norm pass with tensors on both routes: per-tensor flags, one total."""
    from paper_2306_09782_amd.step import LomoStep
    shapes = [(512, 256, 384), (512, 1024, 128), (300, 264, 136), (512, 4096, 4096), (512, 128, 128)]
    ts, want = [], 0.0
    for i, (T, K, N) in enumerate(shapes):
        X, dY = gen(20 + i, (T, K), 1.0, 0), gen(40 + i, (T, N), 0.25, 1)
        if i == 1:
            dY[511, 127] = np.inf
        W = gen(60 + i, (N, K), 0.02, 2)
        ts.append({"kind": "linear", "X": dev(X), "dY": dev(dY), "W": dev(W)})
        if i != 1:
            want += O.sqnorm(O.linear_grad(X, dY))
    stepper = LomoStep(DEV, max_T=512, max_H=4096, max_tensors=len(ts), norm_algorithm=mode)
    stepper.norm_pass(ts)
    res = stepper.read_back(len(ts))
    assert res["flags"] == [False, True, False, False, False] and res["overflow"] is True
    ts[1]["dY"][511, 127] = 0.0
    stepper.norm_pass(ts)
    res = stepper.read_back(len(ts))
    hX, hdY = ts[1]["X"].cpu().numpy(), ts[1]["dY"].cpu().numpy()
    total = want + O.sqnorm(O.linear_grad(hX, hdY))
    assert not any(res["flags"]) and res["overflow"] is False
    assert abs(res["total_sqnorm"] / total - 1) < 2e-5


def test_norm_route_is_an_argument(L):
    """The route is chosen per call: the plain call stays on the direct kernels whatever an earlier call used, and
    an unknown code is refused before anything is launched."""
    L.lomo_timing_enable(True)
    fam = L.KERNEL_FAMILIES.index("gram_sqnorm")
    X, dY = gen(7, (512, 256), 1.0, 0), gen(8, (512, 384), 1.0, 1)
    device_sqnorm(L, X, dY, "gram")
    assert L.lomo_timing_read(fam)[1] == 1
    acc = torch.zeros(1, dtype=torch.float64, device=DEV)
    L.lomo_wgrad_sqnorm(dev(X), dev(dY), acc)
    assert L.lomo_timing_read(fam)[1] == 1
    L.lomo_timing_enable(False)
    with pytest.raises(L.LomoError):
        L.lomo_wgrad_sqnorm_route(dev(X), dev(dY), acc, None, 7)
    with pytest.raises(L.LomoError):
        L.lomo_step_norm_pass(L.make_tensor_list([]), acc, torch.zeros(1, dtype=torch.int32, device=DEV), None, None, 7)


@pytest.mark.parametrize("K,N", [(8192, 8192), (8192, 22016), (22016, 8192)])
def test_gram_llama65b_tensor_shapes(gram, K, N):
    """The linear tensors of the 65B layer at its token count (T = 2048), where the Gram route pays most:
    same inputs as the workload (device generator), norm against the oracle's materialised gradient."""
    L = gram
    T = 2048
    X = S.normal_f16_torch(S.tensor_key(0, 3, 1, 0), (T, K), S.normal_mult(1.0), DEV)
    dY = S.normal_f16_torch(S.tensor_key(0, 3, 1, 1), (T, N), S.normal_mult(1e-3, 65536.0), DEV)
    acc = torch.zeros(2, dtype=torch.float64, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    L.lomo_timing_enable(True)
    L.lomo_wgrad_sqnorm_route(X, dY, acc[0:1], flag, "gram")
    used = L.lomo_timing_read(L.KERNEL_FAMILIES.index("gram_sqnorm"))[1]
    L.lomo_timing_enable(False)
    L.lomo_wgrad_sqnorm(X, dY, acc[1:2], flag)
    torch.cuda.synchronize()
    want = O.sqnorm(O.linear_grad(X.cpu().numpy(), dY.cpu().numpy()))
    g, d = acc.cpu().numpy()
    assert used == 1 and int(flag.item()) == 0
    assert abs(g / want - 1) < 1e-3 and abs(g / want - 1) < 2e-5
    assert abs(d / want - 1) < 2e-5
