"""The allocation-free entry point lomo_vector_update_static against lomo_vector_update (same kernels, the
library's fixed scratch array in place of the caller's workspace): bit-identical results on two calls in a row,
the second on a smaller input, and a clear error beyond the array's size."""
import os

import numpy as np
import pytest
import torch

import lomo_synth as S

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


def inputs(seed, T, H):
    g = lambda i, sig: S.normal_f16_torch(S.tensor_key(seed, 21, i, 0), (T, H), S.normal_mult(sig), DEV)
    return g(0, 1.0), g(1, 0.5), S.normal_f16_torch(S.tensor_key(seed, 21, 2, 0), (H,), S.normal_mult(1.0), DEV)


def test_static_vector_update_matches_workspace_call(L):
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    # the larger call first (it leaves its partial sums in the array), then a smaller one, then a ragged one
    for seed, (T, H) in enumerate([(4096, 4096), (200, 264), (8192, 8192), (1, 8)]):
        xhat, dy, w0 = inputs(seed, T, H)
        lr, inv_s, clip = 0.25, 1.0 / 64.0, 0.5
        want = w0.clone()
        ws = torch.empty(L.lomo_vector_workspace_bytes(T, H), dtype=torch.uint8, device=DEV)
        L.lomo_vector_update(xhat, dy, want, lr, inv_s, clip, ws, flag)
        got = w0.clone()
        before = torch.cuda.memory_allocated()
        L.lomo_vector_update_static(xhat, dy, got, lr, inv_s, clip, flag)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (T, H)
        assert not torch.equal(got.view(torch.int16), w0.view(torch.int16)), (T, H)


def test_static_vector_update_honours_the_flag_and_its_limit(L):
    xhat, dy, w0 = inputs(9, 512, 1024)
    w = w0.clone()
    raised = torch.ones(1, dtype=torch.int32, device=DEV)
    L.lomo_vector_update_static(xhat, dy, w, 0.25, 1.0, 1.0, raised)
    torch.cuda.synchronize()
    assert torch.equal(w.view(torch.int16), w0.view(torch.int16))          # dropped step: nothing written
    # beyond the array: 128 row splits x 16384 columns x 4 bytes = 8 MiB > 4 MiB
    T, H = 8192, 16384
    assert L.lomo_vector_workspace_bytes(T, H) > L.VECTOR_STATIC_BYTES
    big = torch.zeros(T, H, dtype=torch.float16, device=DEV)
    wbig = torch.ones(H, dtype=torch.float16, device=DEV)
    with pytest.raises(L.LomoError, match="fixed scratch"):
        L.lomo_vector_update_static(big, big, wbig, 0.25, 1.0, 1.0, None)
    assert bool((wbig == 1).all())
    lib = L.load_library()
    assert lib.lomo_vector_update_static(None, None, None, 4, 12, 0.1, 1.0, 1.0, None, None) == 2     # H % 8
    assert lib.lomo_vector_update_static(None, None, None, 4, 8, 0.1, 1.0, 1.0, None, None) == 1      # null pointers
