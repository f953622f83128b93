"""The seeded input generators: determinism, subset consistency, CPU/torch twin, distributions."""
import numpy as np
import pytest
import torch

import lomo_synth as S
from lomo_synth.generators import ROLE_X, _mix_py


def test_splitmix_vector_matches_scalar():
    key = S.tensor_key(0, 3, 1, ROLE_X)
    c = np.array([0, 1, 2, 1000, 2 ** 40], dtype=np.uint64)
    got = S.splitmix64_np(key, c)
    for ci, g in zip(c.tolist(), got.tolist()):
        assert g == _mix_py(key + (ci + 1) * 0x9E3779B97F4A7C15)


def test_subset_equals_slice_and_is_deterministic():
    key = S.tensor_key(0, 1, 2, ROLE_X)
    m = S.normal_mult(1.0)
    full = S.normal_f16_np(key, (37, 29), m)
    again = S.normal_f16_np(key, (37, 29), m)
    np.testing.assert_array_equal(full.view(np.uint16), again.view(np.uint16))
    rows, cols = np.array([0, 5, 36]), np.array([1, 28, 7])
    sub = S.normal_f16_np(key, (37, 29), m, rows=rows, cols=cols)
    np.testing.assert_array_equal(sub.view(np.uint16), full[np.ix_(rows, cols)].view(np.uint16))
    other = S.normal_f16_np(S.tensor_key(0, 1, 2, 1), (37, 29), m)
    assert (other.view(np.uint16) != full.view(np.uint16)).mean() > 0.9


def test_torch_twin_is_bit_identical_on_cpu():
    key = S.tensor_key(0, 0, 0, 2)
    for mult in (S.normal_mult(0.02), S.normal_mult(1e-3, 65536.0), S.normal_mult(1.0)):
        a = S.normal_f16_np(key, (123, 77), mult)
        b = S.normal_f16_torch(key, (123, 77), mult, "cpu").numpy()
        np.testing.assert_array_equal(a.view(np.uint16), b.view(np.uint16))


def test_normal_moments():
    a = S.normal_f16_np(S.tensor_key(0, 0, 0, 0), (512, 1024), S.normal_mult(1.0)).astype(np.float64)
    assert abs(a.mean()) < 5e-3 and abs(a.std() - 1.0) < 5e-3
    assert np.abs(a).max() <= 6.0
    w = S.normal_f16_np(S.tensor_key(0, 0, 0, 2), (512, 1024), S.normal_mult(0.02)).astype(np.float64)
    assert abs(w.std() - 0.02) < 2e-4


def test_zipf_ids_shape_of_distribution():
    ids = S.zipf_ids(0, 4096, 32000)
    assert ids.dtype == np.int32 and ids.min() >= 0 and ids.max() < 32000
    vals, counts = np.unique(ids, return_counts=True)
    assert 1100 < vals.size < 1650            # about 1365 distinct ids expected at T = 4096
    assert 0.11 < counts.max() / 4096 < 0.18  # hottest id carries about 14 % of the tokens
    assert (counts == 1).sum() / vals.size > 0.6
    np.testing.assert_array_equal(ids, S.zipf_ids(0, 4096, 32000))
    assert vals.std() > 5000                  # hot ids are spread over the vocabulary


@pytest.mark.parametrize("name,params,flops", [
    ("linear1024", 1_048_576, 2 * 512 * 1024 * 1024),
    ("llama7b_layer", 202_375_168, 2 * 4096 * 202_375_168),
    ("llama7b_stack", 6_738_411_520, None),
    ("llama13b_stack", 13_015_859_200, None),
    ("llama65b_stack", 65_285_652_480, None),
])
def test_workload_tables(name, params, flops):
    w = S.workload(name)
    assert w.n_params == params
    if flops is not None:
        assert w.gemm_flops_per_pass == flops
    assert w.tensors[0].kind == "linear"
    if name.endswith("stack"):
        assert w.tensors[0].name == "lm_head" and w.tensors[-1].kind == "embedding"
        assert sum(t.kind == "vector" for t in w.tensors) == 2 * (len(w.tensors) - 2) // 9


def test_workload_generation_matches_spec_shapes():
    w = S.workload("linear1024")
    t = w.tensors[0]
    X, dY, W = w.X_np(t), w.dY_np(t), w.W_np(t)
    assert X.shape == (512, 1024) and dY.shape == (512, 1024) and W.shape == (1024, 1024)
    assert abs(dY.astype(np.float64).std() - 0.01 * 1024) < 0.1
    assert abs(W.astype(np.float64).std() - 0.02) < 2e-4
    cols = np.array([3, 900])
    np.testing.assert_array_equal(w.dY_np(t, cols=cols), dY[:, cols])
