"""The C-ABI library loads, exports what include/lomo.h declares, and its host functions agree
with the oracle.  No GPU work here."""
import os
import re

import pytest

import paper_2306_09782_amd as L
from paper_2306_09782_amd import binding
from oracle import lomo_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(L.library_path()):
        from paper_2306_09782_amd.build import build
        build(verbose=False)
    return L.load_library()


def _declared():
    text = open(os.path.join(ROOT, "include", "lomo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lomo_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    names = _declared()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
        assert hasattr(L, n), f"python binding lacks {n}"
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def test_status_strings(lib):
    assert L.lomo_status_str(0) == "ok"
    assert len({L.lomo_status_str(i) for i in range(6)}) == 6


def test_clip_coef_matches_oracle(lib):
    for sq, S in [(335.0, 1.0), (1e17, 65536.0), (0.25, 1.0), (0.0, 1024.0), (3.0e9, 1024.0)]:
        want = O.clip_coef(O.grad_norm(sq, S), 1.0, 1e-6)
        assert L.lomo_clip_coef(sq, S, 1.0, 1e-6) == pytest.approx(want, rel=1e-15)
    assert L.lomo_clip_coef(0.25, 1.0, 1.0, 1e-6) == 1.0
    assert L.lomo_clip_coef(float("inf"), 1.0) == 0.0 and L.lomo_clip_coef(float("nan"), 1.0) == 0.0


def test_scaler_matches_oracle(lib):
    S, c = 65536.0, 0
    So, co = 65536.0, 0
    for ov in [True, False, False, False, True, True, False, False, False, False]:
        S, c = L.lomo_scaler_step(S, c, 2, ov)
        So, co = O.scaler_step(So, co, 2, ov)
        assert (S, c) == (So, co)
    assert L.lomo_scaler_step(1.0, 3, 2, True) == O.scaler_step(1.0, 3, 2, True) == (1.0, 0)
    assert L.lomo_scaler_step(2.0 ** 24, 1, 2, False) == O.scaler_step(2.0 ** 24, 1, 2, False)


def test_shape_errors_are_reported_before_any_launch(lib):
    P = None
    assert lib.lomo_wgrad_sqnorm(P, P, 4, 12, 8, P, P, P) == 2        # K not a multiple of 8
    assert lib.lomo_wgrad_sqnorm(P, P, -1, 8, 8, P, P, P) == 2
    assert lib.lomo_wgrad_sqnorm(P, P, 4, 8, 8, P, P, P) == 1         # acc missing
    assert lib.lomo_linear_backward_update(P, P, P, P, 4, 8, 9, 0.1, 1.0, 1.0, P, P) == 2
    assert lib.lomo_linear_backward_update(P, P, P, P, 4, 8, 8, 0.1, 1.0, 1.0, P, P) == 1
    assert lib.lomo_embedding_update(P, P, P, 4, 12, 10, 0.1, 1.0, 1.0, P, P, 0, P) == 2
    assert lib.lomo_vector_update(P, P, P, 4, 8, 0.1, 1.0, 1.0, P, P, 0, P) == 1
    assert lib.lomo_vector_sqnorm(P, P, 0, 8, P, 0, P, P, P) == 1     # acc still required
    assert lib.lomo_step_norm_pass(None, 3, P, P, P, 0, None, P) == 1          # descriptor list missing
    assert lib.lomo_step_norm_pass(None, -1, P, P, P, 0, None, P) == 2
    bad = (binding.LomoTensor * 1)()
    bad[0].kind, bad[0].T, bad[0].K, bad[0].N = 0, 4, 12, 8
    assert lib.lomo_step_norm_pass(bad, 1, P, P, P, 0, None, P) == 2           # K not a multiple of 8
    bad[0].kind = 7
    assert lib.lomo_step_update_pass(bad, 1, 0.1, 1.0, 1.0, P, P, 0, None, P) == 2
    import ctypes
    opt = binding.LomoStepOptions(9, 0)
    assert lib.lomo_step_norm_pass(None, 0, P, P, P, 0, ctypes.byref(opt), P) == 2      # unknown norm route
    assert lib.lomo_wgrad_sqnorm_route(P, P, 4, 8, 8, P, P, 9, P) == 2
    assert lib.lomo_probe_mfma(P, 1, 3, 0, 0, P, 0, None, P) == 2 and lib.lomo_probe_copy(P, P, 24, P) == 2
    assert lib.lomo_cross_entropy_mean(P, P, 1.0, P, P, P, 4, 8, P) == 1                # stats missing
    vec = (binding.LomoTensor * 2)()
    for v in vec:
        v.kind, v.T, v.K, v.N = 2, 4096, 4096, 1
    one = lib.lomo_vector_workspace_bytes(4096, 4096)
    assert lib.lomo_step_workspace_min_bytes(vec, 2) == one and lib.lomo_step_workspace_bytes(vec, 2) == 2 * one
    assert lib.lomo_step_workspace_bytes(bad, 0) == 0
    assert lib.lomo_embedding_workspace_bytes(0, 4096) == 0
    assert lib.lomo_embedding_workspace_bytes(4096, 4096) >= 4096 * 8 + 3 * 4096 * 4
    # above 8192 positions the grouping merges sorted chunks between two key buffers
    assert lib.lomo_embedding_workspace_bytes(20000, 64) >= 2 * 32768 * 8 + 3 * 20000 * 4
    emb = (binding.LomoTensor * 1)()
    emb[0].kind, emb[0].T, emb[0].K, emb[0].N = 1, 20000, 64, 32000
    assert lib.lomo_step_workspace_bytes(emb, 1) == lib.lomo_embedding_workspace_bytes(20000, 64)
    assert lib.lomo_vector_workspace_bytes(4096, 4096) >= 4096 * 4


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(L.LomoError):
        binding.load_library()


def test_product_path_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2306_09782_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
