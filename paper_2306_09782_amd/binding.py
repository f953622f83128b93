"""ctypes binding: one Python function per C entry point of include/lomo.h, same names.

Tensors are torch CUDA(HIP) tensors used purely as device memory; shapes supply T, K, N, H, V.
``stream`` is a torch.cuda.Stream (or None for the current stream).
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_void_p, c_int64, c_int32, c_float, c_double, c_size_t, c_int, c_char_p, POINTER

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTED_SYMBOLS = (
    "lomo_version", "lomo_status_str", "lomo_wgrad_sqnorm", "lomo_embedding_sqnorm", "lomo_vector_sqnorm",
    "lomo_clip_coef", "lomo_scaler_step", "lomo_reduce_flags", "lomo_linear_backward_update",
    "lomo_embedding_update", "lomo_vector_update", "lomo_embedding_workspace_bytes",
    "lomo_vector_workspace_bytes", "lomo_embedding_grouping", "lomo_timing_enable", "lomo_timing_read",
    "lomo_step_workspace_bytes", "lomo_step_norm_pass", "lomo_step_update_pass",
    "lomo_linear_backward_update_clip_value", "lomo_step_update_pass_clip_value",
    "lomo_wgrad_sqnorm_route", "lomo_step_workspace_min_bytes", "lomo_step_scalars_device", "lomo_step_update_pass_device",
    "lomo_linear_dgrad", "lomo_swiglu_backward", "lomo_rmsnorm_backward", "lomo_attention_backward",
    "lomo_linear_forward", "lomo_rmsnorm_forward", "lomo_swiglu_forward", "lomo_rope_forward", "lomo_attention_forward",
    "lomo_cross_entropy", "lomo_embedding_forward", "lomo_linear_forward_residual", "lomo_cross_entropy_mean",
    "lomo_probe_mfma", "lomo_probe_copy", "lomo_vector_update_static",
)


class LomoTensor(ctypes.Structure):
    """Mirror of the C struct lomo_tensor."""
    _fields_ = [("kind", c_int32), ("X", c_void_p), ("dY", c_void_p), ("W", c_void_p), ("dX", c_void_p),
                ("ids", c_void_p), ("T", c_int64), ("K", c_int64), ("N", c_int64)]


class LomoStepOptions(ctypes.Structure):
    """Mirror of the C struct lomo_step_options."""
    _fields_ = [("norm_algorithm", c_int32), ("reuse_grouping", c_int32)]


KIND_CODES = {"linear": 0, "embedding": 1, "vector": 2}


class LomoError(RuntimeError):
    pass


def library_path() -> str:
    """In-tree library; LOMO_LIBRARY names another build of the same sources (development aid)."""
    return os.environ.get("LOMO_LIBRARY") or os.path.join(_HERE, "lib", "liblomo.so")


def load_library():
    """Load liblomo.so (built in-tree by ``python -m paper_2306_09782_amd.build``). No fallback."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise LomoError(f"{path} is missing: build it with `python paper_2306_09782_amd/build.py` "
                        "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    P, I64 = c_void_p, c_int64
    sig = {
        "lomo_version": (c_int, []),
        "lomo_status_str": (c_char_p, [c_int]),
        "lomo_wgrad_sqnorm": (c_int, [P, P, I64, I64, I64, P, P, P]),
        "lomo_wgrad_sqnorm_route": (c_int, [P, P, I64, I64, I64, P, P, c_int, P]),
        "lomo_embedding_sqnorm": (c_int, [P, P, I64, I64, I64, P, c_size_t, P, P, P]),
        "lomo_vector_sqnorm": (c_int, [P, P, I64, I64, P, c_size_t, P, P, P]),
        "lomo_clip_coef": (c_double, [c_double, c_double, c_double, c_double]),
        "lomo_scaler_step": (None, [POINTER(c_float), POINTER(c_int32), c_int32, c_int]),
        "lomo_reduce_flags": (c_int, [P, I64, P, P]),
        "lomo_linear_backward_update": (c_int, [P, P, P, P, I64, I64, I64, c_float, c_float, c_float, P, P]),
        "lomo_embedding_update": (c_int, [P, P, P, I64, I64, I64, c_float, c_float, c_float, P, P, c_size_t, P]),
        "lomo_vector_update": (c_int, [P, P, P, I64, I64, c_float, c_float, c_float, P, P, c_size_t, P]),
        "lomo_vector_update_static": (c_int, [P, P, P, I64, I64, c_float, c_float, c_float, P, P]),
        "lomo_embedding_workspace_bytes": (c_size_t, [I64, I64]),
        "lomo_vector_workspace_bytes": (c_size_t, [I64, I64]),
        "lomo_embedding_grouping": (c_int, [P, I64, I64, P, c_size_t, P, P, P, P, P]),
        "lomo_step_workspace_bytes": (c_size_t, [POINTER(LomoTensor), I64]),
        "lomo_step_workspace_min_bytes": (c_size_t, [POINTER(LomoTensor), I64]),
        "lomo_step_norm_pass": (c_int, [POINTER(LomoTensor), I64, P, P, P, c_size_t, POINTER(LomoStepOptions), P]),
        "lomo_step_update_pass": (c_int, [POINTER(LomoTensor), I64, c_float, c_float, c_float, P, P, c_size_t,
                                          POINTER(LomoStepOptions), P]),
        "lomo_linear_backward_update_clip_value": (c_int, [P, P, P, P, I64, I64, I64, c_float, c_float, c_float, P, P]),
        "lomo_step_update_pass_clip_value": (c_int, [POINTER(LomoTensor), I64, c_float, c_float, c_float, P, P,
                                                     c_size_t, P]),
        "lomo_step_scalars_device": (c_int, [P, P, c_double, c_double, c_double, c_double, P, P]),
        "lomo_step_update_pass_device": (c_int, [POINTER(LomoTensor), I64, P, P, P, c_size_t, POINTER(LomoStepOptions), P]),
        "lomo_linear_dgrad": (c_int, [P, P, P, I64, I64, I64, P]),
        "lomo_swiglu_backward": (c_int, [P, P, P, I64, I64, P]),
        "lomo_rmsnorm_backward": (c_int, [P, P, P, P, P, P, I64, I64, P]),
        "lomo_attention_backward": (c_int, [P, P, P, P, P, P, P, P, I64, I64, I64, I64, P]),
        "lomo_linear_forward": (c_int, [P, P, P, I64, I64, I64, c_int, P]),
        "lomo_rmsnorm_forward": (c_int, [P, P, c_float, P, P, P, I64, I64, P]),
        "lomo_swiglu_forward": (c_int, [P, P, I64, I64, P]),
        "lomo_rope_forward": (c_int, [P, P, P, I64, I64, I64, I64, P]),
        "lomo_attention_forward": (c_int, [P, P, P, I64, I64, I64, I64, P]),
        "lomo_cross_entropy": (c_int, [P, P, c_float, P, P, I64, I64, P]),
        "lomo_embedding_forward": (c_int, [P, P, P, I64, I64, I64, P]),
        "lomo_linear_forward_residual": (c_int, [P, P, P, P, I64, I64, I64, P]),
        "lomo_cross_entropy_mean": (c_int, [P, P, c_double, P, P, P, I64, I64, P]),
        "lomo_probe_mfma": (c_int, [P, I64, c_int, c_int, c_int, P, I64, POINTER(c_double), P]),
        "lomo_probe_copy": (c_int, [P, P, c_size_t, P]),
        "lomo_timing_enable": (c_int, [c_int]),
        "lomo_timing_read": (c_int, [c_int, POINTER(c_double), POINTER(c_int64)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _LIB = lib
    return lib


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return c_void_p(stream.cuda_stream)


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _check(code):
    if code != 0:
        raise LomoError(f"lomo status {code}: {load_library().lomo_status_str(code).decode()}")


def lomo_version() -> int:
    return load_library().lomo_version()


def lomo_status_str(code: int) -> str:
    return load_library().lomo_status_str(code).decode()


def on_stream(stream):
    """Context in which torch's own operations (fills, copies) are queued on `stream` (None: the current one)."""
    import contextlib
    import torch
    return contextlib.nullcontext() if stream is None else torch.cuda.stream(stream)


def _route(norm_algorithm) -> int:
    return NORM_ALGORITHMS[norm_algorithm] if isinstance(norm_algorithm, str) else int(norm_algorithm)


def _options(norm_algorithm="direct", reuse_grouping=False):
    return ctypes.byref(LomoStepOptions(_route(norm_algorithm), 1 if reuse_grouping else 0))


def lomo_wgrad_sqnorm(X, dY, acc, overflow_flag=None, stream=None):
    T, K = X.shape
    N = dY.shape[1]
    assert dY.shape[0] == T
    _check(load_library().lomo_wgrad_sqnorm(_ptr(X), _ptr(dY), T, K, N, _ptr(acc), _ptr(overflow_flag), _stream(stream)))


def lomo_wgrad_sqnorm_route(X, dY, acc, overflow_flag=None, norm_algorithm="direct", stream=None):
    """lomo_wgrad_sqnorm on the route named ('direct', 'auto', 'gram' or the integer code)."""
    T, K = X.shape
    N = dY.shape[1]
    assert dY.shape[0] == T
    _check(load_library().lomo_wgrad_sqnorm_route(_ptr(X), _ptr(dY), T, K, N, _ptr(acc), _ptr(overflow_flag),
                                                  _route(norm_algorithm), _stream(stream)))


def lomo_embedding_sqnorm(ids, dY, V, ws, acc, overflow_flag=None, stream=None):
    T, H = dY.shape
    _check(load_library().lomo_embedding_sqnorm(_ptr(ids), _ptr(dY), T, H, V, _ptr(ws), _nbytes(ws), _ptr(acc),
                                                _ptr(overflow_flag), _stream(stream)))


def lomo_vector_sqnorm(Xhat, dY, ws, acc, overflow_flag=None, stream=None):
    T, H = dY.shape
    _check(load_library().lomo_vector_sqnorm(_ptr(Xhat), _ptr(dY), T, H, _ptr(ws), _nbytes(ws), _ptr(acc),
                                             _ptr(overflow_flag), _stream(stream)))


def lomo_clip_coef(acc_sqnorm_scaled: float, loss_scale: float, max_norm: float = 1.0, eps: float = 1e-6) -> float:
    return load_library().lomo_clip_coef(acc_sqnorm_scaled, loss_scale, max_norm, eps)


def lomo_scaler_step(loss_scale: float, clean_steps: int, growth_interval: int, overflow: bool):
    s, c = c_float(loss_scale), c_int32(clean_steps)
    load_library().lomo_scaler_step(ctypes.byref(s), ctypes.byref(c), growth_interval, int(bool(overflow)))
    return s.value, c.value


def lomo_reduce_flags(flags, out, stream=None):
    _check(load_library().lomo_reduce_flags(_ptr(flags), flags.numel(), _ptr(out), _stream(stream)))


def lomo_linear_backward_update(X, dY, W, dX, lr, inv_loss_scale, clip_coef, overflow_flag=None, stream=None):
    T, K = X.shape
    N = dY.shape[1]
    assert dY.shape[0] == T and tuple(W.shape) == (N, K) and (dX is None or tuple(dX.shape) == (T, K))
    _check(load_library().lomo_linear_backward_update(_ptr(X), _ptr(dY), _ptr(W), _ptr(dX), T, K, N, lr, inv_loss_scale,
                                                      clip_coef, _ptr(overflow_flag), _stream(stream)))


def lomo_embedding_update(ids, dY, W, lr, inv_loss_scale, clip_coef, ws, overflow_flag=None, stream=None):
    T, H = dY.shape
    V = W.shape[0]
    assert W.shape[1] == H
    _check(load_library().lomo_embedding_update(_ptr(ids), _ptr(dY), _ptr(W), T, H, V, lr, inv_loss_scale, clip_coef,
                                                _ptr(overflow_flag), _ptr(ws), _nbytes(ws), _stream(stream)))


def lomo_vector_update(Xhat, dY, w, lr, inv_loss_scale, clip_coef, ws, overflow_flag=None, stream=None):
    T, H = dY.shape
    assert w.numel() == H
    _check(load_library().lomo_vector_update(_ptr(Xhat), _ptr(dY), _ptr(w), T, H, lr, inv_loss_scale, clip_coef,
                                             _ptr(overflow_flag), _ptr(ws), _nbytes(ws), _stream(stream)))


VECTOR_STATIC_BYTES = 4 << 20


def lomo_vector_update_static(Xhat, dY, w, lr, inv_loss_scale, clip_coef, overflow_flag=None, stream=None):
    """lomo_vector_update without a workspace argument: the library's fixed scratch array takes its place."""
    T, H = dY.shape
    assert w.numel() == H
    _check(load_library().lomo_vector_update_static(_ptr(Xhat), _ptr(dY), _ptr(w), T, H, lr, inv_loss_scale, clip_coef,
                                                    _ptr(overflow_flag), _stream(stream)))


def lomo_embedding_workspace_bytes(T: int, H: int) -> int:
    return load_library().lomo_embedding_workspace_bytes(T, H)


def lomo_vector_workspace_bytes(T: int, H: int) -> int:
    return load_library().lomo_vector_workspace_bytes(T, H)


def lomo_embedding_grouping(ids, V, ws, unique_ids, seg_offsets, perm, n_unique, stream=None):
    T = ids.numel()
    _check(load_library().lomo_embedding_grouping(_ptr(ids), T, V, _ptr(ws), _nbytes(ws), _ptr(unique_ids),
                                                  _ptr(seg_offsets), _ptr(perm), _ptr(n_unique), _stream(stream)))


KERNEL_FAMILIES = ("wgrad_update", "wgrad_sqnorm", "dgrad", "embedding", "vector", "gram_sqnorm", "chain", "attention",
                   "forward", "probe")
NORM_ALGORITHMS = {"direct": 0, "auto": 1, "gram": 2}


def lomo_timing_enable(on: bool):
    _check(load_library().lomo_timing_enable(int(bool(on))))


def lomo_timing_read(family: int):
    """(total kernel milliseconds, timed launches) of one kernel family since timing was enabled."""
    ms, n = c_double(0.0), c_int64(0)
    _check(load_library().lomo_timing_read(family, ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value


def make_tensor_list(tensors):
    """ctypes array of lomo_tensor from records {kind, X / ids, dY, W, dX?} holding torch tensors."""
    arr = (LomoTensor * len(tensors))()
    for rec, t in zip(arr, tensors):
        kind = t["kind"]
        rec.kind = KIND_CODES[kind]
        dY, W = t["dY"], t["W"]
        rec.dY, rec.W = dY.data_ptr(), W.data_ptr()
        rec.T = dY.shape[0]
        if kind == "linear":
            X = t["X"]
            rec.X, rec.K, rec.N = X.data_ptr(), X.shape[1], dY.shape[1]
            dX = t.get("dX")
            rec.dX = dX.data_ptr() if dX is not None else None
            assert tuple(W.shape) == (rec.N, rec.K) and X.shape[0] == rec.T
        elif kind == "embedding":
            rec.ids, rec.K, rec.N = t["ids"].data_ptr(), dY.shape[1], W.shape[0]
            assert W.shape[1] == rec.K and t["ids"].numel() == rec.T
        else:
            rec.X, rec.K, rec.N = t["X"].data_ptr(), dY.shape[1], 1
            assert W.numel() == rec.K
    return arr


def lomo_step_workspace_bytes(tensor_list) -> int:
    return load_library().lomo_step_workspace_bytes(tensor_list, len(tensor_list))


def lomo_step_workspace_min_bytes(tensor_list) -> int:
    return load_library().lomo_step_workspace_min_bytes(tensor_list, len(tensor_list))


def lomo_step_norm_pass(tensor_list, acc, flags, ws, stream=None, norm_algorithm="direct"):
    assert flags.numel() >= len(tensor_list) + 1
    _check(load_library().lomo_step_norm_pass(tensor_list, len(tensor_list), _ptr(acc), _ptr(flags), _ptr(ws),
                                              _nbytes(ws), _options(norm_algorithm), _stream(stream)))


def lomo_step_update_pass(tensor_list, lr, inv_loss_scale, clip_coef, step_flag, ws, stream=None, reuse_grouping=False):
    """reuse_grouping: `ws` still holds what lomo_step_norm_pass left there for the same list."""
    _check(load_library().lomo_step_update_pass(tensor_list, len(tensor_list), lr, inv_loss_scale, clip_coef,
                                                _ptr(step_flag), _ptr(ws), _nbytes(ws),
                                                _options(reuse_grouping=reuse_grouping), _stream(stream)))


def lomo_linear_dgrad(dY, W, dX, stream=None):
    T, N = dY.shape
    K = W.shape[1]
    assert W.shape[0] == N and tuple(dX.shape) == (T, K)
    _check(load_library().lomo_linear_dgrad(_ptr(dY), _ptr(W), _ptr(dX), T, K, N, _stream(stream)))


def lomo_linear_forward(X, W, Y, accumulate=False, stream=None):
    T, K = X.shape
    N = W.shape[0]
    assert W.shape[1] == K and tuple(Y.shape) == (T, N)
    _check(load_library().lomo_linear_forward(_ptr(X), _ptr(W), _ptr(Y), T, K, N, 1 if accumulate else 0, _stream(stream)))


def lomo_linear_forward_residual(X, W, R, Y, stream=None):
    T, K = X.shape
    N = W.shape[0]
    assert W.shape[1] == K and tuple(Y.shape) == (T, N) and tuple(R.shape) == (T, N)
    _check(load_library().lomo_linear_forward_residual(_ptr(X), _ptr(W), _ptr(R), _ptr(Y), T, K, N, _stream(stream)))


def lomo_embedding_forward(ids, W, h, stream=None):
    T, H = h.shape
    assert ids.numel() == T and W.shape[1] == H
    _check(load_library().lomo_embedding_forward(_ptr(ids), _ptr(W), _ptr(h), T, H, W.shape[0], _stream(stream)))


def lomo_rmsnorm_forward(h, gain, eps, xhat, rstd, xn, stream=None):
    T, H = h.shape
    assert gain.numel() == H and tuple(xhat.shape) == (T, H) and tuple(xn.shape) == (T, H) and rstd.numel() == T
    _check(load_library().lomo_rmsnorm_forward(_ptr(h), _ptr(gain), eps, _ptr(xhat), _ptr(rstd), _ptr(xn), T, H,
                                               _stream(stream)))


def lomo_swiglu_forward(gate_up, a, stream=None):
    T, F = a.shape
    assert tuple(gate_up.shape) == (T, 2 * F)
    _check(load_library().lomo_swiglu_forward(_ptr(gate_up), _ptr(a), T, F, _stream(stream)))


def lomo_rope_forward(qkv, rope_cos, rope_sin, s, n_heads, stream=None):
    T, H3 = qkv.shape
    assert H3 == 3 * n_heads * 128 and T % s == 0 and tuple(rope_cos.shape) == (s, 64) and tuple(rope_sin.shape) == (s, 64)
    _check(load_library().lomo_rope_forward(_ptr(qkv), _ptr(rope_cos), _ptr(rope_sin), T, s, n_heads, 128, _stream(stream)))


def lomo_attention_forward(qkv, o, lse, B, s, n_heads, stream=None):
    T, H = o.shape
    assert T == B * s and H == n_heads * 128 and tuple(qkv.shape) == (T, 3 * H) and lse.numel() == T * n_heads
    _check(load_library().lomo_attention_forward(_ptr(qkv), _ptr(o), _ptr(lse), B, s, n_heads, 128, _stream(stream)))


def lomo_cross_entropy(logits, targets, grad_scale, loss, dlogits, stream=None):
    T, V = logits.shape
    assert targets.numel() == T and loss.numel() == T and tuple(dlogits.shape) == (T, V)
    _check(load_library().lomo_cross_entropy(_ptr(logits), _ptr(targets), grad_scale, _ptr(loss), _ptr(dlogits), T, V,
                                             _stream(stream)))


def lomo_cross_entropy_mean(logits, targets, loss_scale, loss, dlogits, stats, stream=None):
    """stats: device float64[3]; receives (mean loss over the counted targets, their number, scratch)."""
    T, V = logits.shape
    assert targets.numel() == T and loss.numel() == T and tuple(dlogits.shape) == (T, V) and _nbytes(stats) >= 24
    _check(load_library().lomo_cross_entropy_mean(_ptr(logits), _ptr(targets), loss_scale, _ptr(loss), _ptr(dlogits),
                                                  _ptr(stats), T, V, _stream(stream)))


PROBE_OPERAND_BYTES = 16 * 64 * 16


def lomo_probe_mfma(operands, iters, waves_per_simd, sink, idle_sleeps=0, lds_reads=False, stream=None) -> float:
    """Launches the matrix-core loop; returns the flop count of the launch."""
    assert _nbytes(operands) >= PROBE_OPERAND_BYTES
    flops = c_double(0.0)
    _check(load_library().lomo_probe_mfma(_ptr(operands), iters, waves_per_simd, idle_sleeps, 1 if lds_reads else 0,
                                          _ptr(sink), sink.numel(), ctypes.byref(flops), _stream(stream)))
    return flops.value


def lomo_probe_copy(src, dst, stream=None):
    assert _nbytes(src) == _nbytes(dst)
    _check(load_library().lomo_probe_copy(_ptr(src), _ptr(dst), _nbytes(src), _stream(stream)))


def lomo_swiglu_backward(da, gate_up, dgate_up, stream=None):
    T, F = da.shape
    assert tuple(gate_up.shape) == (T, 2 * F) and tuple(dgate_up.shape) == (T, 2 * F)
    _check(load_library().lomo_swiglu_backward(_ptr(da), _ptr(gate_up), _ptr(dgate_up), T, F, _stream(stream)))


def lomo_rmsnorm_backward(dxn, xhat, rstd, gain, dres, dh, stream=None):
    T, H = dxn.shape
    assert tuple(xhat.shape) == (T, H) and rstd.numel() == T and gain.numel() == H and tuple(dh.shape) == (T, H)
    assert dres is None or tuple(dres.shape) == (T, H)
    _check(load_library().lomo_rmsnorm_backward(_ptr(dxn), _ptr(xhat), _ptr(rstd), _ptr(gain), _ptr(dres), _ptr(dh),
                                                T, H, _stream(stream)))


def lomo_attention_backward(qkv, o, dO, lse, rope_cos, rope_sin, delta_ws, dqkv, B, s, n_heads, stream=None):
    T, H = o.shape
    assert T == B * s and H % n_heads == 0 and tuple(qkv.shape) == (T, 3 * H) and tuple(dqkv.shape) == (T, 3 * H)
    assert tuple(dO.shape) == (T, H) and lse.numel() == T * n_heads and delta_ws.numel() >= T * n_heads
    _check(load_library().lomo_attention_backward(_ptr(qkv), _ptr(o), _ptr(dO), _ptr(lse), _ptr(rope_cos), _ptr(rope_sin),
                                                  _ptr(delta_ws), _ptr(dqkv), B, s, n_heads, H // n_heads, _stream(stream)))


SCALARS_BYTES = 24   # sizeof(lomo_step_scalars): double clip_coef, double grad_norm, float step, int32 overflow


def lomo_step_scalars_device(acc, step_flag, loss_scale, max_norm, eps, lr, scalars, stream=None):
    """scalars: device uint8 tensor of at least SCALARS_BYTES bytes, 8-byte aligned."""
    assert _nbytes(scalars) >= SCALARS_BYTES
    _check(load_library().lomo_step_scalars_device(_ptr(acc), _ptr(step_flag), loss_scale, max_norm, eps, lr,
                                                   _ptr(scalars), _stream(stream)))


def lomo_step_update_pass_device(tensor_list, scalars, step_flag, ws, stream=None, reuse_grouping=False):
    _check(load_library().lomo_step_update_pass_device(tensor_list, len(tensor_list), _ptr(scalars), _ptr(step_flag),
                                                       _ptr(ws), _nbytes(ws), _options(reuse_grouping=reuse_grouping),
                                                       _stream(stream)))


def unpack_step_scalars(host_bytes):
    """{clip_coef, norm, step, overflow} from the SCALARS_BYTES bytes of a lomo_step_scalars (host uint8 tensor)."""
    import struct
    clip, norm, step, ovf = struct.unpack("<ddfi", bytes(host_bytes[:SCALARS_BYTES].tolist()))
    return {"clip_coef": clip, "norm": norm, "step": step, "overflow": bool(ovf)}


def lomo_linear_backward_update_clip_value(X, dY, W, dX, lr, inv_loss_scale, clip_value, overflow_flag=None,
                                           stream=None):
    T, K = X.shape
    N = dY.shape[1]
    assert dY.shape[0] == T and tuple(W.shape) == (N, K) and (dX is None or tuple(dX.shape) == (T, K))
    _check(load_library().lomo_linear_backward_update_clip_value(_ptr(X), _ptr(dY), _ptr(W), _ptr(dX), T, K, N, lr,
                                                                 inv_loss_scale, clip_value, _ptr(overflow_flag),
                                                                 _stream(stream)))


def lomo_step_update_pass_clip_value(tensor_list, lr, inv_loss_scale, clip_value, flags, ws, stream=None):
    assert flags.numel() >= len(tensor_list) + 1
    _check(load_library().lomo_step_update_pass_clip_value(tensor_list, len(tensor_list), lr, inv_loss_scale,
                                                           clip_value, _ptr(flags), _ptr(ws), _nbytes(ws),
                                                           _stream(stream)))
