"""Counter-based generators: the same bits from numpy (CPU) and from torch (device).

Normal values are an integer-exact Irwin-Hall approximation: twelve 16-bit uniform
fields taken from three SplitMix64 outputs are summed and centred (an integer with
|c| < 2^24, exactly representable in fp32), multiplied once in fp32 by
``sigma * scale / 65536`` and rounded once to fp16 (round-to-nearest-even).  No
transcendental function is involved, so CPU and GPU agree bit for bit.  The sum
has standard deviation sqrt(65536^2 - 1) and support +-6 sigma.

SplitMix64 (Steele, Lea, Flood 2014) is used as a stateless hash of a 64-bit
counter: word(c) = mix(key + (c + 1) * GOLDEN).
"""
from __future__ import annotations

import numpy as np

GOLDEN = 0x9E3779B97F4A7C15
MIX1 = 0xBF58476D1CE4E5B9
MIX2 = 0x94D049BB133111EB
MASK64 = (1 << 64) - 1

ROLE_X, ROLE_DY, ROLE_W, ROLE_IDS, ROLE_PERM = 0, 1, 2, 3, 4


def _mix_py(z: int) -> int:
    z &= MASK64
    z = ((z ^ (z >> 30)) * MIX1) & MASK64
    z = ((z ^ (z >> 27)) * MIX2) & MASK64
    return z ^ (z >> 31)


def tensor_key(seed: int, layer: int, tensor: int, role: int) -> int:
    """64-bit stream key for one (seed, layer, tensor, role) tuple."""
    k = _mix_py(seed + GOLDEN)
    for v in (layer + 1, tensor + 1, role + 1):
        k = _mix_py(k ^ ((v * GOLDEN) & MASK64))
    return k


def splitmix64_np(key: int, counters: np.ndarray) -> np.ndarray:
    """word(c) for an array of uint64 counters."""
    with np.errstate(over="ignore"):
        z = np.uint64(key) + (counters.astype(np.uint64) + np.uint64(1)) * np.uint64(GOLDEN)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(MIX1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(MIX2)
        return z ^ (z >> np.uint64(31))


def normal_mult(sigma: float, scale: float = 1.0) -> np.float32:
    """The single fp32 multiplier applied to the centred integer sum."""
    return np.float32(float(sigma) * float(scale) / 65536.0)


def _centred_sum_np(key: int, flat_idx: np.ndarray) -> np.ndarray:
    base = flat_idx.astype(np.uint64) * np.uint64(3)
    s = np.zeros(flat_idx.shape, dtype=np.int64)
    for j in range(3):
        w = splitmix64_np(key, base + np.uint64(j))
        for f in range(4):
            s += ((w >> np.uint64(16 * f)) & np.uint64(0xFFFF)).astype(np.int64)
    return s - 6 * 65535


def normal_f16_np(key: int, shape, mult, rows=None, cols=None) -> np.ndarray:
    """fp16 tensor of the given logical 2-D (or 1-D) shape, or a row/column subset of it.

    ``rows`` / ``cols`` are index arrays into the logical tensor; element (r, c) always
    has flat counter r * ncols + c, so a subset equals the same slice of the full tensor.
    """
    if len(shape) == 1:
        shape = (1, shape[0])
        squeeze = True
    else:
        squeeze = False
    nrows, ncols = int(shape[0]), int(shape[1])
    r = np.arange(nrows, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    c = np.arange(ncols, dtype=np.int64) if cols is None else np.asarray(cols, dtype=np.int64)
    out = np.empty((r.size, c.size), dtype=np.float16)
    m = np.float32(mult)
    step = max(1, (1 << 22) // max(1, c.size))          # bound temporaries to ~4M elements
    for r0 in range(0, r.size, step):
        rr = r[r0:r0 + step]
        flat = rr[:, None] * np.int64(ncols) + c[None, :]
        cs = _centred_sum_np(key, flat)
        out[r0:r0 + step] = (cs.astype(np.float32) * m).astype(np.float16)
    return out[0] if squeeze else out


def _i64(v: int) -> int:
    """Two's-complement view of a 64-bit constant as a Python int that fits int64."""
    v &= MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_GEN_LIB = None


def _gen_lib():
    """The HIP generator kernel (built in-tree next to this file), or None if it is not built."""
    global _GEN_LIB
    if _GEN_LIB is None:
        import ctypes
        import os
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libsynthgen.so")
        if not os.path.exists(path):
            _GEN_LIB = False
        else:
            lib = ctypes.CDLL(path)
            lib.synth_normal_f16.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64, ctypes.c_float,
                                             ctypes.c_void_p, ctypes.c_void_p]
            lib.synth_normal_f16.restype = ctypes.c_int
            _GEN_LIB = lib
    return _GEN_LIB or None


def normal_f16_torch(key: int, shape, mult, device, out=None, force_torch_ops: bool = False):
    """Device twin of :func:`normal_f16_np` (full tensor only). Integer ops wrap mod 2^64.

    On a GPU the fill is one HIP kernel when lomo_synth/lib/libsynthgen.so is built; otherwise (and
    on the CPU) the same integer recipe runs as torch tensor ops.
    """
    import torch

    n = 1
    for d in shape:
        n *= int(d)
    if out is None:
        out = torch.empty(n, dtype=torch.float16, device=device)
    flat_out = out.view(-1)
    m = float(np.float32(mult))
    lib = None if force_torch_ops else _gen_lib()
    if lib is not None and flat_out.is_cuda:
        import ctypes
        rc = lib.synth_normal_f16(key & MASK64, 0, n, m, ctypes.c_void_p(flat_out.data_ptr()),
                                  ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        if rc != 0:
            raise RuntimeError("synth_normal_f16 launch failed")
        return out.view(*[int(d) for d in shape])
    chunk = 1 << 24
    k, g, m1, m2 = _i64(key), _i64(GOLDEN), _i64(MIX1), _i64(MIX2)
    for i0 in range(0, n, chunk):
        i1 = min(n, i0 + chunk)
        idx = torch.arange(i0, i1, dtype=torch.int64, device=device)
        s = torch.zeros(i1 - i0, dtype=torch.int64, device=device)
        for j in range(3):
            z = (idx * 3 + (j + 1)) * g + k
            z = (z ^ ((z >> 30) & ((1 << 34) - 1))) * m1
            z = (z ^ ((z >> 27) & ((1 << 37) - 1))) * m2
            z = z ^ ((z >> 31) & ((1 << 33) - 1))
            for f in range(4):
                s += (z >> (16 * f)) & 0xFFFF
        s -= 6 * 65535
        flat_out[i0:i1] = (s.to(torch.float32) * m).to(torch.float16)
    return out.view(*[int(d) for d in shape])


def zipf_ids(seed: int, T: int, V: int, a: float = 1.1) -> np.ndarray:
    """Token ids with bounded-Zipf(a) frequencies over V ids, hot ids spread uniformly.

    Rank r in 1..V has probability proportional to r^-a; a seeded permutation maps ranks
    to ids, so the popular ids are scattered over [0, V) instead of clustered near zero.
    """
    kid = tensor_key(seed, 0, 0, ROLE_IDS)
    kperm = tensor_key(seed, 0, 0, ROLE_PERM)
    p = np.arange(1, V + 1, dtype=np.float64) ** (-float(a))
    cdf = np.cumsum(p)
    cdf /= cdf[-1]
    u = (splitmix64_np(kid, np.arange(T, dtype=np.uint64)) >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
    rank = np.minimum(np.searchsorted(cdf, u, side="right"), V - 1)
    perm = np.argsort(splitmix64_np(kperm, np.arange(V, dtype=np.uint64)), kind="stable")
    return perm[rank].astype(np.int32)
