"""CPU oracle of the GACT quantizer (arXiv 2206.11357, App. A.4; Eq. (ilp)).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's cpu_baseline leg.  The product package never imports this.

The arithmetic lives in ``gact_oracle.c`` (scalar C, built with gcc,
``-ffp-contract=off``); this module only builds it, loads it with ctypes and
marshals numpy arrays.  bf16 tensors travel as ``uint16`` arrays holding the
raw bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

F32 = 0
BF16 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gact_oracle.c")
_LIB = os.path.join(_HERE, "libgact_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
          "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the C oracle next to its source; returns the library path."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, u64, i32 = ctypes.c_int64, ctypes.c_uint64, ctypes.c_int
        vp = ctypes.c_void_p
        L.gact_oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.gact_oracle_philox4x32_10.restype = None
        L.gact_oracle_threads.argtypes = []
        L.gact_oracle_threads.restype = i32
        L.gact_oracle_set_threads.argtypes = [i32]
        L.gact_oracle_set_threads.restype = None
        L.gact_oracle_noise.argtypes = [u64, u64]
        L.gact_oracle_noise.restype = ctypes.c_float
        L.gact_oracle_noise_fill.argtypes = [u64, u64, i64, vp]
        L.gact_oracle_noise_fill.restype = None
        L.gact_oracle_num_groups.argtypes = [i64, i32]
        L.gact_oracle_num_groups.restype = i64
        L.gact_oracle_packed_bytes.argtypes = [i64, i32]
        L.gact_oracle_packed_bytes.restype = i64
        L.gact_oracle_compress.argtypes = [vp, i32, i64, i32, i32, u64, vp, vp, vp]
        L.gact_oracle_compress.restype = i32
        L.gact_oracle_compress_with_noise.argtypes = [vp, i32, i64, i32, i32, vp, vp, vp, vp]
        L.gact_oracle_compress_with_noise.restype = i32
        L.gact_oracle_decompress.argtypes = [vp, vp, vp, i64, i32, i32, vp, i32]
        L.gact_oracle_decompress.restype = i32
        L.gact_oracle_unpack_codes.argtypes = [vp, i64, i32, vp]
        L.gact_oracle_unpack_codes.restype = i32
        L.gact_oracle_allocate_bits.argtypes = [vp, vp, i32, ctypes.c_double, vp]
        L.gact_oracle_allocate_bits.restype = i32
        L.gact_oracle_allocate_bits_levels.argtypes = [vp, vp, i32, ctypes.c_double, vp, i32, vp]
        L.gact_oracle_allocate_bits_levels.restype = i32
        L.gact_oracle_footprint.argtypes = [vp, i64, i32, i32, vp]
        L.gact_oracle_footprint.restype = i32
        L.gact_oracle_sensitivity.argtypes = [vp, vp, vp, vp, i32, i32, vp]
        L.gact_oracle_sensitivity.restype = i32
        L.gact_oracle_grad_stats_update.argtypes = [vp, vp, i64, i32, i64, vp, vp]
        L.gact_oracle_grad_stats_update.restype = i32
        L.gact_oracle_variance_ratio.argtypes = [vp, vp, i32, ctypes.c_double, vp]
        L.gact_oracle_variance_ratio.restype = i32
        _lib = L
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _dtype_of(x: np.ndarray) -> int:
    if x.dtype == np.float32:
        return F32
    if x.dtype == np.uint16:
        return BF16
    raise TypeError("oracle takes float32, or uint16 holding bf16 bit patterns")


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    lib().gact_oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def threads() -> int:
    return int(lib().gact_oracle_threads())


def set_threads(n: int) -> None:
    """Run the oracle's loops on n threads from now on (results do not depend on it)."""
    lib().gact_oracle_set_threads(int(n))


def noise(seed: int, i: int) -> float:
    return float(lib().gact_oracle_noise(seed & (2**64 - 1), i))


def num_groups(n: int, group_size: int) -> int:
    return int(lib().gact_oracle_num_groups(n, group_size))


def packed_bytes(n: int, bits: int) -> int:
    return int(lib().gact_oracle_packed_bytes(n, bits))


def compress(x: np.ndarray, group_size: int, bits: int, seed: int):
    """-> (packed uint8[packed_bytes], gmin f32[NG], gscale f32[NG])"""
    x = np.ascontiguousarray(x).reshape(-1)
    dt = _dtype_of(x)
    n = x.size
    packed = np.empty(max(packed_bytes(n, bits), 0), dtype=np.uint8)
    ng = (n + group_size - 1) // group_size if group_size > 0 else 0
    gmin = np.empty(ng, dtype=np.float32)
    gscale = np.empty(ng, dtype=np.float32)
    rc = lib().gact_oracle_compress(_ptr(x), dt, n, group_size, bits,
                                    seed & (2**64 - 1), _ptr(packed),
                                    _ptr(gmin), _ptr(gscale))
    if rc != 0:
        raise ValueError("gact_oracle_compress: bad argument (rc=%d)" % rc)
    return packed, gmin, gscale


def compress_with_noise(x: np.ndarray, group_size: int, bits: int, u: np.ndarray):
    """Same quantizer, rounding noise u (float32, one per element) supplied."""
    x = np.ascontiguousarray(x).reshape(-1)
    u = np.ascontiguousarray(u, dtype=np.float32).reshape(-1)
    assert u.size == x.size
    dt = _dtype_of(x)
    n = x.size
    packed = np.empty(packed_bytes(n, bits), dtype=np.uint8)
    ng = (n + group_size - 1) // group_size
    gmin = np.empty(ng, dtype=np.float32)
    gscale = np.empty(ng, dtype=np.float32)
    rc = lib().gact_oracle_compress_with_noise(_ptr(x), dt, n, group_size, bits,
                                               _ptr(u), _ptr(packed),
                                               _ptr(gmin), _ptr(gscale))
    if rc != 0:
        raise ValueError("gact_oracle_compress_with_noise: bad argument")
    return packed, gmin, gscale


def noise_array(seed: int, n: int, start: int = 0) -> np.ndarray:
    """u for elements start .. start+n-1 under `seed`."""
    u = np.empty(n, dtype=np.float32)
    lib().gact_oracle_noise_fill(seed & (2**64 - 1), start, n, _ptr(u))
    return u


def compress_slice(x: np.ndarray, group_size: int, bits: int, seed: int, start: int):
    """Oracle result for elements start .. start+len(x)-1 of a larger tensor;
    `start` must be a multiple of the group size."""
    assert start % group_size == 0
    return compress_with_noise(x, group_size, bits, noise_array(seed, x.size, start))


def decompress(packed: np.ndarray, gmin: np.ndarray, gscale: np.ndarray,
               n: int, group_size: int, bits: int, dtype: int = F32) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    gmin = np.ascontiguousarray(gmin, dtype=np.float32)
    gscale = np.ascontiguousarray(gscale, dtype=np.float32)
    y = np.empty(n, dtype=np.float32 if dtype == F32 else np.uint16)
    rc = lib().gact_oracle_decompress(_ptr(packed), _ptr(gmin), _ptr(gscale),
                                      n, group_size, bits, _ptr(y), dtype)
    if rc != 0:
        raise ValueError("gact_oracle_decompress: bad argument (rc=%d)" % rc)
    return y


def unpack_codes(packed: np.ndarray, n: int, bits: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    codes = np.empty(n, dtype=np.uint8)
    rc = lib().gact_oracle_unpack_codes(_ptr(packed), n, bits, _ptr(codes))
    if rc != 0:
        raise ValueError("gact_oracle_unpack_codes: bad argument")
    return codes


def allocate_bits_levels(sensitivity, numel, avg_bit_budget: float, levels) -> np.ndarray:
    c = np.ascontiguousarray(sensitivity, dtype=np.float32)
    d = np.ascontiguousarray(numel, dtype=np.int64)
    lv = np.ascontiguousarray(levels, dtype=np.int32)
    assert c.shape == d.shape and c.ndim == 1
    out = np.empty(c.size, dtype=np.int32)
    rc = lib().gact_oracle_allocate_bits_levels(_ptr(c), _ptr(d), c.size, float(avg_bit_budget),
                                                _ptr(lv), lv.size, _ptr(out))
    if rc != 0:
        raise ValueError("gact_oracle_allocate_bits_levels: rc=%d" % rc)
    return out


def allocate_bits(sensitivity, numel, avg_bit_budget: float) -> np.ndarray:
    c = np.ascontiguousarray(sensitivity, dtype=np.float32)
    d = np.ascontiguousarray(numel, dtype=np.int64)
    assert c.shape == d.shape and c.ndim == 1
    out = np.empty(c.size, dtype=np.int32)
    rc = lib().gact_oracle_allocate_bits(_ptr(c), _ptr(d), c.size,
                                         float(avg_bit_budget), _ptr(out))
    if rc != 0:
        raise ValueError("gact_oracle_allocate_bits: rc=%d" % rc)
    return out


def sensitivity(g0, g1, bits: int) -> float:
    """Alg. 1's return value: 1/2 ||g0 - g1||^2 / S(bits) over lists of buffers
    (float32 arrays, or uint16 arrays of bf16 bit patterns)."""
    g0 = [np.ascontiguousarray(a).reshape(-1) for a in g0]
    g1 = [np.ascontiguousarray(a).reshape(-1) for a in g1]
    assert len(g0) == len(g1) and all(a.size == b.size and a.dtype == b.dtype for a, b in zip(g0, g1))
    K = len(g0)
    P0 = (ctypes.c_void_p * max(K, 1))(*[_ptr(a) for a in g0])
    P1 = (ctypes.c_void_p * max(K, 1))(*[_ptr(a) for a in g1])
    n = np.array([a.size for a in g0], dtype=np.int64)
    dt = np.array([_dtype_of(a) for a in g0], dtype=np.int32)
    out = ctypes.c_double(0.0)
    rc = lib().gact_oracle_sensitivity(ctypes.addressof(P0), ctypes.addressof(P1), _ptr(n), _ptr(dt),
                                       K, bits, ctypes.addressof(out))
    if rc != 0:
        raise ValueError("gact_oracle_sensitivity: bad argument")
    return out.value


def grad_stats_update(g: np.ndarray, mean: np.ndarray, t: int):
    """In-place running-mean step; returns (sum g^2, sum mean_new^2)."""
    g = np.ascontiguousarray(g).reshape(-1)
    assert mean.dtype == np.float32 and mean.flags.c_contiguous and mean.size == g.size
    a, b = ctypes.c_double(0.0), ctypes.c_double(0.0)
    rc = lib().gact_oracle_grad_stats_update(_ptr(g), _ptr(mean), g.size, _dtype_of(g), t,
                                             ctypes.addressof(a), ctypes.addressof(b))
    if rc != 0:
        raise ValueError("gact_oracle_grad_stats_update: bad argument")
    return a.value, b.value


def variance_ratio(c, bits, grad_var: float) -> float:
    c = np.ascontiguousarray(c, dtype=np.float32)
    b = np.ascontiguousarray(bits, dtype=np.int32)
    out = ctypes.c_double(0.0)
    rc = lib().gact_oracle_variance_ratio(_ptr(c), _ptr(b), c.size, float(grad_var), ctypes.addressof(out))
    if rc != 0:
        raise ValueError("gact_oracle_variance_ratio: bad argument")
    return out.value


def footprint(x: np.ndarray, n_samples: int) -> np.ndarray:
    """[sum, x[floor(j n / n_samples)] for j < n_samples] as float64."""
    x = np.ascontiguousarray(x).reshape(-1)
    out = np.zeros(1 + n_samples, dtype=np.float64)
    rc = lib().gact_oracle_footprint(_ptr(x), x.size, _dtype_of(x), n_samples, _ptr(out))
    if rc != 0:
        raise ValueError("gact_oracle_footprint: bad argument")
    return out
