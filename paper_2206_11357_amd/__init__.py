"""MI355X-native GACT activation compressor / decompressor (arXiv 2206.11357).

Thin ctypes binding over ``libgact.so`` (hand-written HIP for gfx950 behind the
C ABI of ``include/gact.h``).  The functions carry the C names and only marshal
arguments: torch supplies device memory and the current stream, every step of
the path runs in the library's kernels.  There is no CPU fallback: if the
shared library cannot be loaded the import fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch   # imported before the library so that both share one HIP runtime

from . import build as _build

GACT_F32 = 0
GACT_BF16 = 1

GACT_OK = 0
GACT_E_ARG = -1
GACT_E_BITS = -2
GACT_E_GROUP = -3
GACT_E_BUDGET = -4
GACT_E_HIP = -5

EXPORTS = (
    "gact_num_groups", "gact_packed_bytes", "gact_error_string", "gact_compress",
    "gact_decompress", "gact_multi_workspace_bytes", "gact_compress_multi",
    "gact_decompress_multi", "gact_allocate_bits",
)


class GactError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (code %d)" % (where, error_string(code), code))


class TensorDesc(ctypes.Structure):
    """Mirror of gact_tensor_desc."""
    _fields_ = [("x", ctypes.c_void_p), ("packed", ctypes.c_void_p), ("gmin", ctypes.c_void_p),
                ("gscale", ctypes.c_void_p), ("y", ctypes.c_void_p), ("n", ctypes.c_int64),
                ("seed", ctypes.c_uint64), ("bits", ctypes.c_int32), ("dtype", ctypes.c_int32)]


def _load() -> ctypes.CDLL:
    path = _build.LIB
    if not os.path.exists(path):
        _build.build()
    lib = ctypes.CDLL(path)
    vp, i64, u64, i32, sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int,
                             ctypes.c_size_t)
    lib.gact_num_groups.argtypes = [i64, i32]
    lib.gact_num_groups.restype = sz
    lib.gact_packed_bytes.argtypes = [i64, i32]
    lib.gact_packed_bytes.restype = sz
    lib.gact_error_string.argtypes = [i32]
    lib.gact_error_string.restype = ctypes.c_char_p
    lib.gact_compress.argtypes = [vp, i32, i64, i32, i32, u64, vp, vp, vp, vp]
    lib.gact_compress.restype = i32
    lib.gact_decompress.argtypes = [vp, vp, vp, i64, i32, i32, vp, i32, vp]
    lib.gact_decompress.restype = i32
    lib.gact_multi_workspace_bytes.argtypes = [i32]
    lib.gact_multi_workspace_bytes.restype = sz
    lib.gact_compress_multi.argtypes = [vp, i32, i32, vp, sz, vp]
    lib.gact_compress_multi.restype = i32
    lib.gact_decompress_multi.argtypes = [vp, i32, i32, vp, sz, vp]
    lib.gact_decompress_multi.restype = i32
    lib.gact_allocate_bits.argtypes = [vp, vp, i32, ctypes.c_double, vp]
    lib.gact_allocate_bits.restype = i32
    return lib


lib = _load()


# ------------------------------------------------------------------ helpers
def error_string(code: int) -> str:
    return lib.gact_error_string(code).decode()


def gact_num_groups(n: int, group_size: int) -> int:
    return int(lib.gact_num_groups(n, group_size))


def gact_packed_bytes(n: int, bits: int) -> int:
    return int(lib.gact_packed_bytes(n, bits))


def gact_multi_workspace_bytes(L: int) -> int:
    return int(lib.gact_multi_workspace_bytes(L))


def dtype_code(dtype: torch.dtype) -> int:
    if dtype == torch.float32:
        return GACT_F32
    if dtype == torch.bfloat16:
        return GACT_BF16
    raise TypeError("gact handles float32 and bfloat16 tensors, got %s" % dtype)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _flat(x: torch.Tensor) -> torch.Tensor:
    if not x.is_cuda:
        raise ValueError("gact needs device tensors")
    if not x.is_contiguous():
        raise ValueError("gact needs contiguous tensors")
    return x.view(-1)


def alloc_compressed(n: int, group_size: int, bits: int, device) -> Tuple[torch.Tensor, ...]:
    """(packed uint8, gmin f32, gscale f32) buffers of the sizes the C ABI asks for."""
    packed = torch.empty(gact_packed_bytes(n, bits), dtype=torch.uint8, device=device)
    ng = gact_num_groups(n, group_size)
    gmin = torch.empty(ng, dtype=torch.float32, device=device)
    gscale = torch.empty(ng, dtype=torch.float32, device=device)
    return packed, gmin, gscale


# --------------------------------------------------------------- single tensor
def gact_compress(x: torch.Tensor, group_size: int, bits: int, seed: int,
                  packed: Optional[torch.Tensor] = None, gmin: Optional[torch.Tensor] = None,
                  gscale: Optional[torch.Tensor] = None, stream=None):
    """Compress one tensor; returns (packed, gmin, gscale) device tensors."""
    x = _flat(x)
    n = x.numel()
    if packed is None:
        packed, gmin, gscale = alloc_compressed(n, max(group_size, 1), bits if bits > 0 else 1,
                                                x.device)
    rc = lib.gact_compress(x.data_ptr(), dtype_code(x.dtype), n, group_size, bits,
                           seed & (2**64 - 1), packed.data_ptr(), gmin.data_ptr(),
                           gscale.data_ptr(), _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_compress")
    return packed, gmin, gscale


def gact_decompress(packed: torch.Tensor, gmin: torch.Tensor, gscale: torch.Tensor, n: int,
                    group_size: int, bits: int, dtype: torch.dtype = torch.float32,
                    y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Decompress into y (allocated when not given); returns y."""
    if y is None:
        y = torch.empty(n, dtype=dtype, device=packed.device)
    rc = lib.gact_decompress(packed.data_ptr(), gmin.data_ptr(), gscale.data_ptr(), n,
                             group_size, bits, _flat(y).data_ptr(), dtype_code(y.dtype),
                             _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_decompress")
    return y


# ---------------------------------------------------------------- multi tensor
def make_descs(xs: Sequence[Optional[torch.Tensor]], packed: Sequence[torch.Tensor],
               gmin: Sequence[torch.Tensor], gscale: Sequence[torch.Tensor],
               ys: Sequence[Optional[torch.Tensor]], ns: Sequence[int], bits: Sequence[int],
               seeds: Sequence[int], dtypes: Sequence[torch.dtype]):
    """ctypes array of gact_tensor_desc from per-tensor buffers."""
    L = len(ns)
    arr = (TensorDesc * max(L, 1))()
    for l in range(L):
        d = arr[l]
        d.x = xs[l].data_ptr() if xs[l] is not None else None
        d.y = ys[l].data_ptr() if ys[l] is not None else None
        d.packed = packed[l].data_ptr()
        d.gmin = gmin[l].data_ptr()
        d.gscale = gscale[l].data_ptr()
        d.n = int(ns[l])
        d.seed = int(seeds[l]) & (2**64 - 1)
        d.bits = int(bits[l])
        d.dtype = dtype_code(dtypes[l])
    return arr


def gact_compress_multi(descs, L: int, group_size: int, workspace: torch.Tensor, stream=None):
    rc = lib.gact_compress_multi(ctypes.addressof(descs), L, group_size, workspace.data_ptr(),
                                 workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_compress_multi")


def gact_decompress_multi(descs, L: int, group_size: int, workspace: torch.Tensor, stream=None):
    rc = lib.gact_decompress_multi(ctypes.addressof(descs), L, group_size, workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_decompress_multi")


# ------------------------------------------------------------------- allocator
def gact_allocate_bits(sensitivity, numel, avg_bit_budget: float) -> np.ndarray:
    c = np.ascontiguousarray(sensitivity, dtype=np.float32)
    d = np.ascontiguousarray(numel, dtype=np.int64)
    if c.shape != d.shape or c.ndim != 1:
        raise ValueError("sensitivity and numel must be 1-D and of equal length")
    out = np.empty(c.size, dtype=np.int32)
    rc = lib.gact_allocate_bits(c.ctypes.data, d.ctypes.data, c.size, float(avg_bit_budget),
                                out.ctypes.data)
    if rc != GACT_OK:
        raise GactError(rc, "gact_allocate_bits")
    return out
