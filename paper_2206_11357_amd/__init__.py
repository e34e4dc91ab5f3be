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
from typing import Optional, Sequence, Tuple

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
GACT_E_CAPTURE = -6
GACT_E_SCRATCH = -7
GACT_NOALLOC_SCRATCH_BYTES = 2 << 20

EXPORTS = (
    "gact_num_groups", "gact_packed_bytes", "gact_error_string", "gact_compress",
    "gact_decompress", "gact_multi_workspace_bytes", "gact_compress_multi",
    "gact_decompress_multi", "gact_allocate_bits", "gact_reduce_workspace_bytes",
    "gact_sensitivity", "gact_grad_stats_update", "gact_variance_alert",
    "gact_allocate_bits_levels", "gact_footprint", "gact_compress_footprint",
    "gact_compress_footprint_workspace_bytes", "gact_compress_footprint_noalloc", "gact_copy_bounded",
)
GACT_BITS_UNCOMPRESSED = 32


class GactError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (code %d)" % (where, error_string(code), code))


class TensorDesc(ctypes.Structure):
    """Mirror of gact_tensor_desc."""
    _fields_ = [("x", ctypes.c_void_p), ("packed", ctypes.c_void_p), ("gmin", ctypes.c_void_p),
                ("gscale", ctypes.c_void_p), ("y", ctypes.c_void_p), ("n", ctypes.c_int64),
                ("seed", ctypes.c_uint64), ("bits", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("index_base", ctypes.c_int64)]


class GradPair(ctypes.Structure):
    """Mirror of gact_grad_pair."""
    _fields_ = [("g0", ctypes.c_void_p), ("g1", ctypes.c_void_p), ("n", ctypes.c_int64),
                ("dtype", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class GradStat(ctypes.Structure):
    """Mirror of gact_grad_stat."""
    _fields_ = [("g", ctypes.c_void_p), ("mean", ctypes.c_void_p), ("n", ctypes.c_int64),
                ("dtype", ctypes.c_int32), ("reserved", ctypes.c_int32)]


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
    lib.gact_allocate_bits_levels.argtypes = [vp, vp, i32, ctypes.c_double, vp, i32, vp]
    lib.gact_allocate_bits_levels.restype = i32
    lib.gact_reduce_workspace_bytes.argtypes = [i32, i64]
    lib.gact_reduce_workspace_bytes.restype = sz
    lib.gact_sensitivity.argtypes = [vp, i32, i32, vp, vp, sz, vp]
    lib.gact_sensitivity.restype = i32
    lib.gact_grad_stats_update.argtypes = [vp, i32, i64, vp, vp, sz, vp]
    lib.gact_grad_stats_update.restype = i32
    lib.gact_footprint.argtypes = [vp, i32, i64, i32, vp, vp, sz, vp]
    lib.gact_footprint.restype = i32
    lib.gact_compress_footprint_workspace_bytes.argtypes = [i64, i32]
    lib.gact_compress_footprint_workspace_bytes.restype = sz
    lib.gact_compress_footprint.argtypes = [vp, i32, i64, i32, i32, ctypes.c_uint64, vp, vp, vp, i32, vp,
                                            vp, sz, vp]
    lib.gact_compress_footprint.restype = i32
    lib.gact_compress_footprint_noalloc.argtypes = [vp, i32, i64, i32, i32, ctypes.c_uint64, vp, vp, vp, i32, vp, vp]
    lib.gact_compress_footprint_noalloc.restype = i32
    lib.gact_copy_bounded.argtypes = [vp, vp, sz, i32, vp]
    lib.gact_copy_bounded.restype = i32
    lib.gact_variance_alert.argtypes = [vp, vp, i32, ctypes.c_double, ctypes.c_double, vp]
    lib.gact_variance_alert.restype = i32
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


_DTYPE_CODES = {torch.float32: GACT_F32, torch.bfloat16: GACT_BF16}


def dtype_code(dtype: torch.dtype) -> int:
    try:
        return _DTYPE_CODES[dtype]
    except KeyError:
        raise TypeError("gact handles float32 and bfloat16 tensors, got %s" % dtype) from None


def _stream(stream) -> int:
    """hipStream_t as an integer: None = torch's current stream; a torch stream; or the integer itself
    (a call site that issues many calls resolves the stream once and passes the handle)."""
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if type(stream) is int:
        return stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(x: torch.Tensor) -> torch.Tensor:
    if not x.is_cuda:
        raise ValueError("gact needs device tensors")
    if not x.is_contiguous():
        raise ValueError("gact needs contiguous tensors")
    return x


def _flat(x: torch.Tensor) -> torch.Tensor:
    return _check(x).view(-1)


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
    n = _check(x).numel()
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
                             group_size, bits, _check(y).data_ptr(), dtype_code(y.dtype),
                             _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_decompress")
    return y


class PreparedCall:
    """One single-tensor call with its arguments marshalled once: ``call(stream_handle)`` enqueues it
    on that stream (an integer hipStream_t, e.g. ``torch.cuda.current_stream().cuda_stream``).  For
    loops that issue the same call many times (a serving loop, one call per saved tensor and step):
    nothing is looked up or converted per call.  The object keeps the tensors alive."""
    __slots__ = ("_fn", "_args", "_name", "_keep")

    def __init__(self, fn, name, args, keep):
        self._fn, self._name, self._args, self._keep = fn, name, args, keep

    def __call__(self, stream_handle: int = 0) -> None:
        rc = self._fn(*self._args, stream_handle)
        if rc != GACT_OK:
            raise GactError(rc, self._name)


def prepare_compress(x: torch.Tensor, group_size: int, bits: int, seed: int, packed: torch.Tensor,
                     gmin: torch.Tensor, gscale: torch.Tensor) -> PreparedCall:
    """gact_compress(x, ...) into the given buffers, as a PreparedCall."""
    vp = ctypes.c_void_p
    args = (vp(_check(x).data_ptr()), dtype_code(x.dtype), ctypes.c_int64(x.numel()), group_size, bits,
            ctypes.c_uint64(seed & (2**64 - 1)), vp(packed.data_ptr()), vp(gmin.data_ptr()), vp(gscale.data_ptr()))
    return PreparedCall(lib.gact_compress, "gact_compress", args, (x, packed, gmin, gscale))


def prepare_decompress(packed: torch.Tensor, gmin: torch.Tensor, gscale: torch.Tensor, n: int,
                       group_size: int, bits: int, y: torch.Tensor) -> PreparedCall:
    """gact_decompress(...) into y, as a PreparedCall."""
    vp = ctypes.c_void_p
    args = (vp(packed.data_ptr()), vp(gmin.data_ptr()), vp(gscale.data_ptr()), ctypes.c_int64(n), group_size, bits,
            vp(_check(y).data_ptr()), dtype_code(y.dtype))
    return PreparedCall(lib.gact_decompress, "gact_decompress", args, (packed, gmin, gscale, y))


# ---------------------------------------------------------------- multi tensor
def make_descs(xs: Sequence[Optional[torch.Tensor]], packed: Sequence[torch.Tensor],
               gmin: Sequence[torch.Tensor], gscale: Sequence[torch.Tensor],
               ys: Sequence[Optional[torch.Tensor]], ns: Sequence[int], bits: Sequence[int],
               seeds: Sequence[int], dtypes: Sequence[torch.dtype],
               index_bases: Optional[Sequence[int]] = None):
    """ctypes array of gact_tensor_desc from per-tensor buffers; index_bases gives each
    entry's offset in its tensor's noise stream when the entries are shards (default 0)."""
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
        d.index_base = int(index_bases[l]) if index_bases is not None else 0
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


def gact_allocate_bits_levels(sensitivity, numel, avg_bit_budget: float, levels) -> np.ndarray:
    """Allocator over a level set drawn from {1, 2, 4, 8, 32}; 32 = leave uncompressed."""
    c = np.ascontiguousarray(sensitivity, dtype=np.float32)
    d = np.ascontiguousarray(numel, dtype=np.int64)
    lv = np.ascontiguousarray(levels, dtype=np.int32)
    if c.shape != d.shape or c.ndim != 1 or lv.ndim != 1:
        raise ValueError("sensitivity and numel must be 1-D and of equal length")
    out = np.empty(c.size, dtype=np.int32)
    rc = lib.gact_allocate_bits_levels(c.ctypes.data, d.ctypes.data, c.size, float(avg_bit_budget),
                                       lv.ctypes.data, lv.size, out.ctypes.data)
    if rc != GACT_OK:
        raise GactError(rc, "gact_allocate_bits_levels")
    return out


# ------------------------------------------------- sensitivity and the alert
def gact_reduce_workspace_bytes(K: int, total_elems: int) -> int:
    return int(lib.gact_reduce_workspace_bytes(K, total_elems))


def _reduce_workspace(tensors, workspace):
    total = sum(int(t.numel()) for t in tensors)
    need = gact_reduce_workspace_bytes(len(tensors), total)
    if workspace is None:
        dev = tensors[0].device if tensors else torch.device("cuda")
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    return workspace


def make_grad_pairs(g0: Sequence[torch.Tensor], g1: Sequence[torch.Tensor]):
    """ctypes array of gact_grad_pair (reusable across calls while the buffers live)."""
    K = len(g0)
    if len(g1) != K:
        raise ValueError("g0 and g1 must list the same buffers")
    arr = (GradPair * max(K, 1))()
    for k in range(K):
        a, b = _flat(g0[k]), _flat(g1[k])
        if a.numel() != b.numel() or a.dtype != b.dtype:
            raise ValueError("buffer %d: g0 and g1 differ in size or dtype" % k)
        arr[k].g0, arr[k].g1, arr[k].n, arr[k].dtype = a.data_ptr(), b.data_ptr(), a.numel(), dtype_code(a.dtype)
    return arr


def make_grad_stats(g: Sequence[torch.Tensor], mean: Sequence[torch.Tensor]):
    """ctypes array of gact_grad_stat."""
    K = len(g)
    if len(mean) != K:
        raise ValueError("g and mean must list the same buffers")
    arr = (GradStat * max(K, 1))()
    for k in range(K):
        a, m = _flat(g[k]), _flat(mean[k])
        if a.numel() != m.numel() or m.dtype != torch.float32:
            raise ValueError("buffer %d: mean must be float32 of the gradient's size" % k)
        arr[k].g, arr[k].mean, arr[k].n, arr[k].dtype = a.data_ptr(), m.data_ptr(), a.numel(), dtype_code(a.dtype)
    return arr


def gact_sensitivity(g0: Sequence[torch.Tensor], g1: Sequence[torch.Tensor], bits: int,
                     out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                     stream=None, pairs=None) -> torch.Tensor:
    """1/2 ||g0 - g1||^2 / S(bits) over lists of gradient buffers -> device float64[1].
    `pairs` (from make_grad_pairs) skips re-marshalling the buffer list."""
    K = len(g0)
    arr = pairs if pairs is not None else make_grad_pairs(g0, g1)
    workspace = _reduce_workspace(list(g0), workspace)
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=workspace.device)
    rc = lib.gact_sensitivity(ctypes.addressof(arr), K, bits, out.data_ptr(), workspace.data_ptr(),
                              workspace.numel(), _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_sensitivity")
    return out


def gact_grad_stats_update(g: Sequence[torch.Tensor], mean: Sequence[torch.Tensor], t: int,
                           out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                           stream=None, stats=None) -> torch.Tensor:
    """Running-mean step t over gradient buffers -> device float64[2] = (sum g^2, sum mean^2)."""
    K = len(g)
    arr = stats if stats is not None else make_grad_stats(g, mean)
    workspace = _reduce_workspace(list(g), workspace)
    if out is None:
        out = torch.empty(2, dtype=torch.float64, device=workspace.device)
    rc = lib.gact_grad_stats_update(ctypes.addressof(arr), K, t, out.data_ptr(), workspace.data_ptr(),
                                    workspace.numel(), _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_grad_stats_update")
    return out


def gact_footprint(x: torch.Tensor, n_samples: int = 8, out: Optional[torch.Tensor] = None,
                   workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """-> device float64[1 + n_samples]: sum of x, then n_samples evenly spaced elements."""
    x = _flat(x)
    workspace = _reduce_workspace([x], workspace)
    if out is None:
        out = torch.empty(1 + n_samples, dtype=torch.float64, device=x.device)
    rc = lib.gact_footprint(x.data_ptr(), dtype_code(x.dtype), x.numel(), n_samples, out.data_ptr(),
                            workspace.data_ptr(), workspace.numel(), _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_footprint")
    return out


def gact_compress_footprint_workspace_bytes(n: int, group_size: int) -> int:
    return int(lib.gact_compress_footprint_workspace_bytes(int(n), int(group_size)))


def gact_compress_footprint(x: torch.Tensor, group_size: int, bits: int, seed: int, n_samples: int = 8,
                            packed: Optional[torch.Tensor] = None, gmin: Optional[torch.Tensor] = None,
                            gscale: Optional[torch.Tensor] = None, footprint: Optional[torch.Tensor] = None,
                            workspace: Optional[torch.Tensor] = None, stream=None):
    """Compress one tensor and take its footprint in the same read;
    returns (packed, gmin, gscale, footprint float64[1 + n_samples])."""
    x = _flat(x)
    n = x.numel()
    if packed is None:
        packed, gmin, gscale = alloc_compressed(n, max(group_size, 1), bits if bits > 0 else 1, x.device)
    if footprint is None:
        footprint = torch.empty(1 + n_samples, dtype=torch.float64, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(gact_compress_footprint_workspace_bytes(n, group_size), 16),
                                dtype=torch.uint8, device=x.device)
    rc = lib.gact_compress_footprint(x.data_ptr(), dtype_code(x.dtype), n, group_size, bits,
                                     seed & (2**64 - 1), packed.data_ptr(), gmin.data_ptr(),
                                     gscale.data_ptr(), n_samples, footprint.data_ptr(),
                                     workspace.data_ptr(), workspace.numel(), _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_compress_footprint")
    return packed, gmin, gscale, footprint


def gact_compress_footprint_noalloc(x: torch.Tensor, group_size: int, bits: int, seed: int, n_samples: int,
                                    packed: torch.Tensor, gmin: torch.Tensor, gscale: torch.Tensor,
                                    footprint: torch.Tensor, stream=None) -> None:
    """gact_compress_footprint on the library's own scratch area: every buffer comes from the
    caller and neither the call nor this wrapper allocates."""
    rc = lib.gact_compress_footprint_noalloc(x.data_ptr(), dtype_code(x.dtype), x.numel(), group_size, bits,
                                             seed & (2**64 - 1), packed.data_ptr(), gmin.data_ptr(),
                                             gscale.data_ptr(), n_samples, footprint.data_ptr(),
                                             _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_compress_footprint_noalloc")


def gact_copy_bounded(dst: torch.Tensor, src: torch.Tensor, workgroups: int = 16, stream=None) -> None:
    """dst <- src (same byte size; device tensors or pinned host tensors) by a kernel of `workgroups` workgroups."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst and src differ in size")
    rc = lib.gact_copy_bounded(dst.data_ptr(), src.data_ptr(), nbytes, workgroups, _stream(stream))
    if rc != GACT_OK:
        raise GactError(rc, "gact_copy_bounded")


def gact_variance_alert(sensitivity, bits, grad_var: float, threshold: float):
    """-> (alert: bool, V(b) / grad_var)"""
    c = np.ascontiguousarray(sensitivity, dtype=np.float32)
    b = np.ascontiguousarray(bits, dtype=np.int32)
    if c.shape != b.shape or c.ndim != 1:
        raise ValueError("sensitivity and bits must be 1-D and of equal length")
    ratio = ctypes.c_double(0.0)
    rc = lib.gact_variance_alert(c.ctypes.data, b.ctypes.data, c.size, float(grad_var),
                                 float(threshold), ctypes.addressof(ratio))
    if rc < 0:
        raise GactError(rc, "gact_variance_alert")
    return bool(rc), ratio.value
