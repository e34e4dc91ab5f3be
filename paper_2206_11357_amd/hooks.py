"""Saved-tensor hooks that route autograd's saved activations through the GACT
compressor (arXiv 2206.11357, Sec. 5: one hook interface for all operators;
Sec. 5.2: parameters and tensors that need no gradient are not quantized;
Sec. 5.3: optional swap of the *compressed* tensors to host memory on two side
streams (one out, one in), with prefetch during the backward pass).

This is glue around the library's kernels: ``pack`` calls ``gact_compress``,
``unpack`` calls ``gact_decompress``.  Per-tensor bit widths and the
replayable per-tensor seeds r_l of Alg. 1 come from the ``Controller``.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np
import torch

from . import (GACT_BITS_UNCOMPRESSED, gact_allocate_bits_levels, gact_compress, gact_compress_footprint,
               gact_decompress, gact_num_groups, gact_packed_bytes, gact_sensitivity)


@dataclass
class _Packed:
    index: int                 # position among the context tensors of this iteration
    shape: torch.Size
    dtype: torch.dtype
    n: int
    bits: int
    packed: Optional[torch.Tensor]
    gmin: Optional[torch.Tensor]
    gscale: Optional[torch.Tensor]
    blob: Optional[torch.Tensor] = None   # swap mode: the one device buffer the three above are views of
    host: Optional[torch.Tensor] = None   # pinned copy of the blob when swapped out
    out_event: Optional[torch.cuda.Event] = None
    in_event: Optional[torch.cuda.Event] = None


class Controller:
    """Holds the compression scheme b = (b_l), the seeds (r_l) and the
    sensitivities c_l of the context tensors of one model."""

    def __init__(self, params: Sequence[torch.Tensor] = (), group_size: int = 256, bits: int = 4,
                 seed: int = 0, min_numel: int = 1024, swap: bool = False, dedup: bool = False):
        self.group_size = group_size
        self.default_bits = bits
        self.base_seed = seed
        self.min_numel = min_numel
        self.swap = swap
        # dedup: a tensor saved by several operators is compressed once.  The data pointer
        # alone cannot identify it (the allocator hands a freed activation's address to the
        # next one), so candidates are confirmed by their footprint: sum + sampled points
        # (Sec. 5.2), taken by the compressor in the same read; a duplicate's new copy is dropped.
        self.dedup = dedup
        self.param_ptrs = {p.data_ptr() for p in params}
        self.bits: Dict[int, int] = {}            # index l -> b_l
        self.seed_override: Dict[int, int] = {}   # index l -> r_l (Alg. 1 reseeds one tensor)
        self.numel: List[int] = []                # D_l seen in the last iteration
        self.sensitivity: Optional[np.ndarray] = None
        self._index = 0
        self._live: Dict[int, _Packed] = {}
        self._by_storage: Dict[tuple, tuple] = {}   # (ptr, numel, dtype) -> (handle, footprint)
        # swap-out and swap-in each on a stream of their own (Sec. 5.3), both at default priority
        self._out_stream = torch.cuda.Stream() if swap else None
        self._in_stream = torch.cuda.Stream() if swap else None
        # pinned host memory for the swapped tensors: one arena, handed out front to back within
        # an iteration (a pinned allocation per tensor costs more than the copy it serves)
        self._arena: Optional[torch.Tensor] = None
        self._arena_used = 0

    # ------------------------------------------------------------- iteration
    def begin_iteration(self) -> None:
        # The arena is reused from its start: the copies that read it in the last backward
        # pass were waited for by the main stream, which orders them before this iteration's
        # swap-outs (those wait for an event the main stream records after compressing).
        self._arena_used = 0
        self._index = 0
        self._live.clear()
        self._by_storage.clear()
        self.numel = []

    def seed_of(self, index: int) -> int:
        return self.seed_override.get(index, self.base_seed * 1_000_003 + index)

    def bits_of(self, index: int) -> int:
        return self.bits.get(index, self.default_bits)

    def _eligible(self, x: torch.Tensor) -> bool:
        return (x.is_cuda and x.dtype in (torch.float32, torch.bfloat16) and x.numel() >= self.min_numel
                and x.data_ptr() not in self.param_ptrs and x.is_contiguous())

    # ------------------------------------------------------------------ hooks
    def pack(self, x: torch.Tensor):
        if not self._eligible(x):
            return x
        index = self._index
        b = self.bits_of(index)
        if b == GACT_BITS_UNCOMPRESSED:
            self._index += 1
            self.numel.append(x.numel())
            return x
        blob, out = None, (None, None, None)
        if self.swap:
            # packed codes, minima and steps in one buffer, so that a swap is one copy each way
            blob = torch.empty(self._blob_bytes(x.numel(), b), dtype=torch.uint8, device=x.device)
            out = self._views(blob, x.numel(), b)
        if self.dedup:
            # one read: the sum is taken in the compressor's statistics pass
            packed, gmin, gscale, fp = gact_compress_footprint(x.detach(), self.group_size, b,
                                                               self.seed_of(index), 8, *out)
            key = (x.data_ptr(), x.numel(), x.dtype)
            hit = self._by_storage.get(key)
            if hit is not None and torch.equal(fp, hit[1]):
                return hit[0]                        # saved before in this iteration: share it, drop the new copy
        else:
            packed, gmin, gscale = gact_compress(x.detach(), self.group_size, b, self.seed_of(index), *out)
        self._index += 1
        self.numel.append(x.numel())
        h = _Packed(index, x.shape, x.dtype, x.numel(), b, packed, gmin, gscale, blob)
        if self.swap:
            self._swap_out(h)
        self._live[index] = h
        if self.dedup:
            self._by_storage[key] = (h, fp)
        return h

    def unpack(self, h):
        if not isinstance(h, _Packed):
            return h
        if h.host is not None:
            self._swap_in(h)
            nxt = self._live.get(h.index - 1)          # backward walks the tensors in reverse
            if nxt is not None and nxt.host is not None and nxt.packed is None:
                self._start_swap_in(nxt)
            torch.cuda.current_stream().wait_event(h.in_event)
        y = gact_decompress(h.packed, h.gmin, h.gscale, h.n, self.group_size, h.bits, dtype=h.dtype)
        return y.view(h.shape)

    def hooks(self):
        """Context manager: ``with controller.hooks(): loss = model(x)``."""
        return torch.autograd.graph.saved_tensors_hooks(self.pack, self.unpack)

    # ------------------------------------------------------------------- swap
    def _pinned(self, like: torch.Tensor) -> torch.Tensor:
        """A pinned host buffer shaped like `like`, cut from the arena."""
        nbytes = like.numel() * like.element_size()
        start = (self._arena_used + 255) & ~255
        if self._arena is None or start + nbytes > self._arena.numel():
            # grow: handles of this iteration keep the old arena's storage alive through their views
            grown = max(2 * (self._arena.numel() if self._arena is not None else 0), nbytes, 64 << 20)
            self._arena = torch.empty(grown, dtype=torch.uint8, pin_memory=True)
            start = 0
        self._arena_used = start + nbytes
        return self._arena[start:start + nbytes].view(like.dtype).view(like.shape)

    def _blob_bytes(self, n: int, bits: int) -> int:
        return gact_packed_bytes(n, bits) + 8 * gact_num_groups(n, self.group_size)

    def _views(self, blob: torch.Tensor, n: int, bits: int):
        """(packed, gmin, gscale) inside `blob`; the packed size is a multiple of 16 bytes."""
        pb, ng = gact_packed_bytes(n, bits), gact_num_groups(n, self.group_size)
        return (blob[:pb], blob[pb:pb + 4 * ng].view(torch.float32),
                blob[pb + 4 * ng:pb + 8 * ng].view(torch.float32))

    def _swap_out(self, h: _Packed) -> None:
        done = torch.cuda.Event()
        done.record()                                   # compression finished on the main stream
        buf = self._pinned(h.blob)
        with torch.cuda.stream(self._out_stream):
            self._out_stream.wait_event(done)
            buf.copy_(h.blob, non_blocking=True)
            h.blob.record_stream(self._out_stream)
            h.out_event = torch.cuda.Event()
            h.out_event.record()
        h.host = buf
        h.blob = h.packed = h.gmin = h.gscale = None    # the device copy may be reused once copied

    def _start_swap_in(self, h: _Packed) -> None:
        main = torch.cuda.current_stream()
        with torch.cuda.stream(self._in_stream):
            self._in_stream.wait_event(h.out_event)
            blob = torch.empty(h.host.shape, dtype=torch.uint8, device="cuda")
            blob.copy_(h.host, non_blocking=True)
            blob.record_stream(main)
            h.in_event = torch.cuda.Event()
            h.in_event.record()
        h.blob = blob
        h.packed, h.gmin, h.gscale = self._views(blob, h.n, h.bits)

    def _swap_in(self, h: _Packed) -> None:
        if h.packed is None:
            self._start_swap_in(h)

    # ------------------------------------------------------------ adaptation
    def compute_sensitivities(self, fwdbwd: Callable[[], Sequence[torch.Tensor]]) -> np.ndarray:
        """Alg. 1 for every context tensor.  ``fwdbwd`` runs one forward and
        backward pass under ``self.hooks()`` on a fixed batch and returns the
        gradient buffers.  L + 1 passes: one with the seeds (r_l), then one per
        tensor with only that tensor's seed replaced by r_{L+1}."""
        self.seed_override.clear()
        self.begin_iteration()
        g0 = [g.detach().clone() for g in fwdbwd()]
        L = len(self.numel)
        c = np.zeros(L, dtype=np.float32)
        for l in range(L):
            if self.bits_of(l) == GACT_BITS_UNCOMPRESSED:
                continue
            self.seed_override = {l: self.base_seed * 1_000_003 + L + 1_000_000}
            self.begin_iteration()
            g1 = fwdbwd()
            c[l] = float(gact_sensitivity(g0, [g.detach() for g in g1], self.bits_of(l)).item())
        self.seed_override.clear()
        self.sensitivity = c
        return c

    def adapt(self, avg_bits: float, levels=(1, 2, 4, 8)) -> np.ndarray:
        """Solve Eq. (ilp) for the sensitivities measured last."""
        assert self.sensitivity is not None and len(self.numel) == len(self.sensitivity)
        b = gact_allocate_bits_levels(self.sensitivity, self.numel, avg_bits, levels)
        self.bits = {l: int(v) for l, v in enumerate(b)}
        return b
