"""Saved-tensor hooks that route autograd's saved activations through the GACT
compressor (arXiv 2206.11357, Sec. 5: one hook interface for all operators;
Sec. 5.2: parameters and tensors that need no gradient are not quantized, a
tensor saved by several operators is quantized once; Sec. 5.3: optional swap of
the *compressed* tensors to host memory on two side streams (one out, one in),
with prefetch during the backward pass).

This is glue around the library's kernels and does no arithmetic of its own.
The saved tensors of one iteration are compressed in batches, one
``gact_compress_multi`` launch per batch (the multi-tensor launch exists for
exactly this: many tensors per iteration), into one buffer per batch; the
backward pass decompresses a few tensors ahead of use with one
``gact_decompress_multi`` launch, and swapping moves one buffer per batch.
Per-tensor bit widths and the replayable per-tensor seeds r_l of Alg. 1 come
from the ``Controller``.
"""
from __future__ import annotations

import ctypes
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np
import torch
from torch.multiprocessing.reductions import StorageWeakRef

from . import (GACT_BITS_UNCOMPRESSED, GACT_OK, GactError, TensorDesc, dtype_code, gact_allocate_bits_levels,
               gact_copy_bounded,
               gact_multi_workspace_bytes, gact_num_groups, gact_packed_bytes, gact_sensitivity, lib)

_MASK64 = (1 << 64) - 1
_MAX_BATCH = 64            # a launch table of at most 64 tensors travels in the kernel arguments


def _mix64(z: int) -> int:
    """splitmix64 finaliser: spreads (seed, iteration) over the 64-bit Philox key space."""
    z = (z + 0x9E3779B97F4A7C15) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


_SIDE_STREAMS: Dict[int, tuple] = {}


def _side_streams():
    """The swap-out and swap-in streams of the current device, made once per process: the runtime maps
    streams onto a few hardware queues in turn, and which queues a controller's streams share with each
    other and with the compute stream should not depend on how many controllers came before it."""
    dev = torch.cuda.current_device()
    if dev not in _SIDE_STREAMS:
        _SIDE_STREAMS[dev] = (torch.cuda.Stream(), torch.cuda.Stream())
    return _SIDE_STREAMS[dev]


class _Packed:
    """What autograd holds instead of a saved tensor."""
    __slots__ = ("index", "shape", "dtype", "n", "bits", "seed", "x", "version", "batch", "off", "y", "done",
                 "uses", "left")

    def __init__(self, index, shape, dtype, n, bits, seed, x):
        self.index, self.shape, self.dtype, self.n, self.bits, self.seed = index, shape, dtype, n, bits, seed
        self.x = x                 # the tensor itself until its batch has been compressed
        self.version = x._version
        self.batch = None          # _Batch once compressed
        self.off = None            # (packed, gmin, gscale) byte offsets inside the batch's buffer
        self.y = None              # decompressed ahead of use
        self.done = False          # handed back to autograd at least once
        self.uses = 1              # operators that saved this tensor (more than one when shared)
        self.left = 0              # of those, how many have yet to ask for the current `y`


class _Alias:
    """A second save of a tensor already held, under another shape (the softmax output that the
    attention product saves again as a batch of matrices): the same compressed data, viewed anew."""
    __slots__ = ("base", "shape")

    def __init__(self, base, shape):
        self.base, self.shape = base, shape


class _Batch:
    """Tensors compressed by one launch into one buffer.  Holds no reference to its handles (they
    point here): a cycle would keep the buffer alive until the garbage collector runs."""
    __slots__ = ("index", "count", "blob", "nbytes", "host", "out_event", "in_event", "remaining")

    def __init__(self, index, count, blob):
        self.index, self.count, self.blob, self.nbytes = index, count, blob, blob.numel()
        self.host = None           # pinned copy once swapped out
        self.out_event = None
        self.in_event = None
        self.remaining = count     # tensors not yet decompressed since the buffer came (back) to the device


class Controller:
    """Holds the compression scheme b = (b_l), the seeds (r_l) and the
    sensitivities c_l of the context tensors of one model.

    batch_tensors / batch_bytes   a batch is compressed when it holds this many tensors or bytes of
                                  uncompressed activations (they stay alive until then)
    ahead_tensors / ahead_bytes   the backward pass decompresses up to this much ahead of use
    swap, resident_bytes          swap compressed batches to pinned host memory, except the most recent
                                  `resident_bytes` of them, which the backward pass needs first
    swap_workgroups               size of the kernel that copies a batch to the host
    prefetch_batches              swapped batches fetched ahead of the one the backward pass is using
    swap_limit_bytes              None: every batch beyond `resident_bytes` is swapped.  A number: at most this
                                  many bytes per iteration, oldest batches first (the ones the backward pass
                                  needs last).  A volume that PCIe carries within the forward pass costs
                                  little; beyond it the backward pass is fed at the PCIe rate
    keep_until_copied             True: a swapped batch's device copy is let go only when its swap-out is seen
                                  finished; the backward pass uses the most recent batches (those still
                                  under way, at most `swap_inflight_batches`) from the device.  False: let
                                  go at once; the backward pass waits for every swap-out and fetches every
                                  batch back
    swap_inflight_batches         swap-outs that may be unfinished at a time; the host waits for the oldest
                                  before it compresses the next batch, which bounds the compressed data
                                  on the device during the forward pass and paces it by PCIe when more is
                                  swapped than PCIe carries
    release_after_use             True: a batch that lives on the device is freed once the backward pass has
                                  decompressed all its tensors (autograd frees a saved tensor the same way
                                  unless the graph is retained).  False: kept until the next iteration, for
                                  a second backward pass through a retained graph
    """

    def __init__(self, params: Sequence[torch.Tensor] = (), group_size: int = 256, bits: int = 4,
                 seed: int = 0, min_numel: int = 1024, swap: bool = False, dedup: bool = False,
                 batch_tensors: int = 32, batch_bytes: int = 128 << 20, ahead_tensors: int = 32,
                 ahead_bytes: int = 128 << 20, resident_bytes: int = 0, swap_workgroups: int = 16,
                 prefetch_batches: int = 8, swap_limit_bytes: Optional[int] = None,
                 keep_until_copied: bool = True, release_after_use: bool = True,
                 swap_inflight_batches: int = 8):
        self.group_size = group_size
        self.default_bits = bits
        self.base_seed = seed
        self.min_numel = min_numel
        self.swap = swap
        # dedup: a tensor that several operators save (the input shared by the Q, K and V projections)
        # is compressed once.  A weak reference to the storage of every tensor compressed in this
        # iteration tells whether that storage has been alive ever since; if so, "same storage, same
        # start and length, same version counter" identifies the tensor exactly, and no footprint has
        # to be computed.
        self.dedup = dedup
        self.batch_tensors = max(1, min(batch_tensors, _MAX_BATCH))
        self.batch_bytes = batch_bytes
        self.ahead_tensors = max(1, min(ahead_tensors, _MAX_BATCH))
        self.ahead_bytes = ahead_bytes
        self.resident_bytes = resident_bytes
        self.swap_workgroups = swap_workgroups
        self.prefetch_batches = max(1, prefetch_batches)
        self.swap_limit_bytes = swap_limit_bytes
        self.keep_until_copied = keep_until_copied
        self.release_after_use = release_after_use
        self.swap_inflight_batches = max(1, swap_inflight_batches)
        self._in_backward = False
        self._swapped_bytes = 0
        self.param_ptrs = {p.data_ptr() for p in params}
        self.bits: Dict[int, int] = {}            # index l -> b_l
        self.seed_override: Dict[int, int] = {}   # index l -> r_l (Alg. 1 reseeds one tensor)
        self.numel: List[int] = []                # D_l seen in the last iteration
        self.sensitivity: Optional[np.ndarray] = None
        # Fresh compressor randomness every training step (the convergence argument of Sec. 3 needs
        # it); Alg. 1 needs the same (r_l) in its passes, so the counter is frozen while it runs.
        self.iteration = -1
        self._frozen = False
        self._iter_key = _mix64(seed)
        self._handles: List[_Packed] = []         # by index, this iteration
        self._pending: List[_Packed] = []
        self._pending_bytes = 0
        self._pending_by_storage: Dict[tuple, tuple] = {}   # (storage weak reference, handle)
        self._batches: List[_Batch] = []
        self._resident: List[_Batch] = []         # swap mode: batches still on the device, oldest first
        self._resident_sum = 0
        self._out_inflight: List[_Batch] = []     # swap mode: swap-out enqueued, device copy still held
        self._descs = (TensorDesc * _MAX_BATCH)()
        self._ws: Optional[torch.Tensor] = None
        # swap-out and swap-in each on a stream of their own (Sec. 5.3), both at default priority
        self._out_stream, self._in_stream = _side_streams() if swap else (None, None)
        # pinned host memory for the swapped batches: one arena, handed out front to back within
        # an iteration (a pinned allocation per copy costs more than the copy it serves)
        self._arena: Optional[torch.Tensor] = None
        self._arena_used = 0

    # ------------------------------------------------------------- iteration
    def begin_iteration(self) -> None:
        # The arena is reused from its start: the copies that read it in the last backward
        # pass were waited for by the main stream, which orders them before this iteration's
        # swap-outs (those wait for an event the main stream records after compressing).
        if not self._frozen:
            self.iteration += 1
            self._iter_key = _mix64(self.base_seed ^ _mix64(self.iteration))
        self.release()
        self.numel = []

    def release(self) -> None:
        """Drop what is left of the last iteration's compressed buffers."""
        self._arena_used = 0
        self._swapped_bytes = 0
        self._handles = []
        self._pending = []
        self._pending_bytes = 0
        self._pending_by_storage = {}
        self._batches = []
        self._resident = []
        self._resident_sum = 0
        self._out_inflight = []
        self._in_backward = False

    def set_iteration(self, k: int) -> None:
        """The next ``begin_iteration`` starts iteration k: replays that iteration's seeds."""
        self.iteration = k - 1

    def seed_of(self, index: int) -> int:
        """r_l of context tensor `index` in the current iteration."""
        s = self.seed_override.get(index)
        return s if s is not None else (self._iter_key + index * 0x9E3779B97F4A7C15) & _MASK64

    def bits_of(self, index: int) -> int:
        return self.bits.get(index, self.default_bits)

    def _eligible(self, x: torch.Tensor) -> bool:
        return (x.is_cuda and x.requires_grad and x.numel() >= self.min_numel
                and x.dtype in (torch.float32, torch.bfloat16)
                and x.data_ptr() not in self.param_ptrs and x.is_contiguous())

    # ------------------------------------------------------------------ hooks
    def pack(self, x: torch.Tensor):
        if not self._eligible(x):
            return x
        if self.dedup:
            key = (x.data_ptr(), x.numel(), x.dtype)
            storage = x.untyped_storage()
            held = self._pending_by_storage.get(key)
            if held is not None:
                ref, hit = held
                # Saved before, from a storage that has been alive ever since (so the address was not
                # handed to another tensor) and with the same version counter (so nothing wrote to it):
                # the same elements in the same order, both being contiguous, whatever the shapes.
                if not ref.expired() and ref.cdata == storage._cdata and hit.version == x._version:
                    hit.uses += 1
                    return hit if hit.shape == x.shape else _Alias(hit, x.shape)
        index = len(self._handles)
        n = x.numel()
        b = self.bits_of(index)
        self.numel.append(n)
        if b == GACT_BITS_UNCOMPRESSED:
            self._handles.append(None)
            return x
        h = _Packed(index, x.shape, x.dtype, n, b, self.seed_of(index), x.detach())
        self._handles.append(h)
        self._pending.append(h)
        self._pending_bytes += n * x.element_size()
        if self.dedup:
            self._pending_by_storage[key] = (StorageWeakRef(storage), h)
        if len(self._pending) >= self.batch_tensors or self._pending_bytes >= self.batch_bytes:
            self._flush()
        return h

    def unpack(self, h):
        shape = None
        if isinstance(h, _Alias):
            h, shape = h.base, h.shape
        if not isinstance(h, _Packed):
            return h
        if not self._in_backward:
            self._begin_backward()
        if h.y is None:
            self._decompress_ahead(h)
        # one decompression serves every operator that saved the tensor; the last of them takes it away
        y, h.done = h.y, True
        h.left -= 1
        if h.left <= 0:
            h.y = None
        return y.view(h.shape if shape is None else shape)

    def _begin_backward(self) -> None:
        """First request for a saved tensor: compress what is pending; that batch stays on the device,
        it is the first one needed."""
        self._in_backward = True
        self._flush()

    def hooks(self):
        """Context manager: ``with controller.hooks(): loss = model(x)``."""
        return torch.autograd.graph.saved_tensors_hooks(self.pack, self.unpack)

    # ------------------------------------------------------------ compression
    def _workspace(self, device) -> torch.Tensor:
        if self._ws is None or self._ws.device != device:
            self._ws = torch.empty(gact_multi_workspace_bytes(_MAX_BATCH), dtype=torch.uint8, device=device)
        return self._ws

    def _flush(self) -> None:
        """One gact_compress_multi launch over the pending tensors, into one buffer."""
        pend = self._pending
        if not pend:
            return
        G = self.group_size
        total = 0
        for h in pend:
            if h.x._version != h.version:
                raise RuntimeError("a tensor saved for backward was modified in place before it was compressed")
            pb = gact_packed_bytes(h.n, h.bits)
            ng4 = 4 * gact_num_groups(h.n, G)
            mb = (ng4 + 15) & ~15
            h.off = (total, total + pb, total + pb + mb)          # all multiples of 16
            total += pb + 2 * mb
        dev = pend[0].x.device
        if self.swap:
            # At most `swap_inflight_batches` swap-outs unfinished: the host waits here for the oldest.  The
            # host runs ahead of the GPU, and memory is handed out in host order: without the wait nothing
            # that is being swapped out has been given back by the time the forward pass has been enqueued,
            # and the peak is that of a run without swapping.  With it the compressed data on the device
            # are bounded by this many batches (plus those that are not swapped at all).
            while len(self._out_inflight) >= self.swap_inflight_batches:
                self._out_inflight[0].out_event.synchronize()
                self._reap_out()
            self._reap_out()
        blob = torch.empty(total, dtype=torch.uint8, device=dev)
        base = blob.data_ptr()
        descs = self._descs
        for k, h in enumerate(pend):
            d = descs[k]
            d.x = h.x.data_ptr()
            d.packed, d.gmin, d.gscale = base + h.off[0], base + h.off[1], base + h.off[2]
            d.y = None
            d.n = h.n
            d.seed = h.seed
            d.bits = h.bits
            d.dtype = dtype_code(h.dtype)
            d.index_base = 0
        ws = self._workspace(dev)
        rc = lib.gact_compress_multi(ctypes.addressof(descs), len(pend), G, ws.data_ptr(), ws.numel(),
                                     torch.cuda.current_stream().cuda_stream)
        if rc != GACT_OK:
            raise GactError(rc, "gact_compress_multi")
        batch = _Batch(len(self._batches), len(pend), blob)
        for h in pend:
            h.batch = batch
            h.x = None                                # the uncompressed tensor may go now
        self._batches.append(batch)
        self._pending = []
        self._pending_bytes = 0
        if self.swap and not self._in_backward:       # the batch compressed as the backward pass begins is its first
            self._resident.append(batch)
            self._resident_sum += batch.nbytes
            while self._resident and self._resident_sum > self.resident_bytes:
                if (self.swap_limit_bytes is not None
                        and self._swapped_bytes + self._resident[0].nbytes > self.swap_limit_bytes):
                    break                             # this iteration's share of PCIe is used up
                old = self._resident.pop(0)
                self._resident_sum -= old.nbytes
                self._swap_out(old)

    def _decompress_ahead(self, h: _Packed) -> None:
        """One gact_decompress_multi launch for `h` and the tensors the backward pass will ask for
        next (those packed just before it), within the look-ahead limits."""
        todo, nbytes = [h], h.n * (2 if h.dtype == torch.bfloat16 else 4)
        k = h.index - 1
        while k >= 0 and len(todo) < self.ahead_tensors:
            g = self._handles[k]
            k -= 1
            if g is None or g.done or g.y is not None or g.batch is None or (g.batch.blob is None and g.batch.host is None):
                continue
            size = g.n * (2 if g.dtype == torch.bfloat16 else 4)
            if nbytes + size > self.ahead_bytes:
                break
            if self.swap and g.batch is not h.batch and g.batch.blob is None:
                self._start_swap_in(g.batch)         # prefetch its batch; decompress it on a later call
                break
            todo.append(g)
            nbytes += size
        if h.batch.blob is None and h.batch.host is None:
            raise RuntimeError("the compressed data of this tensor were released after their first use in the "
                               "backward pass; for a second pass through a retained graph construct the "
                               "Controller with release_after_use=False")
        if self.swap:
            self._ensure_on_device(h.batch)
        main = torch.cuda.current_stream()
        descs = self._descs
        dev = h.batch.blob.device
        for j, g in enumerate(todo):
            if g.batch.in_event is not None:
                main.wait_event(g.batch.in_event)
            g.y = torch.empty(g.n, dtype=g.dtype, device=dev)
            g.left = g.uses
            base = g.batch.blob.data_ptr()
            d = descs[j]
            d.x = None
            d.packed, d.gmin, d.gscale = base + g.off[0], base + g.off[1], base + g.off[2]
            d.y = g.y.data_ptr()
            d.n = g.n
            d.seed = 0
            d.bits = g.bits
            d.dtype = dtype_code(g.dtype)
            d.index_base = 0
            g.batch.remaining -= 1
        ws = self._workspace(dev)
        rc = lib.gact_decompress_multi(ctypes.addressof(descs), len(todo), self.group_size, ws.data_ptr(),
                                       ws.numel(), main.cuda_stream)
        if rc != GACT_OK:
            raise GactError(rc, "gact_decompress_multi")
        # A batch goes once all its tensors have been decompressed (the launch above is ordered before
        # the release).  A swapped batch leaves the device and a second unpack fetches it again; one that
        # lives on the device only is gone for good unless `release_after_use` is off.
        for g in todo:
            b = g.batch
            if b.remaining <= 0 and b.blob is not None:
                if b.host is not None:
                    b.blob, b.in_event, b.remaining = None, None, b.count
                elif self.release_after_use:
                    b.blob = None
        if self.swap:
            # prefetch the batches packed before this one while it is being used: several, so that the
            # copies run back to back whether the backward pass dwells on a batch or rushes through it
            # (batches still on the device need no fetch and do not count, so the first fetches start
            # with the backward pass even when the most recent batches never left)
            i = h.batch.index
            ahead = sum(1 for b in self._batches[:i] if b.in_event is not None)
            j = i - 1
            while ahead < self.prefetch_batches and j >= 0:
                b = self._batches[j]
                if b.blob is None and b.host is not None:
                    self._start_swap_in(b)
                    ahead += 1
                j -= 1

    # ------------------------------------------------------------------- swap
    def _pinned(self, nbytes: int) -> torch.Tensor:
        """A pinned host buffer of nbytes, cut from the arena."""
        start = (self._arena_used + 255) & ~255
        if self._arena is None or start + nbytes > self._arena.numel():
            # grow: batches of this iteration keep the old arena's storage alive through their views
            grown = max(2 * (self._arena.numel() if self._arena is not None else 0), nbytes, 64 << 20)
            self._arena = torch.empty(grown, dtype=torch.uint8, pin_memory=True)
            start = 0
        self._arena_used = start + nbytes
        return self._arena[start:start + nbytes]

    def _swap_out(self, batch: _Batch) -> None:
        done = torch.cuda.Event()
        done.record()                                   # its compression is enqueued on the main stream
        buf = self._pinned(batch.nbytes)
        with torch.cuda.stream(self._out_stream):
            self._out_stream.wait_event(done)
            # a copy kernel of a few workgroups: it keeps PCIe busy and leaves the wave slots of the
            # GPU to the forward pass, which the runtime's whole-chip device-to-host copy does not
            gact_copy_bounded(buf, batch.blob, self.swap_workgroups, self._out_stream)
            batch.blob.record_stream(self._out_stream)
            batch.out_event = torch.cuda.Event()
            batch.out_event.record()
        self._swapped_bytes += batch.nbytes
        batch.host = buf
        self._out_inflight.append(batch)
        if not self.keep_until_copied:
            batch.blob = None                           # the allocator reuses the memory once the copy is through

    def _reap_out(self) -> None:
        """Forward pass: let go of the device copies of batches whose swap-out has finished.  Until then
        the memory cannot be reused anyway, so the copy on the device costs nothing, and a batch the
        backward pass reaches while its swap-out is still under way (the most recent ones: the first it
        needs are the last that were sent) is used from the device without waiting for PCIe at all.
        Nothing is let go during the backward pass: memory only falls there, and a batch let go would
        be fetched back soon after."""
        q = self._out_inflight
        while q and q[0].out_event.query():
            q.pop(0).blob = None

    def _start_swap_in(self, batch: _Batch) -> None:
        if batch.blob is not None or batch.host is None:
            return
        # The buffer comes from the main stream's pool (a buffer allocated under the side stream would
        # be handed back to that stream's pool only after cross-stream bookkeeping, and the next
        # iteration would find the pool empty and go to the driver).  Its memory may still be in use
        # by work already enqueued on the main stream, so the copy waits for that point.
        main = torch.cuda.current_stream()
        blob = torch.empty(batch.nbytes, dtype=torch.uint8, device="cuda")
        here = torch.cuda.Event()
        here.record(main)
        with torch.cuda.stream(self._in_stream):
            self._in_stream.wait_event(here)
            self._in_stream.wait_event(batch.out_event)
            blob.copy_(batch.host, non_blocking=True)
            blob.record_stream(self._in_stream)
            batch.in_event = torch.cuda.Event()
            batch.in_event.record()
        batch.blob = blob

    def _ensure_on_device(self, batch: _Batch) -> None:
        if batch.blob is None:
            self._start_swap_in(batch)

    # ------------------------------------------------------------ adaptation
    def compute_sensitivities(self, fwdbwd: Callable[[], Sequence[torch.Tensor]]) -> np.ndarray:
        """Alg. 1 for every context tensor.  ``fwdbwd`` runs one forward and
        backward pass under ``self.hooks()`` on a fixed batch and returns the
        gradient buffers.  L + 1 passes: one with the seeds (r_l), then one per
        tensor with only that tensor's seed replaced by r_{L+1}.  All passes use
        the seeds of one iteration: the iteration counter does not advance here."""
        self.seed_override.clear()
        self.begin_iteration()
        self._frozen = True
        try:
            g0 = [g.detach().clone() for g in fwdbwd()]
            L = len(self.numel)
            c = np.zeros(L, dtype=np.float32)
            other = (self._iter_key + (L + 1_000_000) * 0x9E3779B97F4A7C15) & _MASK64      # r_{L+1}
            for l in range(L):
                if self.bits_of(l) == GACT_BITS_UNCOMPRESSED:
                    continue
                self.seed_override = {l: other}
                self.begin_iteration()
                g1 = fwdbwd()
                c[l] = float(gact_sensitivity(g0, [g.detach() for g in g1], self.bits_of(l)).item())
        finally:
            self._frozen = False
            self.seed_override.clear()
        self.sensitivity = c
        return c

    def adapt(self, avg_bits: float, levels=(1, 2, 4, 8)) -> np.ndarray:
        """Solve Eq. (ilp) for the sensitivities measured last."""
        assert self.sensitivity is not None and len(self.numel) == len(self.sensitivity)
        b = gact_allocate_bits_levels(self.sensitivity, self.numel, avg_bits, levels)
        self.bits = {l: int(v) for l, v in enumerate(b)}
        return b
