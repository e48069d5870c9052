"""Saved-tensor hook that keeps convolution inputs as COMET containers between the forward and the
backward pass (COMET Sec. 3.4: an activation is compressed right after its layer's forward pass and
decompressed when the backward pass needs it).

Glue only: every compression and decompression is a call into libcomet.  PyTorch supplies the hook
(``torch.autograd.graph.saved_tensors_hooks``), the device buffers and the stream.
"""
from __future__ import annotations

import weakref

import torch

from . import comet


class _Packed:
    """What autograd holds instead of a saved activation."""
    __slots__ = ("buf", "used", "shape", "dtype", "raw", "hdr", "event")

    def __init__(self, shape, dtype):
        self.buf, self.used, self.shape, self.dtype = None, 0, shape, dtype
        self.raw = self.hdr = self.event = None


class saved_activations:
    """Context manager.  Inside it, every tensor autograd saves for backward that is a contiguous 4-D
    fp32, fp16 or bf16 CUDA tensor of at least ``min_elems`` elements (16-bit ones: at most 512 columns)
    and no parameter is held as a container.

    ctx        a ``comet.Context`` whose ``max_elems`` covers the largest such tensor
    eb         absolute error bound, or a callable ``tensor -> float`` (e.g. the adaptive rule)
    exact_size True: the call waits for the compression and keeps a copy of exactly the container's
               size (frees the rest; one synchronisation per tensor); False: keeps the
               ``capacity_frac`` buffer and never waits: the tensor is held until the container's header has
               reached the host (polled at the next hook call), then dropped, or kept instead of the container
               if that did not fit the buffer
    """

    def __init__(self, ctx: comet.Context, eb, nbins: int = 1024, min_elems: int = 1 << 16,
                 capacity_frac: float = 0.6, exact_size: bool = True):
        self.ctx, self.eb, self.nbins = ctx, eb, nbins
        self.min_elems, self.capacity_frac, self.exact_size = min_elems, capacity_frac, exact_size
        self.packed = 0                 # tensors compressed
        self.unpacked = 0               # tensors decompressed
        self.bytes_in = 0               # bytes of the tensors compressed
        self.bytes_kept = 0             # bytes held for them instead
        self.kept_raw = 0               # tensors that did not fit capacity_frac and were kept as they are
        self._pending = []              # asynchronous compressions whose outcome is not known yet
        self._seen = {}                 # id(tensor) -> (weak reference, version, packed): a tensor object saved twice is compressed once
        self._hooks = torch.autograd.graph.saved_tensors_hooks(self._pack, self._unpack)

    def __enter__(self):
        self._hooks.__enter__()
        return self

    def __exit__(self, *exc):
        self._seen.clear()
        return self._hooks.__exit__(*exc)

    def _eligible(self, t: torch.Tensor) -> bool:
        if not (t.is_cuda and t.dim() == 4 and t.numel() >= self.min_elems and t.is_contiguous()
                and not isinstance(t, torch.nn.Parameter)):
            return False
        return t.dtype == torch.float32 or (t.dtype in (torch.float16, torch.bfloat16) and t.shape[3] <= 512)

    def _pack(self, t: torch.Tensor):
        self._poll()
        if not self._eligible(t):
            return t
        key = id(t)
        hit = self._seen.get(key)
        if hit is not None and hit[0]() is t and hit[1] == t._version:      # the same live object, unchanged since
            return hit[2]
        eb = float(self.eb(t)) if callable(self.eb) else float(self.eb)
        cap = max(4096, int(t.numel() * t.element_size() * self.capacity_frac) // 16 * 16)
        buf = torch.empty(cap, dtype=torch.uint8, device=t.device)
        x = t.detach()
        compress = self.ctx.comet_compress if t.dtype == torch.float32 else self.ctx.comet_compress_16
        packed = _Packed(tuple(t.shape), t.dtype)
        if self.exact_size:
            try:
                used = compress(x, eb, self.nbins, buf, stream=torch.cuda.current_stream())
            except comet.CometError as e:
                if e.code != comet.ERR_CAPACITY:
                    raise
                self.kept_raw += 1      # the unexpectedly low ratio of Sec. 3.4: not worth compressing
                return t
            packed.buf, packed.used = buf[:used].clone(), used
        else:
            # Asynchronous: whether the container fitted is only known on the device.  The header (its status
            # word) follows the compression to pinned host memory on the same stream, and the tensor itself is
            # kept until that copy has landed: dropped if the container is complete, returned as it is if not.
            compress(x, eb, self.nbins, buf, stream=torch.cuda.current_stream(), sync=False)
            packed.buf, packed.used = buf, cap
            packed.raw = x
            packed.hdr = torch.empty(comet.HEADER_BYTES, dtype=torch.uint8, pin_memory=True)
            packed.hdr.copy_(buf[:comet.HEADER_BYTES], non_blocking=True)
            packed.event = torch.cuda.Event()
            packed.event.record(torch.cuda.current_stream())
            self._pending.append(packed)
        self.packed += 1
        self.bytes_in += t.numel() * t.element_size()
        self.bytes_kept += packed.buf.numel()
        self._seen[key] = (weakref.ref(t), t._version, packed)
        return packed

    def _resolve(self, p: "_Packed", wait: bool) -> bool:
        """Settle an asynchronous compression once its header has reached the host."""
        if p.event is None:
            return True
        if wait:
            p.event.synchronize()
        elif not p.event.query():
            return False
        status = int(p.hdr[8:12].view(torch.int32)[0])
        complete = status == 0 and bytes(p.hdr[:4].tolist()) == b"CMT1"
        p.event = p.hdr = None
        if complete:
            p.raw = None                # the container stands in for the tensor from here on
        else:
            p.buf = None                # the low-ratio case of Sec. 3.4: the tensor is kept as it is
            self.kept_raw += 1
            self.packed -= 1
            try:                        # take the error the library has latched for this call off the context
                self.ctx.comet_sync(torch.cuda.current_stream())
            except comet.CometError as e:
                if e.code != comet.ERR_CAPACITY:
                    raise
        return True

    def _poll(self) -> None:
        self._pending = [p for p in self._pending if not self._resolve(p, wait=False)]

    def _unpack(self, packed):
        if not isinstance(packed, _Packed):
            return packed
        self._resolve(packed, wait=True)
        self._pending = [p for p in self._pending if p is not packed]
        if packed.raw is not None:
            return packed.raw
        out = torch.empty(packed.shape, dtype=packed.dtype, device=packed.buf.device)
        decompress = self.ctx.comet_decompress if packed.dtype == torch.float32 else self.ctx.comet_decompress_16
        decompress(packed.buf, packed.used, packed.shape, out, stream=torch.cuda.current_stream())
        self.unpacked += 1
        return out
