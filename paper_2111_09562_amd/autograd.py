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


class saved_activations:
    """Context manager.  Inside it, every tensor autograd saves for backward that is a contiguous 4-D
    fp32, fp16 or bf16 CUDA tensor of at least ``min_elems`` elements (16-bit ones: at most 512 columns)
    and no parameter is held as a container.

    ctx        a ``comet.Context`` whose ``max_elems`` covers the largest such tensor
    eb         absolute error bound, or a callable ``tensor -> float`` (e.g. the adaptive rule)
    exact_size True: the call waits for the compression and keeps a copy of exactly the container's
               size (frees the rest; one synchronisation per tensor); False: keeps the
               ``capacity_frac`` buffer, fully asynchronous
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
        if self.exact_size:
            try:
                used = compress(x, eb, self.nbins, buf, stream=torch.cuda.current_stream())
            except comet.CometError as e:
                if e.code != comet.ERR_CAPACITY:
                    raise
                self.kept_raw += 1      # the unexpectedly low ratio of Sec. 3.4: not worth compressing
                return t
            buf = buf[:used].clone()
        else:
            compress(x, eb, self.nbins, buf, stream=torch.cuda.current_stream(), sync=False)
            used = cap
        self.packed += 1
        self.bytes_in += t.numel() * t.element_size()
        self.bytes_kept += buf.numel()
        packed = ("comet", buf, used, tuple(t.shape), t.dtype)
        self._seen[key] = (weakref.ref(t), t._version, packed)
        return packed

    def _unpack(self, packed):
        if not (isinstance(packed, tuple) and len(packed) == 5 and packed[0] == "comet"):
            return packed
        _, buf, used, shape, dtype = packed
        out = torch.empty(shape, dtype=dtype, device=buf.device)
        decompress = self.ctx.comet_decompress if dtype == torch.float32 else self.ctx.comet_decompress_16
        decompress(buf, used, shape, out, stream=torch.cuda.current_stream())
        self.unpacked += 1
        return out
