"""Thin ctypes binding of libcomet (include/comet.h): same entry-point names,
argument marshalling only.  Every step of the codec runs in the HIP kernels of
``libcomet.so``; PyTorch supplies device tensors and streams, nothing else.

The library must have been built (``python -m paper_2111_09562_amd.build``);
there is no fallback: a missing library raises at first use.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcomet.so")

OK, ERR_INVALID, ERR_CAPACITY, ERR_FORMAT, ERR_HIP, ERR_NOMEM, ERR_INTERNAL, ERR_CODEBOOK = 0, -1, -2, -3, -4, -5, -6, -7
HEADER_BYTES = 128
DEFAULT_CHUNK_SYMS = 64

EXPORTS = (
    "comet_create", "comet_destroy", "comet_set_chunk_syms", "comet_set_zero_chunks", "comet_compress_bound", "comet_compress", "comet_compress_with_codebook",
    "comet_decompress", "comet_decompress_static", "comet_compress_16", "comet_decompress_16", "comet_sync", "comet_peek", "comet_adapt_defaults", "comet_adapt_eb", "comet_abs_mean",
    "comet_controller_init", "comet_controller_tick", "comet_controller_update",
    "comet_stage_quantize", "comet_stage_codebook", "comet_stage_encode", "comet_stage_decode",
    "comet_stage_reconstruct", "comet_profile_enable", "comet_profile_reset", "comet_profile_read", "comet_strerror",
)
KERNEL_NAMES = ("k_quantize_rows", "k_codebook", "k_encode_pack", "k_decode_tables", "k_scan_store", "k_decode_chunks",
                "k_gather_records", "k_encode_count", "k_decode_scan")


class Shape(C.Structure):
    _fields_ = [("n", C.c_uint32), ("c", C.c_uint32), ("h", C.c_uint32), ("w", C.c_uint32)]


class Info(C.Structure):
    _fields_ = [("shape", Shape), ("nbins", C.c_uint32), ("chunk_syms", C.c_uint32), ("n_chunks", C.c_uint32),
                ("n_active", C.c_uint32), ("max_len", C.c_uint32), ("n_outlier_records", C.c_uint32),
                ("n_value_records", C.c_uint32), ("eb", C.c_float), ("nnz", C.c_uint64),
                ("payload_words", C.c_uint64), ("total_bytes", C.c_uint64)]


class LayerStats(C.Structure):
    _fields_ = [("momentum_abs_mean", C.c_double), ("loss_grad_mean", C.c_double), ("nonzero_ratio", C.c_double),
                ("batch", C.c_uint32)]


class AdaptCfg(C.Structure):
    _fields_ = [("a", C.c_double), ("sigma_frac", C.c_double), ("eb_min", C.c_float), ("eb_max", C.c_float)]


class CometError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {strerror(code)} ({code})")
        self.code = code


_lib = None


def lib():
    """Load libcomet.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2111_09562_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, u64 = C.c_void_p, C.c_uint64
        L.comet_create.argtypes = [C.POINTER(vp), u64, C.c_uint32]
        L.comet_destroy.argtypes = [vp]
        L.comet_destroy.restype = None
        L.comet_set_chunk_syms.argtypes = [vp, C.c_uint32]
        L.comet_set_zero_chunks.argtypes = [vp, C.c_int]
        L.comet_compress_bound.argtypes = [Shape, C.c_uint32, C.c_uint32]
        L.comet_compress_bound.restype = u64
        L.comet_compress.argtypes = [vp, vp, Shape, C.c_float, C.c_uint32, vp, vp, u64, C.POINTER(u64)]
        L.comet_compress_with_codebook.argtypes = [vp, vp, Shape, C.c_float, C.c_uint32, vp, vp, vp, u64, C.POINTER(u64)]
        L.comet_decompress.argtypes = [vp, vp, u64, Shape, vp, vp]
        L.comet_decompress_static.argtypes = [vp, u64, Shape, vp, vp, vp]
        L.comet_compress_16.argtypes = [vp, vp, C.c_int, Shape, C.c_float, C.c_uint32, vp, vp, u64, C.POINTER(u64)]
        L.comet_decompress_16.argtypes = [vp, vp, u64, Shape, C.c_int, vp, vp]
        L.comet_sync.argtypes = [vp, vp]
        L.comet_abs_mean.argtypes = [vp, vp, u64, vp, C.POINTER(C.c_double)]
        L.comet_controller_init.argtypes = [vp, C.c_uint32]
        L.comet_controller_tick.argtypes = [vp, C.POINTER(C.c_int)]
        L.comet_controller_update.argtypes = [vp, vp, vp, C.c_uint32]
        L.comet_peek.argtypes = [vp, vp, u64, vp, C.POINTER(Info)]
        L.comet_adapt_defaults.argtypes = [C.POINTER(AdaptCfg)]
        L.comet_adapt_defaults.restype = None
        L.comet_adapt_eb.argtypes = [C.POINTER(LayerStats), C.POINTER(AdaptCfg), C.POINTER(C.c_float)]
        L.comet_stage_quantize.argtypes = [vp, vp, Shape, C.c_float, C.c_uint32, vp, vp, vp, vp, u64, vp]
        L.comet_stage_codebook.argtypes = [vp, vp, C.c_uint32, vp, vp, vp]
        L.comet_stage_encode.argtypes = [vp, vp, u64, C.c_uint32, C.c_uint32, vp, vp, vp, u64, vp]
        L.comet_stage_decode.argtypes = [vp, vp, C.c_uint32, vp, vp, u64, u64, C.c_uint32, vp, vp]
        L.comet_stage_reconstruct.argtypes = [vp, vp, vp, u64, Shape, C.c_uint32, C.c_float, vp, vp]
        L.comet_profile_enable.argtypes = [vp, C.c_int]
        L.comet_profile_reset.argtypes = [vp]
        L.comet_profile_read.argtypes = [vp, C.c_uint32, C.POINTER(C.c_uint32), C.POINTER(C.c_double)]
        L.comet_strerror.argtypes = [C.c_int]
        L.comet_strerror.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("comet_destroy", "comet_compress_bound", "comet_adapt_defaults", "comet_strerror"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().comet_strerror(code).decode()


def _chk(rc: int, where: str) -> None:
    if rc != OK:
        raise CometError(rc, where)


F16, BF16 = 1, 2


def _dtype16(t) -> int:
    name = str(t.dtype)
    if name == "torch.float16":
        return F16
    if name == "torch.bfloat16":
        return BF16
    raise TypeError(f"float16 or bfloat16 tensor expected, got {name}")


def _ptr(t):
    """Device pointer of a torch tensor (or None)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _shape(shape) -> Shape:
    n, c, h, w = (int(v) for v in shape)
    return Shape(n, c, h, w)


def comet_compress_bound(shape, nbins: int, chunk_syms: int = DEFAULT_CHUNK_SYMS) -> int:
    return int(lib().comet_compress_bound(_shape(shape), nbins, chunk_syms))


def comet_adapt_eb(momentum_abs_mean: float, loss_grad_mean: float, nonzero_ratio: float, batch: int,
                   a: float | None = None, sigma_frac: float | None = None,
                   eb_min: float | None = None, eb_max: float | None = None) -> float:
    st = LayerStats(momentum_abs_mean, loss_grad_mean, nonzero_ratio, batch)
    cfg = AdaptCfg()
    lib().comet_adapt_defaults(C.byref(cfg))
    if a is not None:
        cfg.a = a
    if sigma_frac is not None:
        cfg.sigma_frac = sigma_frac
    if eb_min is not None:
        cfg.eb_min = eb_min
    if eb_max is not None:
        cfg.eb_max = eb_max
    out = C.c_float()
    _chk(lib().comet_adapt_eb(C.byref(st), C.byref(cfg), C.byref(out)), "comet_adapt_eb")
    return out.value


STATIC_MAX_ELEMS = 4 << 20


def comet_decompress_static(container, nbytes: int, shape, out, status=None, stream=None) -> None:
    """comet_decompress without a context (the library's static scratch array; allocates nothing).
    status: optional int32 device tensor of one element that receives 0 or ERR_FORMAT."""
    _chk(lib().comet_decompress_static(_ptr(container), int(nbytes), _shape(shape), _stream(stream), _ptr(out), _ptr(status)),
         "comet_decompress_static")


class ControllerState(C.Structure):
    _fields_ = [("w_default", C.c_uint32), ("w", C.c_uint32), ("since", C.c_uint32)]


class Controller:
    """The active factor W of the controller (host-side counter)."""

    def __init__(self, w_default: int = 0):
        self._s = ControllerState()
        _chk(lib().comet_controller_init(C.byref(self._s), int(w_default)), "comet_controller_init")

    @property
    def w(self) -> int:
        return int(self._s.w)

    def comet_controller_tick(self) -> bool:
        c = C.c_int()
        _chk(lib().comet_controller_tick(C.byref(self._s), C.byref(c)), "comet_controller_tick")
        return bool(c.value)

    def comet_controller_update(self, eb_old, eb_new) -> int:
        n = len(eb_old)
        assert n == len(eb_new)
        a = (C.c_float * n)(*[float(v) for v in eb_old])
        b = (C.c_float * n)(*[float(v) for v in eb_new])
        _chk(lib().comet_controller_update(C.byref(self._s), a, b, n), "comet_controller_update")
        return self.w


class Context:
    """Owns one comet_ctx (device workspace).  One per stream."""

    def __init__(self, max_elems: int, max_nbins: int = 65536):
        self._h = C.c_void_p()
        _chk(lib().comet_create(C.byref(self._h), int(max_elems), int(max_nbins)), "comet_create")

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            lib().comet_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def comet_set_zero_chunks(self, enable: bool) -> None:
        """Containers of version 2: chunks that hold the centre code only take no payload words."""
        _chk(lib().comet_set_zero_chunks(self._h, 1 if enable else 0), "comet_set_zero_chunks")

    def comet_set_chunk_syms(self, chunk_syms: int) -> None:
        _chk(lib().comet_set_chunk_syms(self._h, chunk_syms), "comet_set_chunk_syms")

    def comet_compress(self, x, eb: float, nbins: int, out, stream=None, sync: bool = True):
        """x: fp32 NCHW device tensor; out: uint8 device tensor (the container buffer).
        Returns the container size in bytes when sync, else None."""
        assert x.dim() == 4 and str(x.dtype) == "torch.float32"
        used = C.c_uint64()
        rc = lib().comet_compress(self._h, _ptr(x), _shape(x.shape), C.c_float(eb), nbins, _stream(stream), _ptr(out),
                                  out.numel() * out.element_size(), C.byref(used) if sync else None)
        _chk(rc, "comet_compress")
        return int(used.value) if sync else None

    def comet_compress_with_codebook(self, x, eb: float, nbins: int, dev_len, out, stream=None, sync: bool = True):
        """As comet_compress, with the code lengths of an earlier compression: dev_len is a uint8 device tensor of
        nbins entries (e.g. ``earlier_container[HEADER_BYTES:HEADER_BYTES + nbins]``)."""
        assert x.dim() == 4 and str(x.dtype) == "torch.float32"
        assert str(dev_len.dtype) == "torch.uint8" and dev_len.numel() == nbins and dev_len.is_contiguous()
        used = C.c_uint64()
        rc = lib().comet_compress_with_codebook(self._h, _ptr(x), _shape(x.shape), C.c_float(eb), nbins, _ptr(dev_len),
                                                _stream(stream), _ptr(out), out.numel() * out.element_size(),
                                                C.byref(used) if sync else None)
        _chk(rc, "comet_compress_with_codebook")
        return int(used.value) if sync else None

    def comet_decompress(self, container, nbytes: int, shape, out, stream=None) -> None:
        _chk(lib().comet_decompress(self._h, _ptr(container), int(nbytes), _shape(shape), _stream(stream), _ptr(out)),
             "comet_decompress")

    def comet_compress_16(self, x, eb: float, nbins: int, out, stream=None, sync: bool = True):
        """As comet_compress for a float16 or bfloat16 NCHW device tensor."""
        assert x.dim() == 4
        used = C.c_uint64()
        rc = lib().comet_compress_16(self._h, _ptr(x), _dtype16(x), _shape(x.shape), C.c_float(eb), nbins, _stream(stream),
                                     _ptr(out), out.numel() * out.element_size(), C.byref(used) if sync else None)
        _chk(rc, "comet_compress_16")
        return int(used.value) if sync else None

    def comet_decompress_16(self, container, nbytes: int, shape, out, stream=None) -> None:
        """As comet_decompress into a float16 or bfloat16 device tensor."""
        _chk(lib().comet_decompress_16(self._h, _ptr(container), int(nbytes), _shape(shape), _dtype16(out), _stream(stream),
                                       _ptr(out)), "comet_decompress_16")

    def comet_abs_mean(self, x, stream=None) -> float:
        """Mean of |x| over a contiguous fp32 device tensor (synchronises the stream)."""
        assert str(x.dtype) == "torch.float32" and x.is_contiguous()
        out = C.c_double()
        _chk(lib().comet_abs_mean(self._h, _ptr(x), x.numel(), _stream(stream), C.byref(out)), "comet_abs_mean")
        return out.value

    def comet_sync(self, stream=None) -> None:
        _chk(lib().comet_sync(self._h, _stream(stream)), "comet_sync")

    def comet_peek(self, container, nbytes: int, stream=None) -> Info:
        info = Info()
        _chk(lib().comet_peek(self._h, _ptr(container), int(nbytes), _stream(stream), C.byref(info)), "comet_peek")
        return info

    def comet_profile_enable(self, enable: bool) -> None:
        _chk(lib().comet_profile_enable(self._h, 1 if enable else 0), "comet_profile_enable")

    def comet_profile_reset(self) -> None:
        _chk(lib().comet_profile_reset(self._h), "comet_profile_reset")

    def comet_profile_read(self, kernel_id: int):
        """(launches, total milliseconds) of one kernel since the last reset."""
        n, ms = C.c_uint32(), C.c_double()
        _chk(lib().comet_profile_read(self._h, kernel_id, C.byref(n), C.byref(ms)), "comet_profile_read")
        return int(n.value), float(ms.value)

    # ---- stage-level entry points -------------------------------------------------
    def comet_stage_quantize(self, x, eb: float, nbins: int, codes, hist, records, counts, stream=None) -> None:
        cap = 0 if records is None else records.numel() // 2
        _chk(lib().comet_stage_quantize(self._h, _ptr(x), _shape(x.shape), C.c_float(eb), nbins, _stream(stream), _ptr(codes),
                                        _ptr(hist), _ptr(records), cap, _ptr(counts)), "comet_stage_quantize")

    def comet_stage_codebook(self, hist, nbins: int, lens, codes=None, stream=None) -> None:
        _chk(lib().comet_stage_codebook(self._h, _ptr(hist), nbins, _stream(stream), _ptr(lens), _ptr(codes)),
             "comet_stage_codebook")

    def comet_stage_encode(self, codes, n: int, nbins: int, chunk_syms: int, chunk_off, payload, payload_words, stream=None) -> None:
        _chk(lib().comet_stage_encode(self._h, _ptr(codes), n, nbins, chunk_syms, _stream(stream), _ptr(chunk_off), _ptr(payload),
                                      payload.numel(), _ptr(payload_words)), "comet_stage_encode")

    def comet_stage_decode(self, lens, nbins: int, chunk_off, payload, payload_words: int, n: int, chunk_syms: int, codes_out,
                           stream=None) -> None:
        _chk(lib().comet_stage_decode(self._h, _ptr(lens), nbins, _ptr(chunk_off), _ptr(payload), payload_words, n, chunk_syms,
                                      _stream(stream), _ptr(codes_out)), "comet_stage_decode")

    def comet_stage_reconstruct(self, codes, records, n_records: int, shape, nbins: int, eb: float, out, stream=None) -> None:
        _chk(lib().comet_stage_reconstruct(self._h, _ptr(codes), _ptr(records), n_records, _shape(shape), nbins, C.c_float(eb),
                                           _stream(stream), _ptr(out)), "comet_stage_reconstruct")
