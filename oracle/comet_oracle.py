"""ctypes front end of the plain-C CPU oracle (``comet_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports this module, and this module never imports the product package.

Every function here only marshals numpy arrays into the C entry points; the
arithmetic lives in the C file, which cites the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "comet_oracle.c")
_LIB = os.path.join(_HERE, "libcomet_oracle.so")

OK, ERR_INVALID, ERR_CAPACITY, ERR_FORMAT, ERR_NOMEM = 0, -1, -2, -3, -5
HEADER_BYTES = 128


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        u8p, u16p, u32p, i32p, u64p, f32p = (C.POINTER(t) for t in (C.c_uint8, C.c_uint16, C.c_uint32, C.c_int32, C.c_uint64, C.c_float))
        L.oracle_constants.argtypes = [C.c_float, f32p, f32p]
        L.oracle_constants.restype = None
        L.oracle_prequant.argtypes = [f32p, C.c_uint64, C.c_float, i32p, u8p, u64p]
        L.oracle_predict_code.argtypes = [i32p] + [C.c_uint32] * 5 + [u16p, i32p]
        L.oracle_histogram.argtypes = [u16p, C.c_uint64, C.c_uint32, u32p]
        L.oracle_code_lengths.argtypes = [u32p, C.c_uint32, u8p]
        L.oracle_canonical_codes.argtypes = [u8p, C.c_uint32, u64p]
        L.oracle_encode.argtypes = [u16p, C.c_uint64, C.c_uint32, C.c_uint32, u8p, u64p, u32p, C.c_uint64, u32p, C.c_uint64, u64p]
        L.oracle_decode.argtypes = [u8p, C.c_uint32, u32p, u32p, C.c_uint64, C.c_uint64, C.c_uint32, u16p]
        L.oracle_reconstruct.argtypes = [u16p, u32p, C.c_uint64] + [C.c_uint32] * 5 + [C.c_float, f32p]
        L.oracle_compress_bound.argtypes = [C.c_uint32] * 6
        L.oracle_compress_bound.restype = C.c_uint64
        L.oracle_compress.argtypes = [f32p] + [C.c_uint32] * 4 + [C.c_float, C.c_uint32, C.c_uint32, u8p, C.c_uint64, u64p]
        L.oracle_compress_variant.argtypes = [f32p] + [C.c_uint32] * 4 + [C.c_float, C.c_uint32, C.c_uint32, C.c_uint32, u8p, C.c_uint64, u64p]
        L.oracle_prequant_zero_first.argtypes = [f32p, C.c_uint64, C.c_float, i32p, u8p, u64p]
        L.oracle_encode_zero_chunks.argtypes = L.oracle_encode.argtypes
        L.oracle_decode_zero_chunks.argtypes = L.oracle_decode.argtypes
        L.oracle_compress_with_lengths.argtypes = [f32p] + [C.c_uint32] * 4 + [C.c_float, C.c_uint32, C.c_uint32, u8p, u8p, C.c_uint64, u64p]
        L.oracle_decompress.argtypes = [u8p, C.c_uint64, f32p, C.c_uint64, u32p]
        L.oracle_adapt_eb.argtypes = [C.c_double, C.c_double, C.c_double, C.c_uint32, C.c_double, C.c_double, C.c_float, C.c_float, f32p]
        L.oracle_abs_mean.argtypes = [f32p, C.c_uint64, C.POINTER(C.c_double)]
        L.oracle_controller_init.argtypes = [u32p, C.c_uint32]
        L.oracle_controller_tick.argtypes = [u32p, C.POINTER(C.c_int)]
        L.oracle_controller_update.argtypes = [u32p, f32p, f32p, C.c_uint32]
        L.oracle_widen16.argtypes = [u16p, C.c_int, f32p, C.c_uint64]
        L.oracle_narrow16.argtypes = [f32p, C.c_int, u16p, C.c_uint64]
        for name in ("oracle_prequant", "oracle_predict_code", "oracle_histogram", "oracle_code_lengths",
                     "oracle_canonical_codes", "oracle_encode", "oracle_decode", "oracle_reconstruct",
                     "oracle_compress", "oracle_compress_with_lengths", "oracle_decompress", "oracle_adapt_eb",
                     "oracle_abs_mean", "oracle_controller_init", "oracle_controller_tick", "oracle_controller_update"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where} failed with code {code}")
        self.code = code


def _chk(rc: int, where: str) -> None:
    if rc != OK:
        raise OracleError(rc, where)


def _p(a: np.ndarray, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def constants(eb: float):
    e2, r = C.c_float(), C.c_float()
    lib().oracle_constants(C.c_float(eb), C.byref(e2), C.byref(r))
    return np.float32(e2.value), np.float32(r.value)


def prequant(x, eb: float, zero_first: bool = False):
    """zero_first: the alternative of Sec. 3.4 (values within eb of zero are zeroed in this step)."""
    x = _c(x, np.float32).ravel()
    q = np.empty(x.size, np.int32)
    v = np.empty(x.size, np.uint8)
    nnz = C.c_uint64()
    fn = lib().oracle_prequant_zero_first if zero_first else lib().oracle_prequant
    _chk(fn(_p(x, C.c_float), x.size, C.c_float(eb), _p(q, C.c_int32), _p(v, C.c_uint8), C.byref(nnz)), "oracle_prequant")
    return q, v, int(nnz.value)


def predict_code(q, shape, nbins: int):
    q = _c(q, np.int32).ravel()
    n_, c_, h_, w_ = (int(s) for s in shape)
    assert q.size == n_ * c_ * h_ * w_
    codes = np.empty(q.size, np.uint16)
    delta = np.empty(q.size, np.int32)
    _chk(lib().oracle_predict_code(_p(q, C.c_int32), n_, c_, h_, w_, nbins, _p(codes, C.c_uint16), _p(delta, C.c_int32)), "oracle_predict_code")
    return codes, delta


def histogram(codes, nbins: int):
    codes = _c(codes, np.uint16).ravel()
    freq = np.empty(nbins, np.uint32)
    _chk(lib().oracle_histogram(_p(codes, C.c_uint16), codes.size, nbins, _p(freq, C.c_uint32)), "oracle_histogram")
    return freq


def code_lengths(freq):
    freq = _c(freq, np.uint32).ravel()
    ln = np.empty(freq.size, np.uint8)
    _chk(lib().oracle_code_lengths(_p(freq, C.c_uint32), freq.size, _p(ln, C.c_uint8)), "oracle_code_lengths")
    return ln


def canonical_codes(ln):
    ln = _c(ln, np.uint8).ravel()
    code = np.empty(ln.size, np.uint64)
    _chk(lib().oracle_canonical_codes(_p(ln, C.c_uint8), ln.size, _p(code, C.c_uint64)), "oracle_canonical_codes")
    return code


def encode(codes, nbins: int, chunk_syms: int, ln, code, zero_chunks: bool = False):
    """zero_chunks: chunks that hold the centre code only take no words (container version 2)."""
    codes = _c(codes, np.uint16).ravel()
    ln = _c(ln, np.uint8).ravel()
    code = _c(code, np.uint64).ravel()
    n = codes.size
    n_chunks = (n + chunk_syms - 1) // chunk_syms
    chunk_off = np.empty(max(n_chunks, 1), np.uint32)
    total_bits = int(ln[codes].astype(np.uint64).sum()) if n else 0
    cap = total_bits // 32 + n_chunks + 1
    payload = np.zeros(cap, np.uint32)
    words = C.c_uint64()
    fn = lib().oracle_encode_zero_chunks if zero_chunks else lib().oracle_encode
    _chk(fn(_p(codes, C.c_uint16), n, nbins, chunk_syms, _p(ln, C.c_uint8), _p(code, C.c_uint64),
            _p(chunk_off, C.c_uint32), n_chunks, _p(payload, C.c_uint32), cap, C.byref(words)), "oracle_encode")
    return chunk_off[:n_chunks].copy(), payload[: int(words.value)].copy()


def decode(ln, chunk_off, payload, n: int, chunk_syms: int, zero_chunks: bool = False):
    ln = _c(ln, np.uint8).ravel()
    chunk_off = _c(chunk_off, np.uint32).ravel()
    payload = _c(payload, np.uint32).ravel()
    out = np.empty(n, np.uint16)
    pl = payload if payload.size else np.zeros(1, np.uint32)
    co = chunk_off if chunk_off.size else np.zeros(1, np.uint32)
    fn = lib().oracle_decode_zero_chunks if zero_chunks else lib().oracle_decode
    _chk(fn(_p(ln, C.c_uint8), ln.size, _p(co, C.c_uint32), _p(pl, C.c_uint32), payload.size, n, chunk_syms, _p(out, C.c_uint16)), "oracle_decode")
    return out


def reconstruct(codes, records, shape, nbins: int, eb: float):
    """records: uint32 array [n_rec, 2] of (key, payload), ascending key."""
    codes = _c(codes, np.uint16).ravel()
    rec = _c(records, np.uint32).reshape(-1, 2)
    n_, c_, h_, w_ = (int(s) for s in shape)
    out = np.empty(codes.size, np.float32)
    rp = rec if rec.size else np.zeros((1, 2), np.uint32)
    _chk(lib().oracle_reconstruct(_p(codes, C.c_uint16), _p(rp, C.c_uint32), rec.shape[0], n_, c_, h_, w_, nbins, C.c_float(eb), _p(out, C.c_float)), "oracle_reconstruct")
    return out.reshape(n_, c_, h_, w_)


def compress_bound(shape, nbins: int, chunk_syms: int) -> int:
    n_, c_, h_, w_ = (int(s) for s in shape)
    return int(lib().oracle_compress_bound(n_, c_, h_, w_, nbins, chunk_syms))


ZERO_CHUNKS = 1      # container version 2: chunks that hold the centre code only take no words
ZERO_FIRST = 2       # the alternative of Sec. 3.4: values within eb of zero are zeroed in the first quantisation step


def compress(x, eb: float, nbins: int, chunk_syms: int, capacity: int | None = None, flags: int = 0) -> np.ndarray:
    """Full pipeline; returns the container as a uint8 array of its exact size.  flags: ZERO_CHUNKS | ZERO_FIRST."""
    x = _c(x, np.float32)
    assert x.ndim == 4
    n_, c_, h_, w_ = x.shape
    if capacity is None:
        capacity = compress_bound(x.shape, nbins, chunk_syms)
        if capacity == 0:
            raise OracleError(ERR_INVALID, "oracle_compress_bound")
        # the true worst case is rarely needed; start smaller and grow on demand
        capacity = min(capacity, 8 * x.size + 4096 + nbins)
        auto = True
    else:
        auto = False
    while True:
        out = np.empty(capacity, np.uint8)
        used = C.c_uint64()
        if flags:
            rc = lib().oracle_compress_variant(_p(x, C.c_float), n_, c_, h_, w_, C.c_float(eb), nbins, chunk_syms, flags,
                                               _p(out, C.c_uint8), capacity, C.byref(used))
        else:
            rc = lib().oracle_compress(_p(x, C.c_float), n_, c_, h_, w_, C.c_float(eb), nbins, chunk_syms, _p(out, C.c_uint8), capacity, C.byref(used))
        if rc == ERR_CAPACITY and auto and capacity < compress_bound(x.shape, nbins, chunk_syms):
            capacity = compress_bound(x.shape, nbins, chunk_syms)
            continue
        _chk(rc, "oracle_compress")
        return out[: int(used.value)].copy()


def compress_with_lengths(x, eb: float, nbins: int, chunk_syms: int, given_len) -> np.ndarray:
    """Compression that reuses a length table (a code without a code word in it becomes an escape)."""
    x = _c(x, np.float32)
    assert x.ndim == 4
    n_, c_, h_, w_ = x.shape
    given = _c(given_len, np.uint8)
    assert given.size == nbins
    capacity = compress_bound(x.shape, nbins, chunk_syms)
    if capacity == 0:
        raise OracleError(ERR_INVALID, "oracle_compress_bound")
    out = np.empty(capacity, np.uint8)
    used = C.c_uint64()
    rc = lib().oracle_compress_with_lengths(_p(x, C.c_float), n_, c_, h_, w_, C.c_float(eb), nbins, chunk_syms,
                                            _p(given, C.c_uint8), _p(out, C.c_uint8), capacity, C.byref(used))
    _chk(rc, "oracle_compress_with_lengths")
    return out[: int(used.value)].copy()


def decompress(container) -> np.ndarray:
    buf = _c(container, np.uint8).ravel()
    if buf.size < HEADER_BYTES:
        raise OracleError(ERR_FORMAT, "oracle_decompress")
    hdr = buf[:HEADER_BYTES].view("<u4")
    n_elems = int(hdr[3]) * int(hdr[4]) * int(hdr[5]) * int(hdr[6])
    if n_elems <= 0 or n_elems >= 2 ** 31:
        raise OracleError(ERR_FORMAT, "oracle_decompress")
    out = np.empty(n_elems, np.float32)
    shp = (C.c_uint32 * 4)()
    _chk(lib().oracle_decompress(_p(buf, C.c_uint8), buf.size, _p(out, C.c_float), n_elems, shp), "oracle_decompress")
    return out.reshape(tuple(int(s) for s in shp))


F16, BF16 = 1, 2


def widen16(bits, kind: int) -> np.ndarray:
    """fp32 values of 16-bit patterns (uint16 array; kind F16 or BF16)."""
    b = _c(bits, np.uint16)
    out = np.empty(b.shape, np.float32)
    _chk(lib().oracle_widen16(_p(b, C.c_uint16), kind, _p(out, C.c_float), b.size), "oracle_widen16")
    return out


def narrow16(x, kind: int) -> np.ndarray:
    """Nearest (ties to even) 16-bit patterns of fp32 values, as uint16."""
    v = _c(x, np.float32)
    out = np.empty(v.shape, np.uint16)
    _chk(lib().oracle_narrow16(_p(v, C.c_float), kind, _p(out, C.c_uint16), v.size), "oracle_narrow16")
    return out


def compress_16(bits, kind: int, eb: float, nbins: int, chunk_syms: int, capacity: int | None = None) -> np.ndarray:
    """Container of a 16-bit NCHW tensor given as uint16 patterns: the fp32 codec on the widened values."""
    return compress(widen16(bits, kind), eb, nbins, chunk_syms, capacity)


def decompress_16(container, kind: int) -> np.ndarray:
    """The reconstruction rounded to the 16-bit format, as uint16 patterns."""
    return narrow16(decompress(container), kind)


def adapt_eb(momentum_abs_mean, loss_grad_mean, nonzero_ratio, batch, a=0.32, sigma_frac=0.01,
             eb_min=2.0 ** -100, eb_max=2.0 ** 100) -> np.float32:
    out = C.c_float()
    _chk(lib().oracle_adapt_eb(momentum_abs_mean, loss_grad_mean, nonzero_ratio, batch, a, sigma_frac,
                               C.c_float(eb_min), C.c_float(eb_max), C.byref(out)), "oracle_adapt_eb")
    return np.float32(out.value)


def abs_mean(x) -> float:
    x = _c(x, np.float32).ravel()
    out = C.c_double()
    _chk(lib().oracle_abs_mean(_p(x, C.c_float), x.size, C.byref(out)), "oracle_abs_mean")
    return out.value


class Controller:
    """The active factor W (state kept in three uint32, as the C functions see it)."""

    def __init__(self, w_default: int = 0):
        self.state = np.zeros(3, np.uint32)
        _chk(lib().oracle_controller_init(_p(self.state, C.c_uint32), w_default), "oracle_controller_init")

    @property
    def w(self) -> int:
        return int(self.state[1])

    def tick(self) -> bool:
        c = C.c_int()
        _chk(lib().oracle_controller_tick(_p(self.state, C.c_uint32), C.byref(c)), "oracle_controller_tick")
        return bool(c.value)

    def update(self, eb_old, eb_new) -> int:
        a, b = _c(eb_old, np.float32).ravel(), _c(eb_new, np.float32).ravel()
        assert a.size == b.size
        _chk(lib().oracle_controller_update(_p(self.state, C.c_uint32), _p(a, C.c_float), _p(b, C.c_float), a.size), "oracle_controller_update")
        return self.w


# ---------------------------------------------------------------------------
# helpers that only slice a container produced by compress(); no arithmetic
# ---------------------------------------------------------------------------

def parse_container(buf) -> dict:
    """Split a container into its header fields and sections (views)."""
    buf = _c(buf, np.uint8).ravel()
    h32 = buf[:HEADER_BYTES].view("<u4")
    h64 = buf[:HEADER_BYTES].view("<u8")
    d = dict(magic=int(h32[0]), version=int(h32[1]), status=int(h32[2]),
             shape=tuple(int(v) for v in h32[3:7]), nbins=int(h32[7]), chunk_syms=int(h32[8]),
             n_chunks=int(h32[9]), eb_bits=int(h32[10]), ebx2_bits=int(h32[11]), r_bits=int(h32[12]),
             n_active=int(h32[13]), max_len=int(h32[14]), n_records=int(h32[15]),
             nnz=int(h64[8]), payload_words=int(h64[9]), total_bytes=int(h64[10]),
             off_len=int(h64[11]), off_chunk=int(h64[12]), off_outlier=int(h64[13]), off_payload=int(h64[14]),
             n_value_records=int(h32[30]))
    d["len"] = buf[d["off_len"]: d["off_len"] + d["nbins"]]
    d["chunk_off"] = buf[d["off_chunk"]: d["off_chunk"] + 4 * d["n_chunks"]].view("<u4")
    d["records"] = buf[d["off_outlier"]: d["off_outlier"] + 8 * d["n_records"]].view("<u4").reshape(-1, 2)
    d["payload"] = buf[d["off_payload"]: d["off_payload"] + 4 * d["payload_words"]].view("<u4")
    return d
