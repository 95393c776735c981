"""Python face of the CPU oracle (oracle/entro_oracle.c) -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It imports nothing from the GPU library.  Every function is a
thin ctypes call into the plain C routines; see the C file for the passages of
the paper each routine follows and for the stream format.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .build import build as _build, LIB as _LIB

OK = 0
ERR_ARG, ERR_NONFINITE, ERR_RANGE, ERR_SYMBOL, ERR_TOO_LONG, ERR_CAPACITY, ERR_CORRUPT = range(1, 8)
UNSIGNED, ASYMMETRIC = 0, 1
MAX_LEN = 32

_lib = None


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(
                os.path.join(os.path.dirname(_LIB), "entro_oracle.c")):
            _build()
        L = C.CDLL(_LIB)
        u8p, u16p, u32p, u64p = (C.POINTER(t) for t in (C.c_uint8, C.c_uint16, C.c_uint32, C.c_uint64))
        f32p, f64p = C.POINTER(C.c_float), C.POINTER(C.c_double)
        L.oracle_quantize.argtypes = [f32p, C.c_uint64, C.c_int, C.c_int, u8p, f32p, C.POINTER(C.c_int32)]
        L.oracle_histogram.argtypes = [u8p, C.c_uint64, C.c_int, u64p]
        L.oracle_huffman_lengths.argtypes = [u64p, C.c_int, u8p]
        L.oracle_canonical_codes.argtypes = [u8p, C.c_int, u32p]
        L.oracle_stream_bytes.argtypes = [C.c_uint64]
        L.oracle_stream_bytes.restype = C.c_uint64
        L.oracle_encode.argtypes = [u8p, C.c_uint64, u8p, u32p, C.c_int, C.c_uint32, u8p, C.c_uint64, u64p, u64p]
        L.oracle_decode_chunks.argtypes = [u8p, C.c_uint64, u64p, C.c_uint64, C.c_uint32, u8p, u32p, C.c_int,
                                           C.c_uint64, C.c_uint64, u8p]
        L.oracle_decode.argtypes = [u8p, C.c_uint64, u64p, C.c_uint64, C.c_uint32, u8p, u32p, C.c_int, u8p]
        L.oracle_sub_index.argtypes = [u8p, C.c_uint64, u8p, C.c_int, C.c_uint32, C.c_uint32, u16p]
        L.oracle_decode_subs.argtypes = [u8p, C.c_uint64, u64p, u16p, C.c_uint64, C.c_uint32, C.c_uint32, u8p, u32p, C.c_int,
                                         C.c_uint64, C.c_uint64, u8p]
        L.oracle_pack_u4.argtypes = [u8p, C.c_uint64, u8p]
        L.oracle_pack_u4.restype = None
        L.oracle_dequant_f32.argtypes = [u8p, C.c_uint64, C.c_float, C.c_int32, f32p]
        L.oracle_dequant_f32.restype = None
        L.oracle_dequant_bf16.argtypes = [u8p, C.c_uint64, C.c_float, C.c_int32, u16p]
        L.oracle_dequant_bf16.restype = None
        L.oracle_gemv.argtypes = [u8p, C.c_uint64, C.c_uint64, C.c_float, C.c_int32, u16p, f64p, f32p]
        L.oracle_gemv.restype = None
        L.oracle_bruteforce_min_cost.argtypes = [u64p, C.c_int]
        L.oracle_bruteforce_min_cost.restype = C.c_uint64
        L.oracle_limited_lengths.argtypes = [u64p, C.c_int, C.c_int, u8p, u64p]
        L.oracle_bruteforce_min_cost_limited.argtypes = [u64p, C.c_int, C.c_int]
        L.oracle_bruteforce_min_cost_limited.restype = C.c_uint64
        _lib = L
    return _lib


def _p(a: np.ndarray, t):
    return a.ctypes.data_as(C.POINTER(t))


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _check(rc: int, what: str):
    if rc != OK:
        raise OracleError(rc, what)


def quantize(w, bits: int, scheme: int):
    """-> (q uint8[n], s float32, z int)."""
    w = _c(w, np.float32).ravel()
    q = np.empty(w.size, np.uint8)
    s, z = C.c_float(0), C.c_int32(0)
    _check(lib().oracle_quantize(_p(w, C.c_float), w.size, bits, scheme, _p(q, C.c_uint8),
                                 C.byref(s), C.byref(z)), "quantize")
    return q, np.float32(s.value), int(z.value)


def histogram(q, bits: int) -> np.ndarray:
    q = _c(q, np.uint8).ravel()
    cnt = np.zeros(1 << bits, np.uint64)
    _check(lib().oracle_histogram(_p(q, C.c_uint8), q.size, bits, _p(cnt, C.c_uint64)), "histogram")
    return cnt


def huffman_lengths(cnt) -> np.ndarray:
    cnt = _c(cnt, np.uint64)
    ln = np.zeros(cnt.size, np.uint8)
    _check(lib().oracle_huffman_lengths(_p(cnt, C.c_uint64), cnt.size, _p(ln, C.c_uint8)), "huffman_lengths")
    return ln


def canonical_codes(ln) -> np.ndarray:
    ln = _c(ln, np.uint8)
    code = np.zeros(ln.size, np.uint32)
    _check(lib().oracle_canonical_codes(_p(ln, C.c_uint8), ln.size, _p(code, C.c_uint32)), "canonical_codes")
    return code


def stream_bytes(total_bits: int) -> int:
    return int(lib().oracle_stream_bytes(total_bits))


def encode(q, ln, code, chunk_symbols: int):
    """-> (stream uint8[stream_bytes], offsets uint64[n_chunks + 1])."""
    q = _c(q, np.uint8).ravel()
    ln = _c(ln, np.uint8)
    code = _c(code, np.uint32)
    n = q.size
    n_chunks = (n + chunk_symbols - 1) // chunk_symbols
    cap = stream_bytes(int(n) * MAX_LEN)
    total = int(np.sum(ln.astype(np.uint64)[q], dtype=np.uint64)) if n else 0
    cap = min(cap, stream_bytes(total))
    stream = np.zeros(cap, np.uint8)
    offsets = np.zeros(n_chunks + 1, np.uint64)
    nbytes = C.c_uint64(0)
    _check(lib().oracle_encode(_p(q, C.c_uint8), n, _p(ln, C.c_uint8), _p(code, C.c_uint32), ln.size,
                               chunk_symbols, _p(stream, C.c_uint8), stream.size, C.byref(nbytes),
                               _p(offsets, C.c_uint64)), "encode")
    return stream[: nbytes.value], offsets


def decode(stream, offsets, n: int, chunk_symbols: int, ln, code) -> np.ndarray:
    stream = _c(stream, np.uint8)
    offsets = _c(offsets, np.uint64)
    ln = _c(ln, np.uint8)
    code = _c(code, np.uint32)
    out = np.zeros(n, np.uint8)
    _check(lib().oracle_decode(_p(stream, C.c_uint8), stream.size, _p(offsets, C.c_uint64), n, chunk_symbols,
                               _p(ln, C.c_uint8), _p(code, C.c_uint32), ln.size, _p(out, C.c_uint8)), "decode")
    return out


def decode_chunks(stream, offsets, n: int, chunk_symbols: int, ln, code, first_chunk: int,
                  num_chunks: int, out: np.ndarray | None = None) -> np.ndarray:
    """Decode only segments [first_chunk, first_chunk+num_chunks); returns the
    full-length array `out` with those symbol positions filled."""
    stream = _c(stream, np.uint8)
    offsets = _c(offsets, np.uint64)
    ln = _c(ln, np.uint8)
    code = _c(code, np.uint32)
    if out is None:
        out = np.zeros(n, np.uint8)
    _check(lib().oracle_decode_chunks(_p(stream, C.c_uint8), stream.size, _p(offsets, C.c_uint64), n,
                                      chunk_symbols, _p(ln, C.c_uint8), _p(code, C.c_uint32), ln.size,
                                      first_chunk, num_chunks, _p(out, C.c_uint8)), "decode_chunks")
    return out


def sub_index(q, ln, chunk_symbols: int, sub_symbols: int) -> np.ndarray:
    """-> uint16[ceil(n / sub_symbols)]: stream bits of every piece of sub_symbols symbols."""
    q = _c(q, np.uint8).ravel()
    ln = _c(ln, np.uint8)
    out = np.zeros((q.size + sub_symbols - 1) // sub_symbols, np.uint16)
    _check(lib().oracle_sub_index(_p(q, C.c_uint8), q.size, _p(ln, C.c_uint8), ln.size, chunk_symbols, sub_symbols,
                                  _p(out, C.c_uint16)), "sub_index")
    return out


def decode_subs(stream, offsets, sub_bits, n: int, chunk_symbols: int, sub_symbols: int, ln, code, first_sub: int,
                num_subs: int, out: np.ndarray | None = None) -> np.ndarray:
    """Decode only pieces [first_sub, first_sub + num_subs), each from its own entry point."""
    stream = _c(stream, np.uint8)
    offsets = _c(offsets, np.uint64)
    sub_bits = _c(sub_bits, np.uint16)
    ln = _c(ln, np.uint8)
    code = _c(code, np.uint32)
    if out is None:
        out = np.zeros(n, np.uint8)
    _check(lib().oracle_decode_subs(_p(stream, C.c_uint8), stream.size, _p(offsets, C.c_uint64), _p(sub_bits, C.c_uint16), n,
                                    chunk_symbols, sub_symbols, _p(ln, C.c_uint8), _p(code, C.c_uint32), ln.size,
                                    first_sub, num_subs, _p(out, C.c_uint8)), "decode_subs")
    return out


def pack_u4(q) -> np.ndarray:
    q = _c(q, np.uint8).ravel()
    out = np.zeros((q.size + 1) // 2, np.uint8)
    lib().oracle_pack_u4(_p(q, C.c_uint8), q.size, _p(out, C.c_uint8))
    return out


def dequant_f32(q, s, z: int) -> np.ndarray:
    q = _c(q, np.uint8).ravel()
    out = np.empty(q.size, np.float32)
    lib().oracle_dequant_f32(_p(q, C.c_uint8), q.size, float(s), int(z), _p(out, C.c_float))
    return out


def dequant_bf16(q, s, z: int) -> np.ndarray:
    """-> uint16 bfloat16 bit patterns."""
    q = _c(q, np.uint8).ravel()
    out = np.empty(q.size, np.uint16)
    lib().oracle_dequant_bf16(_p(q, C.c_uint8), q.size, float(s), int(z), _p(out, C.c_uint16))
    return out


def gemv(q, rows: int, cols: int, s, z: int, x_bf16):
    """-> (y fp64-accumulated, y fp32 sequentially accumulated)."""
    q = _c(q, np.uint8).ravel()
    x = _c(x_bf16, np.uint16)
    assert q.size == rows * cols and x.size == cols
    y64 = np.empty(rows, np.float64)
    y32 = np.empty(rows, np.float32)
    lib().oracle_gemv(_p(q, C.c_uint8), rows, cols, float(s), int(z), _p(x, C.c_uint16),
                      _p(y64, C.c_double), _p(y32, C.c_float))
    return y64, y32


def bruteforce_min_cost(cnt) -> int:
    cnt = _c(cnt, np.uint64)
    return int(lib().oracle_bruteforce_min_cost(_p(cnt, C.c_uint64), cnt.size))


def limited_lengths(cnt, max_len: int):
    """Cheapest prefix-code lengths with no code longer than max_len (<= 16); -> (len uint8[A], cost)."""
    cnt = _c(cnt, np.uint64)
    ln = np.zeros(cnt.size, np.uint8)
    cost = C.c_uint64(0)
    _check(lib().oracle_limited_lengths(_p(cnt, C.c_uint64), cnt.size, int(max_len), _p(ln, C.c_uint8), C.byref(cost)),
           "limited_lengths")
    return ln, int(cost.value)


def bruteforce_min_cost_limited(cnt, max_len: int) -> int:
    cnt = _c(cnt, np.uint64)
    return int(lib().oracle_bruteforce_min_cost_limited(_p(cnt, C.c_uint64), cnt.size, int(max_len)))


def codebook_from_symbols(q, bits: int):
    """histogram -> lengths -> canonical codes; -> (len uint8[A], code uint32[A], cnt)."""
    cnt = histogram(q, bits)
    ln = huffman_lengths(cnt)
    return ln, canonical_codes(ln), cnt
