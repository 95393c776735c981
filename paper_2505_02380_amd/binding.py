"""ctypes binding of include/entro.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))

ENTRO_UNSIGNED, ENTRO_ASYMMETRIC = 0, 1
ENTRO_U8, ENTRO_U4_PACKED, ENTRO_F32, ENTRO_BF16 = 0, 1, 2, 3
ENTRO_OP_DECODE, ENTRO_OP_DEQUANT, ENTRO_OP_GEMV = 0, 1, 2
ENTRO_OK = 0
(ENTRO_ERR_NULL, ENTRO_ERR_BITS, ENTRO_ERR_SCHEME, ENTRO_ERR_SIZE, ENTRO_ERR_NONFINITE, ENTRO_ERR_RANGE,
 ENTRO_ERR_SYMBOL, ENTRO_ERR_CODE_TOO_LONG, ENTRO_ERR_CAPACITY, ENTRO_ERR_CORRUPT, ENTRO_ERR_ALIGN,
 ENTRO_ERR_DEVICE) = range(1, 13)


class QParams(C.Structure):
    _fields_ = [("scale", C.c_float), ("zero_point", C.c_int32), ("bits", C.c_int32), ("scheme", C.c_int32)]


class Codebook(C.Structure):
    _fields_ = [("bits", C.c_int32), ("n_used", C.c_int32), ("max_len", C.c_int32), ("reserved", C.c_int32),
                ("len", C.c_uint8 * 256), ("code", C.c_uint32 * 256)]

    def lengths(self) -> np.ndarray:
        return np.frombuffer(self.len, dtype=np.uint8, count=1 << self.bits).copy()

    def codes(self) -> np.ndarray:
        return np.frombuffer(self.code, dtype=np.uint32, count=1 << self.bits).copy()


class CTensor(C.Structure):
    _fields_ = [("stream", C.c_void_p), ("stream_bytes", C.c_uint64), ("offsets", C.c_void_p),
                ("n", C.c_uint64), ("chunk_symbols", C.c_uint32), ("rows", C.c_uint32), ("cols", C.c_uint32),
                ("sub_symbols", C.c_uint32), ("cb", C.POINTER(Codebook)), ("qp", QParams), ("x", C.c_void_p),
                ("out", C.c_void_p), ("sub_bits", C.c_void_p)]


class Plan(C.Structure):
    _fields_ = [("workspace", C.c_void_p), ("workspace_bytes", C.c_uint64), ("op", C.c_uint32),
                ("out", C.c_uint32), ("count", C.c_uint32), ("n_items", C.c_uint32), ("n_fix", C.c_uint32),
                ("item_units", C.c_uint32), ("pair_tables", C.c_uint32), ("gemv_multirow", C.c_uint32), ("wide_tables", C.c_uint32), ("reserved", C.c_uint32), ("off_tensors", C.c_uint64), ("off_items", C.c_uint64),
                ("off_partials", C.c_uint64), ("off_fix", C.c_uint64)]


class EntroError(RuntimeError):
    def __init__(self, status: int, what: str):
        msg = f"{what}: {entro_status_string(status)} (status {status})"
        if status == ENTRO_ERR_DEVICE:
            msg += f" [{entro_last_device_error()}]"
        super().__init__(msg)
        self.status = status


_lib = None


def library_path() -> str:
    return os.path.join(HERE, "libentro.so")


def lib():
    """Load libentro.so (built in-tree by paper_2505_02380_amd/build.py).  No CPU fallback exists."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: run `python -m paper_2505_02380_amd.build` "
                           "(or __graft_entry__.build()) first; there is no CPU fallback")
    L = C.CDLL(path)
    u8p, u64p, f32p = C.POINTER(C.c_uint8), C.POINTER(C.c_uint64), C.POINTER(C.c_float)
    cbp, tp, pp = C.POINTER(Codebook), C.POINTER(CTensor), C.POINTER(Plan)
    sig = {
        "entro_quantize": (C.c_int, [f32p, C.c_uint64, C.c_int, C.c_int, u8p, C.POINTER(QParams)]),
        "entro_build_codebook": (C.c_int, [u8p, C.c_uint64, C.c_int, cbp]),
        "entro_codebook_from_counts": (C.c_int, [u64p, C.c_int, cbp]),
        "entro_codebook_from_lengths": (C.c_int, [u8p, C.c_int, cbp]),
        "entro_codebook_from_counts_limited": (C.c_int, [u64p, C.c_int, C.c_int, cbp]),
        "entro_build_codebook_limited": (C.c_int, [u8p, C.c_uint64, C.c_int, C.c_int, cbp]),
        "entro_num_chunks": (C.c_uint64, [C.c_uint64, C.c_uint32]),
        "entro_encode_bound": (C.c_uint64, [C.c_uint64, cbp]),
        "entro_encode": (C.c_int, [u8p, C.c_uint64, cbp, C.c_uint32, u8p, C.c_uint64, u64p, u64p]),
        "entro_check_offsets": (C.c_int, [u64p, C.c_uint64, C.c_uint32, C.c_uint64, cbp]),
        "entro_sub_index": (C.c_int, [u8p, C.c_uint64, cbp, C.c_uint32, C.c_uint32, C.POINTER(C.c_uint16)]),
        "entro_bits_saved": (C.c_double, [C.c_int, C.c_double]),
        "entro_theoretical_speedup": (C.c_double, [C.c_int, C.c_double]),
        "entro_status_string": (C.c_char_p, [C.c_int]),
        "entro_decode": (C.c_int, [tp, C.c_int, C.c_void_p]),
        "entro_decode_dequant": (C.c_int, [tp, C.c_int, C.c_void_p]),
        "entro_gemv_workspace_bytes": (C.c_uint64, [tp]),
        "entro_decode_gemv": (C.c_int, [tp, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p]),
        "entro_decode_gemv_static": (C.c_int, [tp, C.c_int, C.c_void_p]),
        "entro_workspace_bytes": (C.c_uint64, [tp, C.c_uint32, C.c_int]),
        "entro_plan_init": (C.c_int, [pp, tp, C.c_uint32, C.c_int, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p]),
        "entro_plan_staging_bytes": (C.c_uint64, [tp, C.c_uint32, C.c_int]),
        "entro_plan_init_staged": (C.c_int, [pp, tp, C.c_uint32, C.c_int, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64,
                                             C.c_void_p]),
        "entro_plan_run": (C.c_int, [pp, C.c_void_p]),
        "entro_decode_batch": (C.c_int, [tp, C.c_uint32, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p]),
        "entro_decode_dequant_batch": (C.c_int, [tp, C.c_uint32, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p]),
        "entro_decode_gemv_batch": (C.c_int, [tp, C.c_uint32, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p]),
        "entro_last_device_error": (C.c_char_p, []),
        "entro_range_device": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]),
        "entro_qparams_from_range": (C.c_int, [C.c_float, C.c_float, C.c_uint32, C.c_int, C.c_int, C.POINTER(QParams)]),
        "entro_scheme_for_range": (C.c_int, [C.c_float, C.c_float]),
        "entro_quantize_device": (C.c_int, [C.c_void_p, C.c_uint64, C.POINTER(QParams), C.c_void_p, C.c_void_p, C.c_void_p]),
        "entro_encoded_bytes": (C.c_uint64, [u64p, cbp]),
        "entro_encode_device": (C.c_int, [C.c_void_p, C.c_uint64, cbp, C.c_uint32, C.c_void_p, C.c_uint64, C.c_void_p,
                                          C.c_void_p, C.c_void_p]),
        "entro_encode_device_status": (C.c_int, [C.c_uint32]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


EXPORTED = ["entro_quantize", "entro_build_codebook", "entro_codebook_from_counts",
            "entro_codebook_from_lengths", "entro_codebook_from_counts_limited", "entro_build_codebook_limited", "entro_num_chunks", "entro_encode_bound", "entro_encode",
            "entro_check_offsets", "entro_sub_index", "entro_bits_saved", "entro_theoretical_speedup", "entro_status_string",
            "entro_decode", "entro_decode_dequant", "entro_gemv_workspace_bytes", "entro_decode_gemv", "entro_decode_gemv_static",
            "entro_workspace_bytes", "entro_plan_init", "entro_plan_staging_bytes", "entro_plan_init_staged", "entro_plan_run", "entro_decode_batch",
            "entro_decode_dequant_batch", "entro_decode_gemv_batch", "entro_last_device_error",
            "entro_range_device", "entro_qparams_from_range", "entro_scheme_for_range", "entro_quantize_device",
            "entro_encoded_bytes", "entro_encode_device", "entro_encode_device_status"]


def _ptr(a: np.ndarray, t):
    return a.ctypes.data_as(C.POINTER(t))


def _check(status: int, what: str):
    if status != ENTRO_OK:
        raise EntroError(status, what)


# ----------------------------------------------------------------- host calls
def entro_status_string(status: int) -> str:
    return lib().entro_status_string(status).decode()


def entro_last_device_error() -> str:
    return lib().entro_last_device_error().decode()


def entro_quantize(w: np.ndarray, bits: int, scheme: int):
    """-> (q uint8[n], QParams)."""
    w = np.ascontiguousarray(w, dtype=np.float32).ravel()
    q = np.empty(w.size, np.uint8)
    qp = QParams()
    _check(lib().entro_quantize(_ptr(w, C.c_float), w.size, bits, scheme, _ptr(q, C.c_uint8), C.byref(qp)),
           "entro_quantize")
    return q, qp


def entro_build_codebook(q: np.ndarray, bits: int) -> Codebook:
    q = np.ascontiguousarray(q, dtype=np.uint8).ravel()
    cb = Codebook()
    _check(lib().entro_build_codebook(_ptr(q, C.c_uint8), q.size, bits, C.byref(cb)), "entro_build_codebook")
    return cb


def entro_codebook_from_counts(counts: np.ndarray, bits: int) -> Codebook:
    counts = np.ascontiguousarray(counts, dtype=np.uint64)
    assert counts.size == 1 << bits
    cb = Codebook()
    _check(lib().entro_codebook_from_counts(_ptr(counts, C.c_uint64), bits, C.byref(cb)),
           "entro_codebook_from_counts")
    return cb


def entro_codebook_from_counts_limited(counts: np.ndarray, bits: int, max_len: int) -> Codebook:
    counts = np.ascontiguousarray(counts, dtype=np.uint64)
    assert counts.size == 1 << bits
    cb = Codebook()
    _check(lib().entro_codebook_from_counts_limited(_ptr(counts, C.c_uint64), bits, int(max_len), C.byref(cb)),
           "entro_codebook_from_counts_limited")
    return cb


def entro_build_codebook_limited(q: np.ndarray, bits: int, max_len: int) -> Codebook:
    q = np.ascontiguousarray(q, dtype=np.uint8).ravel()
    cb = Codebook()
    _check(lib().entro_build_codebook_limited(_ptr(q, C.c_uint8), q.size, bits, int(max_len), C.byref(cb)),
           "entro_build_codebook_limited")
    return cb


def entro_codebook_from_lengths(lengths: np.ndarray, bits: int) -> Codebook:
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    assert lengths.size == 1 << bits
    cb = Codebook()
    _check(lib().entro_codebook_from_lengths(_ptr(lengths, C.c_uint8), bits, C.byref(cb)),
           "entro_codebook_from_lengths")
    return cb


def entro_num_chunks(n: int, chunk_symbols: int) -> int:
    return int(lib().entro_num_chunks(n, chunk_symbols))


def entro_encode_bound(n: int, cb: Codebook) -> int:
    return int(lib().entro_encode_bound(n, C.byref(cb)))


def entro_encode(q: np.ndarray, cb: Codebook, chunk_symbols: int):
    """-> (stream uint8[stream_bytes], offsets uint64[n_chunks + 1])."""
    q = np.ascontiguousarray(q, dtype=np.uint8).ravel()
    n = q.size
    # worst-case capacity; untouched pages of it are never committed
    stream = np.empty(max(entro_encode_bound(n, cb), 32), np.uint8)
    offsets = np.empty(entro_num_chunks(n, chunk_symbols) + 1, np.uint64)
    nbytes = C.c_uint64(0)
    _check(lib().entro_encode(_ptr(q, C.c_uint8), n, C.byref(cb), chunk_symbols, _ptr(stream, C.c_uint8),
                              stream.size, C.byref(nbytes), _ptr(offsets, C.c_uint64)), "entro_encode")
    return stream[: nbytes.value].copy(), offsets


def entro_sub_index(q: np.ndarray, cb: Codebook, chunk_symbols: int, sub_symbols: int) -> np.ndarray:
    """-> uint16[ceil(n / sub_symbols)]: stream bits of every piece of sub_symbols symbols."""
    q = np.ascontiguousarray(q, dtype=np.uint8).ravel()
    sub = np.empty(entro_num_chunks(q.size, sub_symbols), np.uint16)
    _check(lib().entro_sub_index(_ptr(q, C.c_uint8), q.size, C.byref(cb), chunk_symbols, sub_symbols,
                                 _ptr(sub, C.c_uint16)), "entro_sub_index")
    return sub


def entro_check_offsets(offsets: np.ndarray, n: int, chunk_symbols: int, stream_bytes: int, cb: Codebook) -> int:
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    return int(lib().entro_check_offsets(_ptr(offsets, C.c_uint64), n, chunk_symbols, stream_bytes, C.byref(cb)))


def entro_bits_saved(bits: int, mean_code_len: float) -> float:
    return float(lib().entro_bits_saved(bits, mean_code_len))


def entro_theoretical_speedup(bits: int, mean_code_len: float) -> float:
    return float(lib().entro_theoretical_speedup(bits, mean_code_len))


# ------------------------------------------------------------- tensor holders
@dataclass
class EncodedTensor:
    """Host-side result of quantize -> codebook -> encode for one tensor."""
    stream: np.ndarray
    offsets: np.ndarray
    n: int
    chunk_symbols: int
    cb: Codebook
    qp: QParams
    rows: int = 0
    cols: int = 0
    name: str = ""
    sub_symbols: int = 0                   # spacing of the entry points inside the segments (0: none)
    sub_bits: Optional[np.ndarray] = None  # uint16 piece lengths (entro_sub_index)

    @property
    def total_bits(self) -> int:
        return int(self.offsets[-1])

    @property
    def mean_code_len(self) -> float:
        return self.total_bits / self.n


def encode_tensor(w: np.ndarray, bits: int, scheme: int, chunk_symbols: int, rows: int = 0, cols: int = 0,
                  name: str = "", return_q: bool = False, max_len: int = 0, sub_symbols: int = 0):
    """entro_quantize -> entro_build_codebook (length-limited if max_len is given) -> entro_encode
    (-> entro_sub_index if sub_symbols is given)."""
    q, qp = entro_quantize(w, bits, scheme)
    cb = entro_build_codebook_limited(q, bits, max_len) if max_len else entro_build_codebook(q, bits)
    stream, offsets = entro_encode(q, cb, chunk_symbols)
    enc = EncodedTensor(stream, offsets, q.size, chunk_symbols, cb, qp, rows, cols, name)
    if sub_symbols:
        enc.sub_symbols, enc.sub_bits = sub_symbols, entro_sub_index(q, cb, chunk_symbols, sub_symbols)
    return (enc, q) if return_q else enc


class DeviceTensor:
    """Device copies of one encoded tensor plus its output buffer (torch owns the memory)."""

    def __init__(self, enc: EncodedTensor, device="cuda", stream=None, offsets=None):
        import torch
        self.enc = enc
        # stream / offsets given: the tensor was encoded on the device and enc holds no host copy of them
        self.stream = torch.from_numpy(enc.stream).to(device) if stream is None else stream
        self.offsets = torch.from_numpy(enc.offsets.view(np.int64)).to(device) if offsets is None else offsets
        self.sub_bits = torch.from_numpy(enc.sub_bits.view(np.int16)).to(device) if enc.sub_symbols else None
        self.x = None
        self.out = None

    def ctensor(self, out, x=None, entry_points: bool = True) -> CTensor:
        """The tensor as the device entry points take it; entry_points=False leaves the entry points inside
        the segments out (every lane then takes a whole segment)."""
        e = self.enc
        t = CTensor()
        t.stream = self.stream.data_ptr()
        t.stream_bytes = self.stream.numel()
        t.offsets = self.offsets.data_ptr()
        t.n = e.n
        t.chunk_symbols = e.chunk_symbols
        t.sub_symbols = e.sub_symbols if entry_points else 0
        t.sub_bits = self.sub_bits.data_ptr() if (self.sub_bits is not None and entry_points) else None
        t.rows, t.cols = e.rows, e.cols
        t.cb = C.pointer(e.cb)
        t.qp = e.qp
        t.x = x.data_ptr() if x is not None else None
        t.out = out.data_ptr()
        self.out, self.x = out, x
        return t


def to_device(enc: EncodedTensor, device="cuda") -> DeviceTensor:
    return DeviceTensor(enc, device)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _tensor_array(ts: Sequence[CTensor]):
    arr = (CTensor * len(ts))(*ts)
    return arr


# --------------------------------------------------------------- device calls
def entro_decode(t: CTensor, out_type: int, stream=None):
    _check(lib().entro_decode(C.byref(t), out_type, _stream_ptr(stream)), "entro_decode")


def entro_decode_dequant(t: CTensor, out_type: int, stream=None):
    _check(lib().entro_decode_dequant(C.byref(t), out_type, _stream_ptr(stream)), "entro_decode_dequant")


def entro_gemv_workspace_bytes(t: CTensor) -> int:
    return int(lib().entro_gemv_workspace_bytes(C.byref(t)))


def entro_decode_gemv(t: CTensor, y_type: int, workspace=None, stream=None):
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().entro_decode_gemv(C.byref(t), y_type, ws_ptr, ws_bytes, _stream_ptr(stream)), "entro_decode_gemv")


def entro_decode_gemv_static(t: CTensor, y_type: int, stream=None):
    _check(lib().entro_decode_gemv_static(C.byref(t), y_type, _stream_ptr(stream)), "entro_decode_gemv_static")


def entro_workspace_bytes(ts: Sequence[CTensor], op: int) -> int:
    arr = _tensor_array(ts)
    return int(lib().entro_workspace_bytes(arr, len(ts), op))


def entro_plan_init(ts: Sequence[CTensor], op: int, out_type: int, workspace, stream=None) -> Plan:
    arr = _tensor_array(ts)
    plan = Plan()
    _check(lib().entro_plan_init(C.byref(plan), arr, len(ts), op, out_type, workspace.data_ptr(),
                                 workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "entro_plan_init")
    return plan


def entro_plan_staging_bytes(ts: Sequence[CTensor], op: int) -> int:
    arr = _tensor_array(ts)
    return int(lib().entro_plan_staging_bytes(arr, len(ts), op))


def entro_plan_init_staged(ts: Sequence[CTensor], op: int, out_type: int, workspace, staging, stream=None) -> Plan:
    """Non-blocking entro_plan_init: `staging` is a pinned host tensor (torch, uint8) that the caller keeps alive
    until the copy enqueued here has completed."""
    arr = _tensor_array(ts)
    plan = Plan()
    _check(lib().entro_plan_init_staged(C.byref(plan), arr, len(ts), op, out_type, workspace.data_ptr(),
                                        workspace.numel() * workspace.element_size(), staging.data_ptr(),
                                        staging.numel() * staging.element_size(), _stream_ptr(stream)),
           "entro_plan_init_staged")
    return plan


def entro_plan_run(plan: Plan, stream=None):
    _check(lib().entro_plan_run(C.byref(plan), _stream_ptr(stream)), "entro_plan_run")


def _batch(fn_name: str, ts, out_type, workspace, stream):
    arr = _tensor_array(ts)
    fn = getattr(lib(), fn_name)
    _check(fn(arr, len(ts), out_type, workspace.data_ptr(), workspace.numel() * workspace.element_size(),
              _stream_ptr(stream)), fn_name)


# ------------------------------------------------------- device-side compression
def entro_range_device(w, range16, stream=None):
    """min / max / non-finite flag of w (torch float32 device tensor) into range16 (16 bytes of device memory)."""
    _check(lib().entro_range_device(w.data_ptr(), w.numel(), range16.data_ptr(), _stream_ptr(stream)), "entro_range_device")


def entro_qparams_from_range(mn: float, mx: float, nonfinite: int, bits: int, scheme: int) -> QParams:
    qp = QParams()
    _check(lib().entro_qparams_from_range(mn, mx, nonfinite, bits, scheme, C.byref(qp)), "entro_qparams_from_range")
    return qp


def entro_scheme_for_range(mn: float, mx: float) -> int:
    return int(lib().entro_scheme_for_range(mn, mx))


def entro_quantize_device(w, qp: QParams, q, counts, stream=None):
    """q (uint8 device tensor, w.numel() bytes) and counts (int64 device tensor of 256) from w and qp."""
    _check(lib().entro_quantize_device(w.data_ptr(), w.numel(), C.byref(qp), q.data_ptr(), counts.data_ptr(),
                                       _stream_ptr(stream)), "entro_quantize_device")


def entro_encoded_bytes(counts: np.ndarray, cb: Codebook) -> int:
    counts = np.ascontiguousarray(counts, dtype=np.uint64)
    return int(lib().entro_encoded_bytes(_ptr(counts, C.c_uint64), C.byref(cb)))


def entro_encode_device(q, cb: Codebook, chunk_symbols: int, stream_out, offsets, status, stream=None):
    """Encode q (uint8 device tensor) into stream_out / offsets (device tensors); status: 4 bytes of device memory."""
    _check(lib().entro_encode_device(q.data_ptr(), q.numel(), C.byref(cb), chunk_symbols, stream_out.data_ptr(),
                                     stream_out.numel() * stream_out.element_size(), offsets.data_ptr(), status.data_ptr(),
                                     _stream_ptr(stream)), "entro_encode_device")


def entro_encode_device_status(word: int) -> int:
    return int(lib().entro_encode_device_status(int(word) & 0xFFFFFFFF))


def compress_on_device(w, bits: int, scheme: Optional[int], chunk_symbols: int, rows: int = 0, cols: int = 0, name: str = "",
                       max_len: int = 0, return_q: bool = False):
    """Range -> (s, z) -> quantise + count -> codebook -> encode for a float32 tensor that lives on the GPU.

    The three passes over the weights are kernels; the two small steps between them run in the host
    library on the 16 and 2048 bytes copied back.  scheme None: entro_scheme_for_range picks the grid.
    Returns a DeviceTensor ready for the decode calls.
    """
    import torch
    w = w.reshape(-1)
    dev = w.device
    small = torch.empty(4 + 1, dtype=torch.int32, device=dev)          # range (16 bytes) and the encoder's status word
    counts = torch.empty(256, dtype=torch.int64, device=dev)
    entro_range_device(w, small)
    r = small[:4].cpu().numpy()
    mn, mx = r[:2].view(np.float32)
    if scheme is None:
        scheme = entro_scheme_for_range(float(mn), float(mx))
    qp = entro_qparams_from_range(float(mn), float(mx), int(r[2]), bits, scheme)
    q = torch.empty(w.numel(), dtype=torch.uint8, device=dev)
    entro_quantize_device(w, qp, q, counts)
    cnt = counts.cpu().numpy().view(np.uint64)
    cb = (entro_codebook_from_counts_limited(cnt[: 1 << bits], bits, max_len) if max_len
          else entro_codebook_from_counts(cnt[: 1 << bits], bits))
    nbytes = entro_encoded_bytes(cnt, cb)
    stream_out = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    offsets = torch.empty(entro_num_chunks(w.numel(), chunk_symbols) + 1, dtype=torch.int64, device=dev)
    status = small[4:]
    entro_encode_device(q, cb, chunk_symbols, stream_out, offsets, status)
    _check(entro_encode_device_status(int(status.cpu()[0])), "entro_encode_device (status word)")
    enc = EncodedTensor(None, None, w.numel(), chunk_symbols, cb, qp, rows, cols, name)
    dt = DeviceTensor(enc, dev, stream=stream_out, offsets=offsets)
    return (dt, q) if return_q else dt


def entro_decode_batch(ts, out_type, workspace, stream=None):
    _batch("entro_decode_batch", ts, out_type, workspace, stream)


def entro_decode_dequant_batch(ts, out_type, workspace, stream=None):
    _batch("entro_decode_dequant_batch", ts, out_type, workspace, stream)


def entro_decode_gemv_batch(ts, y_type, workspace, stream=None):
    _batch("entro_decode_gemv_batch", ts, y_type, workspace, stream)
