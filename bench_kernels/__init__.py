"""ctypes face of bench_kernels/libentro_bench.so: the memory probe and the plain uint8 GEMV that bench.py
times beside libentro's kernels (comparison only; nothing in the library or its binding uses this)."""
import ctypes as C
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "kernels.hip")
LIB = os.path.join(HERE, "libentro_bench.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-shared"]

ITEM = np.dtype([("q", "<u8"), ("x", "<u8"), ("y", "<u8"), ("rows", "<u4"), ("cols", "<u4"), ("scale", "<f4"),
                 ("zero_point", "<f4"), ("first_task", "<u4"), ("reserved", "<u4")])
EXPORTED = ["bench_stream_probe", "bench_gemv_tasks", "bench_gemv_u8_plain"]
_lib = None


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    subprocess.check_call([HIPCC, *FLAGS, "-I", HERE, "-o", LIB, SRC])
    return LIB


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            raise RuntimeError(f"{LIB} is not built (python -c 'import __graft_entry__ as g; g.build()')")
        _lib = C.CDLL(LIB)
        _lib.bench_stream_probe.restype = C.c_int
        _lib.bench_stream_probe.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
        _lib.bench_gemv_tasks.restype = C.c_uint32
        _lib.bench_gemv_tasks.argtypes = [C.c_uint32]
        _lib.bench_gemv_u8_plain.restype = C.c_int
        _lib.bench_gemv_u8_plain.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p]
    return _lib


def _stream_ptr(stream):
    import torch
    return (stream or torch.cuda.current_stream()).cuda_stream


def stream_probe(src, read_bytes: int, dst, write_bytes: int, scratch, stream=None):
    rc = lib().bench_stream_probe(src.data_ptr(), int(read_bytes), dst.data_ptr(), int(write_bytes), scratch.data_ptr(),
                                  _stream_ptr(stream))
    if rc:
        raise RuntimeError(f"bench_stream_probe: {rc}")


class PlainGemv:
    """The products y_i = s_i (Q_i - z_i) x_i of a list of (q, rows, cols, scale, zero_point, x, y) with
    device tensors q (uint8), x (bf16), y (float32), prepared once, run as one launch per call."""

    def __init__(self, products, device):
        import torch
        items = np.zeros(len(products), ITEM)
        tasks = 0
        for i, (q, rows, cols, scale, zp, x, y) in enumerate(products):
            if cols % 16 or q.numel() != rows * cols or x.numel() != cols or y.numel() < rows:
                raise ValueError("shape")
            if (q.data_ptr() | x.data_ptr()) & 15:
                raise ValueError("alignment")
            items[i] = (q.data_ptr(), x.data_ptr(), y.data_ptr(), rows, cols, scale, float(zp), tasks, 0)
            tasks += lib().bench_gemv_tasks(rows)
        self.keep = products
        self.count, self.tasks = len(products), tasks
        self.items = torch.from_numpy(items.view(np.uint8)).to(device)

    def run(self, stream=None):
        rc = lib().bench_gemv_u8_plain(self.items.data_ptr(), self.count, self.tasks, _stream_ptr(stream))
        if rc:
            raise RuntimeError(f"bench_gemv_u8_plain: {rc}")
