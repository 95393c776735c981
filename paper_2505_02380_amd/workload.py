"""Prepare the synthetic workloads: generate -> quantize -> codebook -> encode, in host threads."""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional

import synth

from . import binding as B


def default_threads() -> int:
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        return int(env)
    return max(1, min(16, os.cpu_count() or 1))


def encode_spec(spec: "synth.TensorSpec", chunk_symbols: Optional[int] = None, max_len: int = 0,
                sub_symbols: int = 0) -> B.EncodedTensor:
    w = synth.make_tensor(spec)
    cs = chunk_symbols or synth.config_chunk_symbols(spec.cfg)
    enc = B.encode_tensor(w, spec.bits, spec.scheme, cs, rows=spec.rows, cols=spec.cols,
                          name=f"L{spec.layer}.{spec.name}", max_len=max_len, sub_symbols=sub_symbols)
    return enc


def prepare_config(cfg: int, layers: Optional[int] = None, threads: Optional[int] = None,
                   progress=None, chunk_symbols: Optional[int] = None, max_len: int = 0,
                   sub_symbols: int = 0) -> List[B.EncodedTensor]:
    """Encoded tensors of workload `cfg` in the order of synth.config_tensors.

    chunk_symbols overrides the workload's own segment size (an encode-time choice per tensor);
    max_len > 0 asks for length-limited codebooks; sub_symbols > 0 adds entry points inside the segments."""
    specs = synth.config_tensors(cfg, layers)
    threads = threads or default_threads()
    # the host library spawns its own threads per call; keep the product bounded
    os.environ.setdefault("ENTRO_HOST_THREADS", "2")
    out: List[Optional[B.EncodedTensor]] = [None] * len(specs)

    def work(i):
        out[i] = encode_spec(specs[i], chunk_symbols, max_len, sub_symbols)
        if progress:
            progress(i, len(specs))
        return i

    order = sorted(range(len(specs)), key=lambda i: -specs[i].n)   # big tensors first
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(work, order))
    return out  # type: ignore[return-value]
