"""GPU parity at full size: every element of every tensor of the five workloads.

Each test prepares a whole workload (synthetic, seeded), runs it through the
prepared batched launch that bench.py times, and compares every output tensor
in full with the CPU oracle, which runs on host threads (one oracle call per
tensor and thread).  Outputs sit in one buffer with guard bytes between them,
which must come back untouched.  Bars as in test_gpu_parity.py: integers and
fp32 patterns bit-exact, bf16 within 1 ulp, GEMV within 1e-3 of the fp64 oracle.
"""
import sys
import time
from concurrent.futures import ThreadPoolExecutor
from functools import lru_cache

import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2505_02380_amd as E
from paper_2505_02380_amd.workload import prepare_config, default_threads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GUARD = 256            # bytes between two outputs
GUARD_BYTE = 0xA5


def _say(msg):
    print(f"[full-config {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


@lru_cache(maxsize=2)
def _prepared(cfg):
    _say(f"preparing workload {cfg}")
    # with entry points inside the segments (every 256 symbols; 512 in the segments of 8192), as bench.py
    # prepares them: batched launches draw what is left over behind a stretch's whole rounds from those
    encs = prepare_config(cfg, sub_symbols=512 if cfg == 3 else 256)
    return encs, [E.to_device(e, DEV) for e in encs]


@lru_cache(maxsize=2)
def _oracle_symbols(cfg):
    """Every tensor of the workload decoded by the oracle (bit-at-a-time tree walk), on host threads."""
    encs, _ = _prepared(cfg)
    _say(f"oracle decode of workload {cfg} on {default_threads()} threads")

    def one(e):
        return oracle.decode(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes())

    with ThreadPoolExecutor(default_threads()) as pool:
        return list(pool.map(one, encs))


def _guarded_outputs(sizes_bytes, torch_dtype):
    """One device buffer holding outputs of the given byte sizes, GUARD bytes of GUARD_BYTE around each."""
    starts, pos = [], GUARD
    for sz in sizes_bytes:
        starts.append(pos)
        pos += (sz + GUARD - 1) // GUARD * GUARD + GUARD
    buf = torch.full((pos,), GUARD_BYTE, dtype=torch.uint8, device=DEV)
    views = [buf[s:s + sz].view(torch_dtype) for s, sz in zip(starts, sizes_bytes)]
    return buf, starts, views


def _check_guards(buf, starts, sizes_bytes):
    """Everything between the outputs still holds the guard pattern."""
    pos = 0
    for s, sz in zip(starts, sizes_bytes):
        assert bool(torch.all(buf[pos:s] == GUARD_BYTE)), "a kernel wrote in front of an output tensor"
        pos = s + sz
    assert bool(torch.all(buf[pos:] == GUARD_BYTE)), "a kernel wrote behind an output tensor"


def _compare_all(views, refs, what, to_host, same):
    """Compare every output with its reference, tensor by tensor (host copies are made one at a time)."""
    for i, (v, make_ref) in enumerate(zip(views, refs)):
        got = to_host(v)
        ref = make_ref()
        assert got.shape == ref.shape, (what, i)
        assert same(got, ref), f"{what}: tensor {i} differs from the oracle"


def _bf16_within_one_ulp(a_bits, b_bits):
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, 0x8000 - u, u)
    return int(np.abs(key(a_bits) - key(b_bits)).max()) <= 1


def _run_plan(ts, op, out_type):
    ws = torch.zeros(max(256, E.entro_workspace_bytes(ts, op)), dtype=torch.uint8, device=DEV)
    plan = E.entro_plan_init(ts, op, out_type, ws)
    E.entro_plan_run(plan)
    torch.cuda.synchronize()
    return ws


def test_config2_smollm_shaped_u8_every_element():
    """configs[1]: 24 layers x 7 linears with outliers plus 49 unsigned norm-gain vectors of half a segment,
    one launch, decoded to bytes."""
    encs, dts = _prepared(2)
    assert sum(1 for e in encs if e.n == 2048) == 49
    sizes = [e.n for e in encs]
    buf, starts, views = _guarded_outputs(sizes, torch.uint8)
    _run_plan([d.ctensor(v) for d, v in zip(dts, views)], E.ENTRO_OP_DECODE, E.ENTRO_U8)
    q = _oracle_symbols(2)
    _compare_all(views, [lambda a=a: a for a in q], "config 2 -> u8", lambda v: v.cpu().numpy(), np.array_equal)
    _check_guards(buf, starts, sizes)
    _say("config 2: every element matches")
    # and as the same launch without the entry points (every lane a whole segment)
    buf.fill_(GUARD_BYTE)
    _run_plan([d.ctensor(v, entry_points=False) for d, v in zip(dts, views)], E.ENTRO_OP_DECODE, E.ENTRO_U8)
    _compare_all(views, [lambda a=a: a for a in q], "config 2 -> u8, whole segments", lambda v: v.cpu().numpy(), np.array_equal)
    _check_guards(buf, starts, sizes)
    _say("config 2 without entry points: every element matches")


def test_config3_phi3_shaped_packed_u4_and_bf16_every_element():
    """configs[2]: 32 layers x 4 tensors of 4-bit symbols, segments of 8192: packed nibbles, and bf16."""
    encs, dts = _prepared(3)
    q = _oracle_symbols(3)
    sizes = [(e.n + 1) // 2 for e in encs]
    buf, starts, views = _guarded_outputs(sizes, torch.uint8)
    _run_plan([d.ctensor(v) for d, v in zip(dts, views)], E.ENTRO_OP_DECODE, E.ENTRO_U4_PACKED)
    _compare_all(views, [lambda a=a: oracle.pack_u4(a) for a in q], "config 3 -> packed u4",
                 lambda v: v.cpu().numpy(), np.array_equal)
    _check_guards(buf, starts, sizes)
    del buf, views
    _say("config 3 packed: every element matches")
    sizes = [2 * e.n for e in encs]
    buf, starts, views = _guarded_outputs(sizes, torch.bfloat16)
    _run_plan([d.ctensor(v) for d, v in zip(dts, views)], E.ENTRO_OP_DEQUANT, E.ENTRO_BF16)
    _compare_all(views, [lambda a=a, e=e: oracle.dequant_bf16(a, e.qp.scale, e.qp.zero_point) for a, e in zip(q, encs)],
                 "config 3 -> bf16", lambda v: v.view(torch.int16).cpu().numpy().view(np.uint16), _bf16_within_one_ulp)
    _check_guards(buf, starts, sizes)
    _say("config 3 bf16: every element matches")


def test_config4_mistral_shaped_bf16_every_element_and_fp32_layer():
    """configs[3], the headline launch: 224 tensors -> bf16, every element; layer 0 also as fp32 bit patterns."""
    encs, dts = _prepared(4)
    q = _oracle_symbols(4)
    sizes = [2 * e.n for e in encs]
    buf, starts, views = _guarded_outputs(sizes, torch.bfloat16)
    _run_plan([d.ctensor(v) for d, v in zip(dts, views)], E.ENTRO_OP_DEQUANT, E.ENTRO_BF16)
    _compare_all(views, [lambda a=a, e=e: oracle.dequant_bf16(a, e.qp.scale, e.qp.zero_point) for a, e in zip(q, encs)],
                 "config 4 -> bf16", lambda v: v.view(torch.int16).cpu().numpy().view(np.uint16), _bf16_within_one_ulp)
    _check_guards(buf, starts, sizes)
    del buf, views
    _say("config 4 bf16: every element matches")
    sizes = [4 * e.n for e in encs[:7]]
    buf, starts, views = _guarded_outputs(sizes, torch.float32)
    _run_plan([d.ctensor(v) for d, v in zip(dts[:7], views)], E.ENTRO_OP_DEQUANT, E.ENTRO_F32)
    _compare_all(views, [lambda a=a, e=e: oracle.dequant_f32(a, e.qp.scale, e.qp.zero_point).view(np.uint32)
                         for a, e in zip(q[:7], encs[:7])],
                 "config 4 layer 0 -> fp32", lambda v: v.view(torch.int32).cpu().numpy().view(np.uint32), np.array_equal)
    _check_guards(buf, starts, sizes)
    _say("config 4 fp32 layer: every element matches")


def _gemv_refs(encs, q, xs):
    def one(i):
        e = encs[i]
        return oracle.gemv(q[i], e.rows, e.cols, e.qp.scale, e.qp.zero_point, xs[i])[0]

    with ThreadPoolExecutor(default_threads()) as pool:
        return list(pool.map(one, range(len(encs))))


def _assert_rows_close(y, y_ref, what):
    rel = np.linalg.norm(y - y_ref) / np.linalg.norm(y_ref)
    rms = np.sqrt(np.mean(y_ref ** 2))
    worst = np.max(np.abs(y - y_ref) / np.maximum(np.abs(y_ref), rms))
    assert rel <= 1e-3 and worst <= 1e-3, (what, rel, worst)


def test_config5_gemv_every_row_of_every_product():
    """configs[4]: all 224 products, every row (the second-stage sum of every `down` included), once as one
    launch and once as the layer's four dependent launches."""
    encs, dts = _prepared(4)
    q = _oracle_symbols(4)
    xs = [synth.make_x_bf16(i // 7, i % 7, e.cols) for i, e in enumerate(encs)]
    _say("oracle GEMV (fp64) of all 224 products")
    refs = _gemv_refs(encs, q, xs)
    xd = [torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16) for x in xs]
    sizes = [4 * e.rows for e in encs]
    buf, starts, views = _guarded_outputs(sizes, torch.float32)
    _run_plan([d.ctensor(y, x) for d, y, x in zip(dts, views, xd)], E.ENTRO_OP_GEMV, E.ENTRO_F32)
    for i, (v, r) in enumerate(zip(views, refs)):
        _assert_rows_close(v.cpu().numpy().astype(np.float64), r, f"one launch, {encs[i].name}")
    _check_guards(buf, starts, sizes)
    _say("config 5, one launch: every row matches")
    buf2, starts2, views2 = _guarded_outputs(sizes, torch.float32)
    keep = []
    for layer in range(len(encs) // 7):
        for a, b in ((0, 3), (3, 4), (4, 6), (6, 7)):          # q,k,v | o | gate,up | down
            idx = range(7 * layer + a, 7 * layer + b)
            keep.append(_run_plan([dts[i].ctensor(views2[i], xd[i]) for i in idx], E.ENTRO_OP_GEMV, E.ENTRO_F32))
    for i, (v, r) in enumerate(zip(views2, refs)):
        _assert_rows_close(v.cpu().numpy().astype(np.float64), r, f"dependent launches, {encs[i].name}")
    _check_guards(buf2, starts2, sizes)
    _say("config 5, four launches per layer: every row matches")
