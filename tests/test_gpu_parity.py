"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Bars: decoded integers bit-exact; fp32 dequant bit-exact; bf16 within 1 ulp
(the kernels round to nearest even, so equality is expected and asserted as
<= 1 ulp); GEMV relative error <= 1e-3 against the fp64 oracle, both as
||y - y*||_2 / ||y*||_2 and as max_r |y_r - y*_r| <= 1e-3 * max(|y*_r|, rms(y*)).
Inputs never come from the HIP path: symbols, codebooks and streams are built
by the oracle (or by the host library and re-decoded by the oracle)."""
import os

import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2505_02380_amd as E
from paper_2505_02380_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _oracle_encoded(sym, bits, chunk, rows=0, cols=0, s=1.0, z=0, sub=0):
    """EncodedTensor whose codebook, stream (and entry points inside the segments, if sub is given) all come from
    the oracle."""
    ln, code, _ = oracle.codebook_from_symbols(sym, bits)
    stream, off = oracle.encode(sym, ln, code, chunk)
    full = np.zeros(1 << bits, np.uint8)
    full[: ln.size] = ln
    cb = E.entro_codebook_from_lengths(full, bits)
    assert np.array_equal(cb.codes(), code)
    qp = B.QParams(np.float32(s), int(z), bits, E.ENTRO_ASYMMETRIC)
    enc = B.EncodedTensor(stream, off, sym.size, chunk, cb, qp, rows, cols)
    if sub:
        enc.sub_symbols, enc.sub_bits = sub, oracle.sub_index(sym, ln, chunk, sub)
    return enc


def _bf16_ulp_diff(a_bits, b_bits):
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, 0x8000 - u, u)       # monotone integer order of bf16 patterns
    return np.abs(key(a_bits) - key(b_bits))


def _gpu_decode(enc, out_type, batch=False):
    dt = E.to_device(enc, DEV)
    nbytes = enc.n if out_type == E.ENTRO_U8 else (enc.n + 1) // 2
    out = torch.full((nbytes + 64,), 0xAB, dtype=torch.uint8, device=DEV)      # guard bytes behind the output
    t = dt.ctensor(out)
    if batch:
        ws = torch.zeros(E.entro_workspace_bytes([t], E.ENTRO_OP_DECODE), dtype=torch.uint8, device=DEV)
        E.entro_decode_batch([t], out_type, ws)
    else:
        E.entro_decode(t, out_type)
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    assert np.all(res[nbytes:] == 0xAB), "wrote past the end of the output"
    return res[:nbytes]


def _gpu_dequant(enc, out_type, batch=False):
    dt = E.to_device(enc, DEV)
    dtype = torch.float32 if out_type == E.ENTRO_F32 else torch.bfloat16
    out = torch.zeros(enc.n + 16, dtype=dtype, device=DEV)
    t = dt.ctensor(out)
    if batch:
        ws = torch.zeros(E.entro_workspace_bytes([t], E.ENTRO_OP_DEQUANT), dtype=torch.uint8, device=DEV)
        E.entro_decode_dequant_batch([t], out_type, ws)
    else:
        E.entro_decode_dequant(t, out_type)
    torch.cuda.synchronize()
    assert torch.all(out[enc.n:] == 0), "wrote past the end of the output"
    if out_type == E.ENTRO_F32:
        return out[: enc.n].cpu().numpy()
    return out[: enc.n].view(torch.int16).cpu().numpy().view(np.uint16)


def _gpu_gemv(enc, xb, y_type, batch=False):
    dt = E.to_device(enc, DEV)
    x = torch.from_numpy(xb.view(np.int16)).to(DEV).view(torch.bfloat16)
    y = torch.zeros(enc.rows + 8, dtype=torch.float32 if y_type == E.ENTRO_F32 else torch.bfloat16, device=DEV)
    t = dt.ctensor(y, x)
    if batch:
        ws = torch.zeros(max(E.entro_workspace_bytes([t], E.ENTRO_OP_GEMV), 16), dtype=torch.uint8, device=DEV)
        E.entro_decode_gemv_batch([t], y_type, ws)
    else:
        need = E.entro_gemv_workspace_bytes(t)
        ws = torch.zeros(need, dtype=torch.uint8, device=DEV) if need else None
        E.entro_decode_gemv(t, y_type, ws)
    torch.cuda.synchronize()
    assert torch.all(y[enc.rows:] == 0)
    return y[: enc.rows].float().cpu().numpy().astype(np.float64)


def _assert_gemv_close(y, y_ref, tol=1e-3):
    rel = np.linalg.norm(y - y_ref) / np.linalg.norm(y_ref)
    rms = np.sqrt(np.mean(y_ref ** 2))
    worst = np.max(np.abs(y - y_ref) / np.maximum(np.abs(y_ref), rms))
    assert rel <= tol and worst <= tol, (rel, worst)


# ---------------------------------------------------------------- integer decode
@pytest.mark.parametrize("batch", [False, True])
def test_config1_round_trip_bit_exact(batch):
    spec = synth.config_tensors(1)[0]
    w = synth.make_tensor(spec)
    q, s, z = oracle.quantize(w, 8, oracle.ASYMMETRIC)
    enc = _oracle_encoded(q, 8, 4096, s=s, z=z)
    assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8, batch), q)
    # the host library's own chain, re-decoded by the oracle
    enc2 = E.encode_tensor(w, 8, E.ENTRO_ASYMMETRIC, 4096)
    ref = oracle.decode(enc2.stream, enc2.offsets, enc2.n, 4096, enc2.cb.lengths(), enc2.cb.codes())
    assert np.array_equal(_gpu_decode(enc2, E.ENTRO_U8, batch), ref)


@pytest.mark.parametrize("bits", [8, 4])
def test_adversarial_streams_bit_exact(bits):
    for name, sym, chunk in synth.adversarial_symbol_cases(bits):
        enc = _oracle_encoded(sym, bits, chunk)
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8), sym), name
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8, batch=True), sym), name
        if bits == 4:
            assert np.array_equal(_gpu_decode(enc, E.ENTRO_U4_PACKED), oracle.pack_u4(sym)), name


def test_odd_chunk_sizes_take_the_scalar_store_path():
    rng = np.random.default_rng(31)
    sym = np.minimum(rng.geometric(0.4, 40001) - 1, 255).astype(np.uint8)
    for chunk in (1, 7, 1000, 4100):
        enc = _oracle_encoded(sym, 8, chunk)
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8), sym), chunk
    sym4 = (sym & 15).astype(np.uint8)
    for chunk in (2, 30, 1002):
        enc = _oracle_encoded(sym4, 4, chunk)
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U4_PACKED), oracle.pack_u4(sym4)), chunk


def test_shorter_last_segment_of_every_shape():
    # the last segment's whole blocks go through the row path and the rest through the scalar path:
    # sweep its length over none / less than a block / whole blocks / blocks and a rest, alone in the
    # tensor, alone in its wave (65 segments) and beside full ones
    rng = np.random.default_rng(77)
    chunk = 512
    base = np.minimum(rng.geometric(0.3, 66 * chunk) - 1, 255).astype(np.uint8)
    base[rng.random(base.size) < 0.002] = 255                       # a few long codes
    for full in (0, 1, 64, 65):
        for last in (1, 63, 64, 65, 127, 128, 129, 256, 383, 511):
            sym = base[: full * chunk + last]
            enc = _oracle_encoded(sym, 8, chunk, s=0.0123, z=3)
            tag = (full, last)
            assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8), sym), tag
            assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8, batch=True), sym), tag
            ref32 = oracle.dequant_f32(sym, enc.qp.scale, 3)
            assert np.array_equal(_gpu_dequant(enc, E.ENTRO_F32).view(np.uint32), ref32.view(np.uint32)), tag
            refb = oracle.dequant_bf16(sym, enc.qp.scale, 3)
            assert _bf16_ulp_diff(_gpu_dequant(enc, E.ENTRO_BF16, batch=True), refb).max() <= 1, tag
            sym4 = (sym & 15).astype(np.uint8)
            enc4 = _oracle_encoded(sym4, 4, chunk)
            assert np.array_equal(_gpu_decode(enc4, E.ENTRO_U4_PACKED), oracle.pack_u4(sym4)), tag
            assert np.array_equal(_gpu_decode(enc4, E.ENTRO_U8), sym4), tag
            assert _bf16_ulp_diff(_gpu_dequant(enc4, E.ENTRO_BF16), oracle.dequant_bf16(sym4, enc4.qp.scale, 0)).max() <= 1, tag


def test_codes_of_every_length_up_to_32():
    # lengths 1..31, 32, 32: the deepest code the format allows; symbols drawn so long codes are common
    ln = np.zeros(256, np.uint8)
    ln[:33] = list(range(1, 32)) + [32, 32]
    rng = np.random.default_rng(32)
    sym = rng.integers(0, 33, 30000).astype(np.uint8)
    code = oracle.canonical_codes(ln)
    stream, off = oracle.encode(sym, ln, code, 512)
    cb = E.entro_codebook_from_lengths(ln, 8)
    enc = B.EncodedTensor(stream, off, sym.size, 512, cb, B.QParams(1.0, 0, 8, 1))
    assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8), sym)


def test_more_long_prefixes_than_the_second_level_holds():
    # lengths 1..7, eight codes of 14 bits and 240 of 15: Kraft sum exactly 1; the 15-bit codes own 120
    # prefixes of the first-level table, so every one of them goes through the canonical search
    ln = np.zeros(256, np.uint8)
    ln[:7] = range(1, 8)
    ln[7:15] = 14
    ln[15:255] = 15
    assert sum(2.0 ** -int(l) for l in ln if l) == 1.0
    rng = np.random.default_rng(15)
    sym = rng.integers(0, 255, 64 * 1024 + 77).astype(np.uint8)          # long codes everywhere
    code = oracle.canonical_codes(ln)
    for chunk in (1024, 4096):
        stream, off = oracle.encode(sym, ln, code, chunk)
        cb = E.entro_codebook_from_lengths(ln, 8)
        enc = B.EncodedTensor(stream, off, sym.size, chunk, cb, B.QParams(1.0, 0, 8, 1))
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8), sym)
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8, batch=True), sym)


@pytest.mark.parametrize("lengths", [
    list(range(1, 15)) + [15, 15],                 # the deepest complete code over 16 symbols
    [1, 3, 3, 4, 4, 5, 5, 6, 6, 7, 7, 8, 8, 8, 8, 0],   # complete over 15 symbols; codes up to 8 bits
    [7, 7, 7, 7, 7, 7, 7, 7, 8, 8, 8, 8, 8, 8, 8, 8],   # incomplete: pairs of 14..16 bits straddle the table width
])
def test_4bit_packed_pairs_that_the_table_does_not_hold(lengths):
    # packed 4-bit output decodes two symbols per lookup where both codes fit into the table index;
    # here many pairs do not (symbols drawn uniformly, so long codes are as common as short ones)
    ln = np.zeros(16, np.uint8)
    ln[:] = lengths
    rng = np.random.default_rng(sum(lengths))
    used = int(np.count_nonzero(ln))
    sym = rng.integers(0, used, 96 * 1024 + 301).astype(np.uint8)
    sym[: 40 * 1024] = np.minimum(rng.geometric(0.5, 40 * 1024) - 1, used - 1)   # and a stretch of mostly short ones
    code = oracle.canonical_codes(ln)
    for chunk in (256, 4096, 1002):
        stream, off = oracle.encode(sym, ln, code, chunk)
        cb = E.entro_codebook_from_lengths(ln, 4)
        enc = B.EncodedTensor(stream, off, sym.size, chunk, cb, B.QParams(1.0, 0, 4, 1))
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U4_PACKED), oracle.pack_u4(sym)), chunk
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U4_PACKED, batch=True), oracle.pack_u4(sym)), chunk
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8), sym), chunk


@pytest.mark.parametrize("max_len", [11, 14, 16])
def test_length_limited_codebooks_decode_like_any_other(max_len):
    # codes capped below, at and above the first-level table's width; lengths from the oracle's
    # minimisation, stream from the oracle's encoder, decoded on the GPU and by the oracle's tree walk
    spec = synth.config_tensors(4)[1]                          # k: 1024 x 4096, the longest codes of the set
    w = synth.make_tensor(spec)
    q, s, z = oracle.quantize(w, 8, oracle.ASYMMETRIC)
    cnt = oracle.histogram(q, 8)
    ln, cost = oracle.limited_lengths(cnt, max_len)
    assert ln.max() <= max_len and oracle.huffman_lengths(cnt).max() > 16
    code = oracle.canonical_codes(ln)
    stream, off = oracle.encode(q, ln, code, 4096)
    assert int(off[-1]) == cost
    cb = E.entro_codebook_from_lengths(ln, 8)
    enc = B.EncodedTensor(stream, off, q.size, 4096, cb, B.QParams(np.float32(s), int(z), 8, E.ENTRO_ASYMMETRIC))
    assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8, batch=True), q)
    assert np.array_equal(oracle.decode(stream, off, q.size, 4096, ln, code), q)
    assert _bf16_ulp_diff(_gpu_dequant(enc, E.ENTRO_BF16), oracle.dequant_bf16(q, s, z)).max() <= 1
    # the library's own limited codebook costs the same and decodes the same
    enc2 = E.encode_tensor(w, 8, E.ENTRO_ASYMMETRIC, 4096, max_len=max_len)
    assert enc2.cb.max_len <= max_len and enc2.total_bits == cost
    assert np.array_equal(_gpu_decode(enc2, E.ENTRO_U8), q)


def test_phi3_shaped_4bit_packed():
    spec = synth.config_tensors(3)[1]                          # o: 3072 x 3072, Laplace, 4-bit
    w = synth.make_tensor(spec)
    q, s, z = oracle.quantize(w, 4, oracle.ASYMMETRIC)
    enc = _oracle_encoded(q, 4, 8192, s=s, z=z)
    assert np.array_equal(_gpu_decode(enc, E.ENTRO_U4_PACKED, batch=True), oracle.pack_u4(q))
    assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8), q)
    # the byte, fp32 and bf16 outputs of an all-4-bit launch also decode two symbols per lookup
    assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8, batch=True), q)
    f = _gpu_dequant(enc, E.ENTRO_F32, batch=True)
    assert np.array_equal(f.view(np.uint32), oracle.dequant_f32(q, s, z).view(np.uint32))
    b = _gpu_dequant(enc, E.ENTRO_BF16)
    assert _bf16_ulp_diff(b, oracle.dequant_bf16(q, s, z)).max() <= 1


def test_4bit_and_8bit_tensors_in_one_launch():
    # a launch with both alphabets cannot use the two-codes-per-entry tables: every tensor, the 4-bit
    # ones included, goes through the single-code tables
    rng = np.random.default_rng(48)
    encs, refs = [], []
    for bits, n in ((4, 300 * 1024 + 5), (8, 200 * 1024), (4, 64 * 1024)):
        sym = np.minimum(rng.geometric(0.35, n) - 1, (1 << bits) - 1).astype(np.uint8)
        encs.append(_oracle_encoded(sym, bits, 1024, s=np.float32(0.05), z=2))
        refs.append(sym)
    dts = [E.to_device(e, DEV) for e in encs]
    outs = [torch.zeros(e.n, dtype=torch.bfloat16, device=DEV) for e in encs]
    ts = [d.ctensor(o) for d, o in zip(dts, outs)]
    ws = torch.zeros(E.entro_workspace_bytes(ts, E.ENTRO_OP_DEQUANT), dtype=torch.uint8, device=DEV)
    plan = E.entro_plan_init(ts, E.ENTRO_OP_DEQUANT, E.ENTRO_BF16, ws)
    assert plan.pair_tables == 0
    E.entro_plan_run(plan)
    torch.cuda.synchronize()
    for e, o, r in zip(encs, outs, refs):
        got = o.view(torch.int16).cpu().numpy().view(np.uint16)
        assert _bf16_ulp_diff(got, oracle.dequant_bf16(r, e.qp.scale, e.qp.zero_point)).max() <= 1
    only4 = [ts[0], ts[2]]
    plan4 = E.entro_plan_init(only4, E.ENTRO_OP_DEQUANT, E.ENTRO_BF16, ws)
    assert plan4.pair_tables == 1


# ----------------------------------------------------------------------- dequant
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("batch", [False, True])
def test_dequant_fp32_bit_exact_and_bf16_within_one_ulp(bits, batch):
    spec = synth.TensorSpec(4, 0, 1, "k", 1024, 4096, "student_t", 5.0, 0.02, 0.0, bits, 1, 4242 + bits)
    w = synth.make_tensor(spec)
    q, s, z = oracle.quantize(w, bits, oracle.ASYMMETRIC)
    enc = _oracle_encoded(q, bits, 4096, s=s, z=z)
    f = _gpu_dequant(enc, E.ENTRO_F32, batch)
    assert np.array_equal(f.view(np.uint32), oracle.dequant_f32(q, s, z).view(np.uint32))
    b = _gpu_dequant(enc, E.ENTRO_BF16, batch)
    assert _bf16_ulp_diff(b, oracle.dequant_bf16(q, s, z)).max() <= 1


def test_dequant_ragged_and_unsigned_and_offgrid_zero_point():
    rng = np.random.default_rng(5)
    sym = rng.integers(170, 256, 2048).astype(np.uint8)        # norm-gain-like, one half-full segment
    enc = _oracle_encoded(sym, 8, 4096, s=np.float32(1.2 / 255), z=0)
    assert np.array_equal(_gpu_dequant(enc, E.ENTRO_F32).view(np.uint32),
                          oracle.dequant_f32(sym, enc.qp.scale, 0).view(np.uint32))
    sym = np.minimum(rng.geometric(0.2, 3 * 4096 + 5) - 1, 255).astype(np.uint8)
    for z in (-255, 300, 17):
        enc = _oracle_encoded(sym, 8, 4096, s=np.float32(0.37), z=z)
        assert np.array_equal(_gpu_dequant(enc, E.ENTRO_F32).view(np.uint32),
                              oracle.dequant_f32(sym, enc.qp.scale, z).view(np.uint32))
        assert _bf16_ulp_diff(_gpu_dequant(enc, E.ENTRO_BF16), oracle.dequant_bf16(sym, enc.qp.scale, z)).max() <= 1


# -------------------------------------------------------------------------- gemv
@pytest.mark.parametrize("rows,cols,chunk", [
    (96, 4096, 4096),        # one row per segment
    (40, 14336, 4096),       # a row is 3.5 segments (the `down` projection)
    (300, 2048, 4096),       # two rows per segment
    (77, 300, 4096),         # rows do not divide segments
    (5, 9000, 1024),         # long rows, ragged last segment
    (1, 100, 4096),          # a single short row
    (512, 128, 1024),        # eight whole rows per segment
    (300, 192, 1024),        # five and a third rows per segment
    (160, 3072, 8192),       # the phi3 shapes: two and two thirds rows per segment
    (4096 + 11, 64, 4096),   # the shortest rows the kernel takes: one per block; ragged last segment
    (100, 72, 512),          # a block may hold the end of one row and the start of the next
    (64, 4096, 64),          # the shortest segments: sixty-four per row
    (7, 1000, 4096),         # rows of 125 pieces of eight, segments of four rows and a bit
    (31, 60, 128),           # rows shorter than a block: element by element
])
@pytest.mark.parametrize("batch", [False, True])
def test_gemv_against_fp64_oracle(rows, cols, chunk, batch):
    spec = synth.TensorSpec(4, 0, 0, "g", rows, cols, "student_t", 5.0, 0.02, 0.0, 8, 1, 9000 + rows)
    w = synth.make_tensor(spec)
    q, s, z = oracle.quantize(w, 8, oracle.ASYMMETRIC)
    enc = _oracle_encoded(q, 8, chunk, rows, cols, s, z)
    xb = synth.make_x_bf16(0, rows % 7, cols)
    y_ref, _ = oracle.gemv(q, rows, cols, s, z, xb)
    _assert_gemv_close(_gpu_gemv(enc, xb, E.ENTRO_F32, batch), y_ref)
    y_bf = _gpu_gemv(enc, xb, E.ENTRO_BF16, batch)
    assert np.all(np.abs(y_bf - y_ref) <= 2.0 ** -7 * np.abs(y_ref) + 1e-3 * np.sqrt(np.mean(y_ref ** 2)))


@pytest.mark.parametrize("rows,cols,chunk", [
    (160, 3072, 8192),       # phi3 shapes: two and two thirds rows per segment
    (64, 8192, 8192),        # one row per segment
    (96, 4096, 1024),        # four segments per row
    (520, 128, 4096),        # thirty-two rows per segment
    (33, 144, 256),          # rows and blocks out of step
    (50, 200, 512),          # cols a multiple of 8 but not of 16
    (300, 64, 256),          # the shortest rows the kernel takes: one per half block
    (90, 72, 128),           # a half block may hold the end of one row and the start of the next
    (40, 100, 256),          # cols not a multiple of 8: element by element, with the pair tables
    (3, 8192, 256),          # a few long rows of many segments
])
@pytest.mark.parametrize("batch", [False, True])
def test_gemv_4bit_two_symbols_per_lookup(rows, cols, chunk, batch):
    rng = np.random.default_rng(rows + cols)
    sym = np.minimum(rng.geometric(0.45, rows * cols) - 1, 15).astype(np.uint8)
    sym[rng.random(sym.size) < 0.01] = 15                      # some long codes
    enc = _oracle_encoded(sym, 4, chunk, rows=rows, cols=cols, s=np.float32(0.07), z=6)
    xb = synth.make_x_bf16(1, rows % 4, cols)
    y_ref, _ = oracle.gemv(sym, rows, cols, enc.qp.scale, 6, xb)
    _assert_gemv_close(_gpu_gemv(enc, xb, E.ENTRO_F32, batch), y_ref)
    _assert_gemv_close(_gpu_gemv(enc, xb, E.ENTRO_BF16, batch), y_ref, tol=5e-3)   # y itself rounded to bf16: half an ulp, up to 2^-8 of the value, on top of the 1e-3


def test_gemv_unit_vector_picks_a_column_exactly():
    rows, cols = 64, 4096
    rng = np.random.default_rng(1)
    q = rng.integers(0, 256, rows * cols).astype(np.uint8)
    s, z = np.float32(0.0123), 131
    enc = _oracle_encoded(q, 8, 4096, rows, cols, s, z)
    e = np.zeros(cols, np.float32)
    e[1234] = 1.0
    y = _gpu_gemv(enc, synth.f32_to_bf16_bits(e), E.ENTRO_F32)
    col = oracle.dequant_f32(q, s, z).reshape(rows, cols)[:, 1234]
    assert np.array_equal(y.astype(np.float32), col)


# ------------------------------------------------------------- batched launches
# ------------------------------------------------- entry points inside the segments
@pytest.mark.parametrize("batch", [False, True])
@pytest.mark.parametrize("bits,chunk,sub,n", [(8, 4096, 256, 300 * 4096), (8, 4096, 256, 70 * 4096 + 1000), (8, 4096, 1024, 9 * 4096 + 5),
                                              (8, 2048, 128, 64 * 2048 + 130), (8, 1024, 64, 33 * 1024 + 63), (4, 8192, 512, 20 * 8192 + 700),
                                              (8, 4096, 4096, 3 * 4096 + 17), (8, 1000, 250, 17 * 1000 + 3)])
def test_entry_points_inside_segments_every_output(bits, chunk, sub, n, batch):
    """A lane decodes a piece of a segment from its entry point: the outputs are those of the oracle's plain decode."""
    rng = np.random.default_rng(n + sub)
    sym = np.clip(np.rint(rng.standard_t(4, n) * (6 if bits == 8 else 0.8) + (1 << (bits - 1))), 0, (1 << bits) - 1).astype(np.uint8)
    enc = _oracle_encoded(sym, bits, chunk, s=0.0173, z=(1 << (bits - 1)) + 3, sub=sub)
    q = oracle.decode(enc.stream, enc.offsets, n, chunk, enc.cb.lengths(), enc.cb.codes())
    assert np.array_equal(q, sym)
    assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8, batch), q)
    if bits == 4:
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U4_PACKED, batch), oracle.pack_u4(q))
    w32 = _gpu_dequant(enc, E.ENTRO_F32, batch)
    assert np.array_equal(w32.view(np.uint32), oracle.dequant_f32(q, enc.qp.scale, enc.qp.zero_point).view(np.uint32))
    assert _bf16_ulp_diff(_gpu_dequant(enc, E.ENTRO_BF16, batch), oracle.dequant_bf16(q, enc.qp.scale, enc.qp.zero_point)).max() <= 1


@pytest.mark.parametrize("batch", [False, True])
@pytest.mark.parametrize("rows,cols,chunk,sub", [(128, 4096, 4096, 256), (96, 14336, 4096, 256), (300, 1024, 4096, 512), (65, 1536, 2048, 128),
                                                 (40, 200, 1024, 64), (520, 128, 4096, 1024), (67, 8192, 2048, 128),
                                                 (200, 2048, 2048, 128)])
def test_gemv_with_entry_points_inside_segments(rows, cols, chunk, sub, batch):
    rng = np.random.default_rng(rows * cols + sub)
    sym = np.clip(np.rint(rng.standard_t(5, rows * cols) * 6 + 128), 0, 255).astype(np.uint8)
    enc = _oracle_encoded(sym, 8, chunk, rows, cols, s=0.011, z=125, sub=sub)
    xb = synth.f32_to_bf16_bits(rng.standard_normal(cols).astype(np.float32))
    y_ref, _ = oracle.gemv(sym, rows, cols, enc.qp.scale, enc.qp.zero_point, xb)
    _assert_gemv_close(_gpu_gemv(enc, xb, E.ENTRO_F32, batch), y_ref)
    plain = _oracle_encoded(sym, 8, chunk, rows, cols, s=0.011, z=125)
    # against the same product with one lane per segment: the same sums in another order
    assert np.allclose(_gpu_gemv(enc, xb, E.ENTRO_F32, batch), _gpu_gemv(plain, xb, E.ENTRO_F32, batch), rtol=1e-4, atol=1e-4)


def test_large_launch_merges_pieces_into_coarser_lanes():
    """A launch with more pieces than the chip has lanes lets a lane take 2^k pieces (the coarsest cut that still
    gives every lane slot a lane): 40 M symbols with entry points every 64 symbols in segments of 1024."""
    n, chunk, sub = 40 * 1024 * 1024, 1024, 64
    rng = np.random.default_rng(5)
    sym = np.clip(np.rint(rng.standard_t(4, n) * 5 + 128), 0, 255).astype(np.uint8)
    enc = _oracle_encoded(sym, 8, chunk, s=0.02, z=131, sub=sub)
    assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8, True), sym)
    assert _bf16_ulp_diff(_gpu_dequant(enc, E.ENTRO_BF16, False), oracle.dequant_bf16(sym, enc.qp.scale, enc.qp.zero_point)).max() <= 1


def test_last_round_of_every_stretch_is_drawn_with_finer_lanes_every_output():
    """A launch of several rounds per workgroup over tensors with entry points inside their segments: the last
    round of every stretch is decoded by lanes that take pieces instead of segments (and as before for the
    tensor that has no entry points); every output element, guard bytes between the outputs."""
    rng = np.random.default_rng(61)
    chunk = 256
    shapes = [(2500, 64), (1125, 64), (2125, 128), (37, 0), (750, 32)]     # (units of 64 segments, entry-point spacing)
    encs, refs = [], []
    for i, (units, sub) in enumerate(shapes):
        n = units * 64 * chunk - (0 if i != 2 else 21 * chunk + 5)          # tensor 2 ends inside a segment
        sym = np.minimum(rng.geometric(0.12 + 0.05 * i, n) - 1, 255).astype(np.uint8)
        encs.append(_oracle_encoded(sym, 8, chunk, s=np.float32(0.01), z=2 + i, sub=sub))
        refs.append(sym)
    dts = [E.to_device(e, DEV) for e in encs]
    for op, out_type, dtype, width in ((E.ENTRO_OP_DECODE, E.ENTRO_U8, torch.uint8, 1),
                                       (E.ENTRO_OP_DEQUANT, E.ENTRO_BF16, torch.bfloat16, 2),
                                       (E.ENTRO_OP_DEQUANT, E.ENTRO_F32, torch.float32, 4)):
        guard = 64 // width
        sizes = [(e.n + guard - 1) // guard * guard + guard for e in encs]   # every output 64-byte aligned, a guard behind it
        buf = torch.full((sum(sizes),), 7, dtype=dtype, device=DEV)
        outs, pos = [], 0
        for e, sz in zip(encs, sizes):
            outs.append(buf[pos:pos + e.n])
            pos += sz
        ts = [d.ctensor(o) for d, o in zip(dts, outs)]
        ws = torch.zeros(E.entro_workspace_bytes(ts, op), dtype=torch.uint8, device=DEV)
        plan = E.entro_plan_init(ts, op, out_type, ws)
        E.entro_plan_run(plan)
        torch.cuda.synchronize()
        pos = 0
        for e, r, o, sz in zip(encs, refs, outs, sizes):
            if dtype == torch.uint8:
                assert np.array_equal(o.cpu().numpy(), r)
            elif dtype == torch.bfloat16:
                assert np.array_equal(o.view(torch.int16).cpu().numpy().view(np.uint16),
                                      oracle.dequant_bf16(r, e.qp.scale, e.qp.zero_point))
            else:
                assert np.array_equal(o.view(torch.int32).cpu().numpy().view(np.uint32),
                                      oracle.dequant_f32(r, e.qp.scale, e.qp.zero_point).view(np.uint32))
            assert bool((buf[pos + e.n:pos + sz] == 7).all()), "a guard element was written"
            pos += sz


def test_staged_plan_init_does_not_block_and_batch_calls_return_before_their_kernel_ends():
    from paper_2505_02380_amd.workload import prepare_config
    encs = prepare_config(4, layers=8)
    dts = [E.to_device(e, DEV) for e in encs]
    outs = [torch.zeros(e.n, dtype=torch.bfloat16, device=DEV) for e in encs]
    ts = [d.ctensor(o) for d, o in zip(dts, outs)]
    ws = torch.zeros(E.entro_workspace_bytes(ts, E.ENTRO_OP_DEQUANT), dtype=torch.uint8, device=DEV)
    staging = torch.zeros(E.entro_plan_staging_bytes(ts, E.ENTRO_OP_DEQUANT), dtype=torch.uint8).pin_memory()
    assert staging.numel() > 0
    torch.cuda.synchronize()
    # something long in front of it on the stream: the staged form must not wait for it
    filler = torch.empty(1 << 30, dtype=torch.uint8, device=DEV)
    for _ in range(8):
        filler.fill_(1)
    busy = torch.cuda.Event()
    busy.record()
    plan = E.entro_plan_init_staged(ts, E.ENTRO_OP_DEQUANT, E.ENTRO_BF16, ws, staging)
    E.entro_plan_run(plan)
    assert not busy.query(), "entro_plan_init_staged or entro_plan_run waited for the stream"
    torch.cuda.synchronize()
    first = [o.clone() for o in outs]
    for o in outs:
        o.zero_()
    # the batch form waits once for the stream (the table upload), then enqueues: it is back before its kernel ends
    done = torch.cuda.Event()
    E.entro_decode_dequant_batch(ts, E.ENTRO_BF16, ws)
    done.record()
    assert not done.query(), "entro_decode_dequant_batch returned only after its kernel had ended"
    torch.cuda.synchronize()
    for a, b in zip(first, outs):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    e = encs[3]
    q = oracle.decode(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes())
    assert _bf16_ulp_diff(outs[3].view(torch.int16).cpu().numpy().view(np.uint16),
                          oracle.dequant_bf16(q, e.qp.scale, e.qp.zero_point)).max() <= 1


def test_many_tensors_in_one_launch():
    rng = np.random.default_rng(12)
    encs, refs = [], []
    for i, (n, chunk) in enumerate([(300000, 4096), (2048, 4096), (4096 * 300 + 1, 4096), (70000, 1000), (5, 4096)]):
        sym = np.minimum(rng.geometric(0.1 + 0.15 * i, n) - 1, 255).astype(np.uint8)
        encs.append(_oracle_encoded(sym, 8, chunk, s=np.float32(0.01 * (i + 1)), z=10 * i))
        refs.append(sym)
    dts = [E.to_device(e, DEV) for e in encs]
    outs = [torch.zeros(e.n, dtype=torch.uint8, device=DEV) for e in encs]
    ts = [d.ctensor(o) for d, o in zip(dts, outs)]
    ws = torch.zeros(E.entro_workspace_bytes(ts, E.ENTRO_OP_DECODE), dtype=torch.uint8, device=DEV)
    plan = E.entro_plan_init(ts, E.ENTRO_OP_DECODE, E.ENTRO_U8, ws)
    for _ in range(2):                                         # a prepared plan can be replayed
        for o in outs:
            o.zero_()
        E.entro_plan_run(plan)
        torch.cuda.synchronize()
        for o, r in zip(outs, refs):
            assert np.array_equal(o.cpu().numpy(), r)
    fouts = [torch.zeros(e.n, dtype=torch.bfloat16, device=DEV) for e in encs]
    ts = [d.ctensor(o) for d, o in zip(dts, fouts)]
    E.entro_decode_dequant_batch(ts, E.ENTRO_BF16, ws)
    torch.cuda.synchronize()
    for e, o, r in zip(encs, fouts, refs):
        got = o.view(torch.int16).cpu().numpy().view(np.uint16)
        assert _bf16_ulp_diff(got, oracle.dequant_bf16(r, e.qp.scale, e.qp.zero_point)).max() <= 1


def test_launch_with_a_few_units_per_work_item():
    # 64-symbol segments make many units (64 segments each) out of little data: ~880 units over the
    # chip's workgroups give work items of a few units, workgroup shares that start and end inside
    # tensors, stretches shorter than a workgroup has wavefronts, and a last unit that is not full
    rng = np.random.default_rng(88)
    chunk, cols = 64, 128
    encs, refs, xs = [], [], []
    for i, units in enumerate((300, 77, 500, 1)):
        n = units * 64 * chunk - (0 if i != 2 else 38 * chunk)          # tensor 2 ends inside a unit
        sym = np.minimum(rng.geometric(0.2 + 0.1 * i, n) - 1, 255).astype(np.uint8)
        encs.append(_oracle_encoded(sym, 8, chunk, rows=n // cols, cols=cols, s=np.float32(0.02), z=3 + i))
        refs.append(sym)
        xs.append(synth.make_x_bf16(9, i, cols))
    dts = [E.to_device(e, DEV) for e in encs]
    outs = [torch.zeros(e.n, dtype=torch.uint8, device=DEV) for e in encs]
    ts = [d.ctensor(o) for d, o in zip(dts, outs)]
    ws = torch.zeros(E.entro_workspace_bytes(ts, E.ENTRO_OP_DECODE), dtype=torch.uint8, device=DEV)
    plan = E.entro_plan_init(ts, E.ENTRO_OP_DECODE, E.ENTRO_U8, ws)
    assert 1 < plan.item_units < 10
    E.entro_plan_run(plan)
    torch.cuda.synchronize()
    for o, r in zip(outs, refs):
        assert np.array_equal(o.cpu().numpy(), r)
    ys = [torch.zeros(e.rows, dtype=torch.float32, device=DEV) for e in encs]
    xd = [torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16) for x in xs]
    ts = [d.ctensor(y, x) for d, y, x in zip(dts, ys, xd)]
    wsg = torch.zeros(max(256, E.entro_workspace_bytes(ts, E.ENTRO_OP_GEMV)), dtype=torch.uint8, device=DEV)
    E.entro_decode_gemv_batch(ts, E.ENTRO_F32, wsg)
    torch.cuda.synchronize()
    for e, y, r, x in zip(encs, ys, refs, xs):
        y_ref, _ = oracle.gemv(r, e.rows, cols, e.qp.scale, e.qp.zero_point, x)
        _assert_gemv_close(y.cpu().numpy().astype(np.float64), y_ref)


def test_random_shapes_all_outputs():
    """Seeded sweep over sizes, segment lengths, alphabets and code-length profiles, every output type,
    single and batched: bit-exact integers and fp32, bf16 within 1 ulp, GEMV within 1e-3."""
    # ENTRO_SWEEP_SEED / ENTRO_SWEEP_CASES widen the sweep for a soak run
    rng = np.random.default_rng(int(os.environ.get("ENTRO_SWEEP_SEED", "2025")))
    chunks8 = [1, 64, 128, 192, 256, 1000, 1024, 4096, 8192]
    for case in range(int(os.environ.get("ENTRO_SWEEP_CASES", "150"))):
        bits = 4 if case % 3 == 0 else 8
        A = 1 << bits
        chunk = int(rng.choice(chunks8))
        if bits == 4 and chunk % 2:
            chunk += 1
        n = int(rng.integers(1, 40 * chunk + 2)) if chunk > 64 else int(rng.integers(1, 5000))
        if case % 2:                                             # a matrix shape, for the GEMV below
            cols = int(rng.choice([8192, 4096, 3072, 1024, 192, 72, 64, 40, 7]))
            n = cols * max(1, n // cols)
        kind = case % 4
        if kind == 0:
            sym = np.minimum(rng.geometric(rng.uniform(0.05, 0.7), n) - 1, A - 1)
        elif kind == 1:
            sym = rng.integers(0, A, n)
        elif kind == 2:
            sym = np.where(rng.random(n) < 0.97, rng.integers(0, 3, n), rng.integers(0, A, n))   # rare long codes
        else:
            sym = np.full(n, int(rng.integers(0, A)))
            sym[rng.integers(0, n, max(1, n // 50))] = int(rng.integers(0, A))
        sym = sym.astype(np.uint8)
        z = int(rng.integers(-3, A + 3))
        enc = _oracle_encoded(sym, bits, chunk, s=np.float32(rng.uniform(1e-3, 1.0)), z=z)
        tag = (case, bits, chunk, n, kind)
        batch = bool(case & 1)
        assert np.array_equal(_gpu_decode(enc, E.ENTRO_U8, batch), sym), tag
        if bits == 4:
            assert np.array_equal(_gpu_decode(enc, E.ENTRO_U4_PACKED, not batch), oracle.pack_u4(sym)), tag
        f = _gpu_dequant(enc, E.ENTRO_F32, not batch)
        assert np.array_equal(f.view(np.uint32), oracle.dequant_f32(sym, enc.qp.scale, z).view(np.uint32)), tag
        b = _gpu_dequant(enc, E.ENTRO_BF16, batch)
        assert _bf16_ulp_diff(b, oracle.dequant_bf16(sym, enc.qp.scale, z)).max() <= 1, tag
        # a matrix shape for the same symbols, if n factors conveniently
        for cols in (8192, 4096, 3072, 1024, 192, 72, 64, 40, 7):
            if n % cols == 0:
                rows = n // cols
                encg = _oracle_encoded(sym, bits, chunk, rows=rows, cols=cols, s=enc.qp.scale, z=z)
                xb = synth.make_x_bf16(case, 0, cols)
                y_ref, _ = oracle.gemv(sym, rows, cols, enc.qp.scale, z, xb)
                if np.linalg.norm(y_ref) > 0:
                    _assert_gemv_close(_gpu_gemv(encg, xb, E.ENTRO_F32, batch), y_ref)
                break


def test_mistral_layer_launch_shape_sampled_against_oracle():
    """Four mistral-7B-shaped layers in the batched launch bench.py uses (more work items than the chip
    holds workgroups, so workgroups walk several items and tensors); sampled segments vs the oracle."""
    from paper_2505_02380_amd.workload import prepare_config
    encs = prepare_config(4, layers=4)
    dts = [E.to_device(e, DEV) for e in encs]
    outs = [torch.zeros(e.n, dtype=torch.bfloat16, device=DEV) for e in encs]
    ts = [d.ctensor(o) for d, o in zip(dts, outs)]
    ws = torch.zeros(E.entro_workspace_bytes(ts, E.ENTRO_OP_DEQUANT), dtype=torch.uint8, device=DEV)
    E.entro_decode_dequant_batch(ts, E.ENTRO_BF16, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    for e, o in zip(encs, outs):
        n_chunks = e.offsets.size - 1
        picks = sorted(set([0, n_chunks - 1] + rng.integers(0, n_chunks, 6).tolist()))
        host = o.view(torch.int16).cpu().numpy().view(np.uint16)
        for k in picks:
            q = oracle.decode_chunks(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes(), k, 1)
            lo, hi = k * e.chunk_symbols, min((k + 1) * e.chunk_symbols, e.n)
            ref = oracle.dequant_bf16(q[lo:hi], e.qp.scale, e.qp.zero_point)
            assert _bf16_ulp_diff(host[lo:hi], ref).max() <= 1, (e.name, k)
    # the same layer through the fused GEMV (7 linears in one launch)
    xs = [torch.from_numpy(synth.make_x_bf16(i // 7, i % 7, e.cols).view(np.int16)).to(DEV).view(torch.bfloat16)
          for i, e in enumerate(encs)]
    ys = [torch.zeros(e.rows, dtype=torch.float32, device=DEV) for e in encs]
    ts = [d.ctensor(y, x) for d, y, x in zip(dts, ys, xs)]
    ws = torch.zeros(E.entro_workspace_bytes(ts, E.ENTRO_OP_GEMV), dtype=torch.uint8, device=DEV)
    E.entro_decode_gemv_batch(ts, E.ENTRO_F32, ws)
    torch.cuda.synchronize()
    for i, (e, y) in enumerate(zip(encs, ys)):
        rows = sorted(set([0, e.rows - 1] + rng.integers(0, e.rows, 4).tolist()))
        yh = y.cpu().numpy().astype(np.float64)
        xb = synth.make_x_bf16(i // 7, i % 7, e.cols)
        sub = np.empty((len(rows), e.cols), np.uint8)
        for j, r in enumerate(rows):
            k0, k1 = (r * e.cols) // e.chunk_symbols, ((r + 1) * e.cols - 1) // e.chunk_symbols
            q = oracle.decode_chunks(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes(),
                                     k0, k1 - k0 + 1)
            sub[j] = q[r * e.cols:(r + 1) * e.cols]
        y_ref, _ = oracle.gemv(sub, len(rows), e.cols, e.qp.scale, e.qp.zero_point, xb)
        rms = np.sqrt(np.mean(yh ** 2))
        assert np.max(np.abs(yh[rows] - y_ref) / np.maximum(np.abs(y_ref), rms)) <= 1e-3, e.name


def test_prepared_launches_replay_in_a_hip_graph():
    """entro_plan_run only enqueues kernels (no allocation, no copies, no memset), so it can be captured:
    every replay of the graph must give the eager result, with eager work and synchronisation between
    the replays."""
    rng = np.random.default_rng(4242)
    encs, refs_q = [], []
    for rows, cols, chunk in [(96, 4096, 4096), (40, 1024, 4096), (33, 3072, 1024)]:
        sym = np.minimum(rng.geometric(0.3, rows * cols) - 1, 255).astype(np.uint8)
        encs.append(_oracle_encoded(sym, 8, chunk, rows=rows, cols=cols, s=np.float32(0.01), z=3))
        refs_q.append(sym)
    dts = [E.to_device(e, DEV) for e in encs]
    # dequant -> bf16
    outs = [torch.zeros(e.n, dtype=torch.bfloat16, device=DEV) for e in encs]
    ts = [d.ctensor(o) for d, o in zip(dts, outs)]
    ws = torch.zeros(E.entro_workspace_bytes(ts, E.ENTRO_OP_DEQUANT), dtype=torch.uint8, device=DEV)
    plan = E.entro_plan_init(ts, E.ENTRO_OP_DEQUANT, E.ENTRO_BF16, ws)
    # GEMV -> fp32 (the third tensor's rows straddle segments: two kernels per launch)
    xs = [torch.from_numpy(synth.make_x_bf16(7, i, e.cols).view(np.int16)).to(DEV).view(torch.bfloat16) for i, e in enumerate(encs)]
    ys = [torch.zeros(e.rows, dtype=torch.float32, device=DEV) for e in encs]
    dts_g = [E.to_device(e, DEV) for e in encs]
    tg = [d.ctensor(y, x) for d, y, x in zip(dts_g, ys, xs)]
    wsg = torch.zeros(max(256, E.entro_workspace_bytes(tg, E.ENTRO_OP_GEMV)), dtype=torch.uint8, device=DEV)
    plan_g = E.entro_plan_init(tg, E.ENTRO_OP_GEMV, E.ENTRO_F32, wsg)
    torch.cuda.synchronize()
    E.entro_plan_run(plan)
    E.entro_plan_run(plan_g)
    torch.cuda.synchronize()
    eager_o = [o.clone() for o in outs]
    eager_y = [y.clone() for y in ys]
    for e, q, o in zip(encs, refs_q, eager_o):
        assert _bf16_ulp_diff(o.view(torch.int16).cpu().numpy().view(np.uint16),
                              oracle.dequant_bf16(q, e.qp.scale, e.qp.zero_point)).max() <= 1
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            E.entro_plan_run(plan)
            E.entro_plan_run(plan_g)
    torch.cuda.synchronize()
    for rep in range(3):
        for o in outs:
            o.fill_(1.0)                                   # eager work between the replays
        for y in ys:
            y.fill_(-7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, ref in zip(outs, eager_o):
            assert torch.equal(o.view(torch.int16), ref.view(torch.int16)), rep
        for y, ref in zip(ys, eager_y):
            assert torch.equal(y, ref), rep                # the row sums are taken in a fixed order: bit-identical


def test_plain_uint8_gemv_comparison_kernel_matches_the_oracle():
    """bench.py's comparison kernel (its own shared object, not the library): all products in one launch."""
    import bench_kernels
    shapes = [(300, 4096), (7, 14336), (1000, 64), (33, 1040), (1, 16)]
    products, refs = [], []
    for rows, cols in shapes:
        rng = np.random.default_rng(rows)
        q = np.minimum(rng.geometric(0.05, rows * cols) - 1, 255).astype(np.uint8)
        xb = synth.make_x_bf16(2, rows % 5, cols)
        y_ref, _ = oracle.gemv(q, rows, cols, np.float32(0.013), 21, xb)
        y = torch.full((rows + 4,), 9.0, dtype=torch.float32, device=DEV)
        products.append((torch.from_numpy(q).to(DEV), rows, cols, np.float32(0.013), 21,
                         torch.from_numpy(xb.view(np.int16)).to(DEV).view(torch.bfloat16), y))
        refs.append(y_ref)
    bench_kernels.PlainGemv(products, DEV).run()
    torch.cuda.synchronize()
    for (q, rows, cols, s, z, x, y), y_ref in zip(products, refs):
        got = y.cpu().numpy()
        assert np.all(got[rows:] == 9.0)
        _assert_gemv_close(got[:rows].astype(np.float64), y_ref)
