"""Host side of libentro against the oracle and the paper's fixed points (CPU only).

Where several optimal Huffman codes exist the comparison is on what is unique:
total cost, Kraft equality and canonical form -- not the length vector."""
import ctypes as C
import os
import re
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth
import paper_2505_02380_amd as E
from paper_2505_02380_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_library_loads_and_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "entro.h")).read()
    declared = set(re.findall(r"\b(entro_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    L = E.lib()
    for name in sorted(declared):
        assert hasattr(L, name), f"libentro.so does not export {name}"
    assert set(B.EXPORTED) == declared


def test_comparison_kernels_live_in_their_own_library():
    """The memory probe and the plain uint8 GEMV that bench.py times are not part of libentro: they are built
    into bench_kernels/libentro_bench.so, which exports what its header declares."""
    import bench_kernels
    header = open(os.path.join(ROOT, "bench_kernels", "entro_bench.h")).read()
    declared = set(re.findall(r"\b(bench_[a-z0-9_]+)\s*\(", header))
    assert declared == set(bench_kernels.EXPORTED)
    if not os.path.exists(bench_kernels.LIB):
        bench_kernels.build()
    extra = C.CDLL(bench_kernels.LIB)
    for name in sorted(declared):
        assert hasattr(extra, name), name
    assert C.sizeof(C.c_void_p) * 3 + 4 * 6 == bench_kernels.ITEM.itemsize       # bench_gemv_item
    assert bench_kernels.lib().bench_gemv_tasks(9) == 3 and bench_kernels.lib().bench_gemv_tasks(8) == 2
    L = E.lib()
    assert not hasattr(L, "entro_stream_probe") and not hasattr(L, "entro_gemv_u8_plain")


def test_every_declaration_cites_the_passage_that_defines_it():
    """Each exported call's own comment names the section, equation, figure or table of the paper that defines
    what it computes; the two error-reporting calls say that none does, and the entry point that allocates
    nothing names the callers it is for."""
    lines = open(os.path.join(ROOT, "include", "entro.h")).read().split("\n")
    cite = re.compile(r'Eq\. 1|Fig\. [23]|Table [23]|"Huffman weight encoding"|"Segmentation for parallel Huffman decoding"'
                      r'|"Latency Reduction from Huffman Coding"|"Mixed Quantization Scheme"')
    decl = re.compile(r"^(?:entro_status|entro_scheme|uint64_t|uint32_t|double|const char \*)\s*(entro_[a-z0-9_]+)\(")
    comment, in_comment, attached, seen = "", False, False, {}
    for ln in lines:
        if in_comment or ln.lstrip().startswith("/*"):
            if not in_comment:
                comment, in_comment = "", True
            comment += " " + ln.strip().lstrip("/*").strip()
            if "*/" in ln:
                in_comment, attached = False, True
                comment = re.sub(r"\s+", " ", comment.replace("*/", ""))
            continue
        m = decl.match(ln)
        if m:
            assert attached, f"{m.group(1)} has no comment of its own"
            seen[m.group(1)] = comment
        elif ln.strip() == "":
            attached = False                                  # a blank line ends a comment's reach
    assert set(seen) == set(B.EXPORTED), set(B.EXPORTED) ^ set(seen)
    for name, text in seen.items():
        if name in ("entro_status_string", "entro_last_device_error"):
            assert "no passage of the paper defines it" in text, name
        elif name == "entro_decode_gemv_static":
            assert "cannot allocate" in text, name
        else:
            assert cite.search(text), f"{name}: no citation in its comment: {text[:80]}"


def test_struct_layouts_match_header():
    assert C.sizeof(B.QParams) == 16
    assert C.sizeof(B.Codebook) == 16 + 256 + 1024
    assert C.sizeof(B.CTensor) == 8 + 8 + 8 + 8 + 16 + 8 + 16 + 8 + 8 + 8
    assert C.sizeof(B.Plan) == 16 + 32 + 8 + 32


@pytest.mark.parametrize("bits,scheme", [(8, 1), (8, 0), (4, 1), (4, 0)])
def test_quantize_matches_oracle(bits, scheme):
    rng = np.random.default_rng(100 + bits + scheme)
    w = (rng.standard_t(4, 300001) * 0.02).astype(np.float32)
    if scheme == 0:
        w = np.abs(w)
    q, qp = E.entro_quantize(w, bits, scheme)
    qo, s, z = oracle.quantize(w, bits, scheme)
    assert np.array_equal(q, qo) and qp.scale == s and qp.zero_point == z
    assert qp.bits == bits and qp.scheme == scheme


def test_quantize_handworked_and_errors():
    for line in [ln.strip() for ln in open(os.path.join(GOLDEN, "handworked_quant.txt")) if ln.strip() and ln[0] != "#"]:
        head, wtxt, stxt, ztxt, qtxt = [p.strip() for p in line.split("|")]
        scheme = E.ENTRO_ASYMMETRIC if head.split()[0] == "asymmetric" else E.ENTRO_UNSIGNED
        w = np.array([float(v) for v in wtxt.split()], np.float32)
        q, qp = E.entro_quantize(w, int(head.split()[1]), scheme)
        num, den = stxt.split("/")
        assert qp.scale == np.float32(num) / np.float32(den) and qp.zero_point == int(ztxt)
        assert q.tolist() == [int(v) for v in qtxt.split()]
    for w, bits, scheme, status in [
        (np.array([1, np.inf], np.float32), 8, 1, B.ENTRO_ERR_NONFINITE),
        (np.array([1, -1], np.float32), 8, 0, B.ENTRO_ERR_RANGE),
        (np.array([2, 2, 2], np.float32), 8, 1, B.ENTRO_ERR_RANGE),
        (np.array([0, 0], np.float32), 4, 0, B.ENTRO_ERR_RANGE),
        (np.array([1, 2], np.float32), 3, 1, B.ENTRO_ERR_BITS),
        (np.array([1, 2], np.float32), 8, 7, B.ENTRO_ERR_SCHEME),
    ]:
        with pytest.raises(E.EntroError) as e:
            E.entro_quantize(w, bits, scheme)
        assert e.value.status == status


def _kraft(ln):
    return sum(Fraction(1, 2 ** int(v)) for v in ln if v)


@pytest.mark.parametrize("bits", [4, 8])
def test_codebook_cost_equals_oracle_and_is_canonical(bits):
    rng = np.random.default_rng(bits)
    A = 1 << bits
    for trial in range(30):
        kind = trial % 4
        if kind == 0:
            cnt = rng.integers(0, 1000, A)
        elif kind == 1:
            cnt = rng.integers(0, 3, A)                                  # ties and absent symbols
        elif kind == 2:
            cnt = (rng.pareto(0.7, A) * 5).astype(np.int64)              # heavy tail
        else:
            cnt = np.zeros(A, np.int64)
            cnt[rng.integers(0, A, 3)] = rng.integers(1, 9, 3)
        if cnt.sum() == 0:
            cnt[0] = 1
        cb = E.entro_codebook_from_counts(cnt.astype(np.uint64), bits)
        ln = cb.lengths()
        lo = oracle.huffman_lengths(cnt)
        assert int(np.sum(cnt * ln.astype(np.int64))) == int(np.sum(cnt * lo.astype(np.int64)))
        assert np.array_equal(ln > 0, cnt > 0)
        present = int((cnt > 0).sum())
        assert _kraft(ln) == (1 if present > 1 else Fraction(1, 2))
        assert cb.n_used == present and cb.max_len == ln.max()
        assert np.array_equal(cb.codes(), oracle.canonical_codes(ln))    # same canonical rule
        assert np.array_equal(E.entro_codebook_from_lengths(ln, bits).codes(), cb.codes())


def test_codebook_brute_force_tiny_alphabets():
    rng = np.random.default_rng(77)
    for m in range(2, 8):
        for _ in range(6):
            cnt = np.zeros(16, np.uint64)
            cnt[:m] = rng.integers(1, 40, m)
            cb = E.entro_codebook_from_counts(cnt, 4)
            cost = int(np.sum(cnt[:m].astype(np.int64) * cb.lengths()[:m].astype(np.int64)))
            assert cost == oracle.bruteforce_min_cost(cnt[:m])


def test_codebook_limits():
    fib = [1, 1]
    while len(fib) < 40:
        fib.append(fib[-1] + fib[-2])
    cnt = np.zeros(256, np.uint64)
    cnt[:33] = fib[:33]
    assert E.entro_codebook_from_counts(cnt, 8).max_len == 32
    cnt[:34] = fib[:34]
    with pytest.raises(E.EntroError) as e:
        E.entro_codebook_from_counts(cnt, 8)
    assert e.value.status == B.ENTRO_ERR_CODE_TOO_LONG
    with pytest.raises(E.EntroError) as e:                               # Kraft sum above 1
        E.entro_codebook_from_lengths(np.array([1, 1, 1] + [0] * 13, np.uint8), 4)
    assert e.value.status == B.ENTRO_ERR_CORRUPT
    with pytest.raises(E.EntroError) as e:                               # symbol 16 in a 4-bit tensor
        E.entro_build_codebook(np.array([1, 16], np.uint8), 4)
    assert e.value.status == B.ENTRO_ERR_SYMBOL


@pytest.mark.parametrize("bits", [4, 8])
def test_limited_codebook_cost_equals_oracle(bits):
    # package-merge in the library against the oracle's minimisation over the Kraft budget: the cost is
    # unique, the length vector is not
    rng = np.random.default_rng(40 + bits)
    A = 1 << bits
    for trial in range(16):
        kind = trial % 4
        if kind == 0:
            cnt = rng.integers(0, 1000, A)
        elif kind == 1:
            cnt = rng.integers(0, 3, A)
        elif kind == 2:
            cnt = (rng.pareto(0.7, A) * 5).astype(np.int64)
        else:
            cnt = (2.0 ** rng.integers(0, 30, A)).astype(np.int64)
        if cnt.sum() == 0:
            cnt[0] = 1
        present = int((cnt > 0).sum())
        lo = max(1, int(np.ceil(np.log2(present)))) if present > 1 else 1
        for L in sorted({lo, lo + 1, 9, 12, 14, 16}):
            if L < lo:
                continue
            cb = E.entro_codebook_from_counts_limited(cnt.astype(np.uint64), bits, L)
            ln = cb.lengths()
            _, ocost = oracle.limited_lengths(cnt, L)
            assert int(np.sum(cnt * ln.astype(np.int64))) == ocost, (trial, L)
            assert ln.max() <= L and np.array_equal(ln > 0, cnt > 0)
            assert _kraft(ln) <= 1 and cb.max_len == ln.max() and cb.n_used == present
            assert np.array_equal(cb.codes(), oracle.canonical_codes(ln))
    # a generous limit gives the unrestricted optimum; from symbols as from counts
    q = np.minimum(rng.geometric(0.2, 50000) - 1, A - 1).astype(np.uint8)
    cnt = np.bincount(q, minlength=A)
    free = E.entro_build_codebook(q, bits)
    lim = E.entro_build_codebook_limited(q, bits, 32)
    assert int(np.sum(cnt * lim.lengths().astype(np.int64))) == int(np.sum(cnt * free.lengths().astype(np.int64)))
    tight = E.entro_build_codebook_limited(q, bits, bits + 1)
    assert tight.max_len <= bits + 1
    assert np.array_equal(tight.lengths(), E.entro_codebook_from_counts_limited(cnt.astype(np.uint64), bits, bits + 1).lengths())
    # errors: more symbols than codes, limits outside 1..32
    with pytest.raises(E.EntroError) as e:
        E.entro_codebook_from_counts_limited(np.ones(A, np.uint64), bits, bits - 1)
    assert e.value.status == B.ENTRO_ERR_CODE_TOO_LONG
    for bad in (0, 33):
        with pytest.raises(E.EntroError):
            E.entro_codebook_from_counts_limited(np.ones(A, np.uint64), bits, bad)


@pytest.mark.parametrize("bits", [4, 8])
def test_encode_equals_oracle_bit_for_bit(bits):
    for name, sym, chunk in synth.adversarial_symbol_cases(bits):
        cb = E.entro_build_codebook(sym, bits)
        stream, off = E.entro_encode(sym, cb, chunk)
        so, oo = oracle.encode(sym, cb.lengths(), cb.codes(), chunk)
        assert np.array_equal(off, oo), name
        assert np.array_equal(stream, so), name
        assert np.array_equal(oracle.decode(stream, off, sym.size, chunk, cb.lengths(), cb.codes()), sym), name
        assert E.entro_check_offsets(off, sym.size, chunk, stream.size, cb) == 0, name
        assert stream.size <= E.entro_encode_bound(sym.size, cb)


def test_encode_threaded_equals_single_thread(monkeypatch):
    rng = np.random.default_rng(8)
    sym = np.minimum(rng.geometric(0.35, 3_000_000) - 1, 255).astype(np.uint8)
    cb = E.entro_build_codebook(sym, 8)
    monkeypatch.setenv("ENTRO_HOST_THREADS", "1")
    s1, o1 = E.entro_encode(sym, cb, 4096)
    monkeypatch.setenv("ENTRO_HOST_THREADS", "7")
    s7, o7 = E.entro_encode(sym, cb, 4096)
    assert np.array_equal(s1, s7) and np.array_equal(o1, o7)
    assert np.array_equal(oracle.decode(s7, o7, sym.size, 4096, cb.lengths(), cb.codes()), sym)


def test_encode_errors():
    sym = np.array([0, 1, 2, 1], np.uint8)
    cb = E.entro_build_codebook(np.array([0, 1, 1], np.uint8), 8)
    with pytest.raises(E.EntroError) as e:
        E.entro_encode(sym, cb, 4)
    assert e.value.status == B.ENTRO_ERR_SYMBOL
    L = E.lib()
    good = np.array([0, 1, 1, 0], np.uint8)
    small = np.zeros(8, np.uint8)
    off = np.zeros(2, np.uint64)
    nb = C.c_uint64()
    st = L.entro_encode(good.ctypes.data_as(C.POINTER(C.c_uint8)), 4, C.byref(cb), 4,
                        small.ctypes.data_as(C.POINTER(C.c_uint8)), small.size, C.byref(nb),
                        off.ctypes.data_as(C.POINTER(C.c_uint64)))
    assert st == B.ENTRO_ERR_CAPACITY
    st = L.entro_encode(None, 4, C.byref(cb), 4, small.ctypes.data_as(C.POINTER(C.c_uint8)), small.size,
                        C.byref(nb), off.ctypes.data_as(C.POINTER(C.c_uint64)))
    assert st == B.ENTRO_ERR_NULL
    assert E.entro_num_chunks(10, 0) == 0 and E.entro_num_chunks(10, 3) == 4


@pytest.mark.parametrize("bits,chunk,sub,n", [(8, 4096, 256, 3 * 4096 + 700), (8, 1024, 1024, 5000), (4, 8192, 512, 40000),
                                              (8, 512, 32, 2049)])
def test_sub_index_equals_oracle(bits, chunk, sub, n):
    rng = np.random.default_rng(bits * 1000 + sub)
    sym = np.minimum(rng.geometric(0.3, n) - 1, (1 << bits) - 1).astype(np.uint8)
    cb = E.entro_build_codebook(sym, bits)
    got = E.entro_sub_index(sym, cb, chunk, sub)
    assert np.array_equal(got, oracle.sub_index(sym, cb.lengths(), chunk, sub))
    # the pieces of a segment add up to the segment
    _, off = E.entro_encode(sym, cb, chunk)
    per = chunk // sub
    for c in range(off.size - 1):
        assert int(got[c * per:(c + 1) * per].astype(np.uint64).sum()) == int(off[c + 1] - off[c])


def test_sub_index_errors():
    sym = np.zeros(4096, np.uint8)
    cb = E.entro_build_codebook(np.array([0, 1, 1, 1], np.uint8), 8)
    L = E.lib()
    out = np.zeros(64, np.uint16)
    args = (sym.ctypes.data_as(C.POINTER(C.c_uint8)), sym.size, C.byref(cb))
    po = out.ctypes.data_as(C.POINTER(C.c_uint16))
    assert L.entro_sub_index(*args, 4096, 96, po) == B.ENTRO_ERR_SIZE          # not a divisor
    assert L.entro_sub_index(*args, 4096, 128, po) == B.ENTRO_ERR_SIZE         # 32 pieces per segment: more than 16
    assert L.entro_sub_index(*args, 3072, 1024, po) == B.ENTRO_ERR_SIZE        # 3 pieces: not a power of two
    assert L.entro_sub_index(None, sym.size, C.byref(cb), 4096, 256, po) == B.ENTRO_ERR_NULL
    bad = np.full(4096, 7, np.uint8)                                           # a symbol without a code
    assert L.entro_sub_index(bad.ctypes.data_as(C.POINTER(C.c_uint8)), bad.size, C.byref(cb), 4096, 256, po) \
        == B.ENTRO_ERR_SYMBOL
    assert L.entro_sub_index(*args, 4096, 256, po) == B.ENTRO_OK


def test_check_offsets_flags_corruption():
    rng = np.random.default_rng(1)
    sym = rng.integers(0, 7, 20000).astype(np.uint8)
    cb = E.entro_build_codebook(sym, 8)
    stream, off = E.entro_encode(sym, cb, 1024)
    ok = lambda o, nbytes=stream.size: E.entro_check_offsets(o, sym.size, 1024, nbytes, cb)
    assert ok(off) == 0
    bad = off.copy(); bad[3], bad[4] = bad[4], bad[3]
    assert ok(bad) == B.ENTRO_ERR_CORRUPT                                # non-monotone
    bad = off.copy(); bad[-1] = stream.size * 8 + 5
    assert ok(bad) == B.ENTRO_ERR_CORRUPT                                # beyond the stream
    bad = off.copy(); bad[0] = 1
    assert ok(bad) == B.ENTRO_ERR_CORRUPT
    bad = off.copy(); bad[5:] += 1024 * 40
    assert ok(bad) == B.ENTRO_ERR_CORRUPT                                # a segment longer than possible
    assert ok(off, stream.size - 16) == B.ENTRO_ERR_CORRUPT              # truncated stream


def test_reporting_matches_paper_values():
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "paper_effective_bits.txt")) if ln[0] != "#" and ln.strip()]
    for bits, eff, saved, speed, less in rows:
        assert round(E.entro_bits_saved(int(bits), float(eff)), 2) == float(saved)
        if speed != "-":
            assert round(E.entro_theoretical_speedup(int(bits), float(eff)), 2) == float(speed)
            assert round(1 - float(eff) / int(bits), 2) == float(less)


def test_device_entry_points_validate_before_touching_the_gpu():
    """Argument errors are detected on the host; no GPU is needed to see them."""
    sym = np.arange(16, dtype=np.uint8).repeat(4)
    cb = E.entro_build_codebook(sym, 4)
    t = B.CTensor()
    L = E.lib()
    assert L.entro_decode(None, E.ENTRO_U8, None) == B.ENTRO_ERR_NULL
    assert L.entro_decode(C.byref(t), E.ENTRO_U8, None) == B.ENTRO_ERR_NULL          # null buffers
    t.stream, t.offsets, t.out = 4096, 8192, 12288                                   # fake aligned addresses
    t.cb = C.pointer(cb)
    t.n, t.chunk_symbols, t.stream_bytes = 64, 32, 64
    assert L.entro_decode(C.byref(t), E.ENTRO_F32, None) == B.ENTRO_ERR_SCHEME        # wrong type for the call
    assert L.entro_decode_dequant(C.byref(t), E.ENTRO_U8, None) == B.ENTRO_ERR_SCHEME
    t.chunk_symbols = 31
    assert L.entro_decode(C.byref(t), E.ENTRO_U4_PACKED, None) == B.ENTRO_ERR_SIZE    # odd chunk, packed output
    t.chunk_symbols = 32
    t.stream_bytes = 40
    assert L.entro_decode(C.byref(t), E.ENTRO_U8, None) == B.ENTRO_ERR_SIZE           # not a padded size
    t.stream_bytes = 64
    t.out = 12289
    assert L.entro_decode(C.byref(t), E.ENTRO_U8, None) == B.ENTRO_ERR_ALIGN
    t.out = 12288
    t.qp.bits = 8
    assert L.entro_decode_dequant(C.byref(t), E.ENTRO_F32, None) == B.ENTRO_ERR_BITS  # qparams for another width
    t.qp.bits = 4
    t.rows, t.cols = 3, 16
    t.x = 16384
    assert L.entro_decode_gemv(C.byref(t), E.ENTRO_F32, None, 0, None) == B.ENTRO_ERR_SIZE   # rows*cols != n
    bad = B.Codebook.from_buffer_copy(cb)
    bad.code[3] ^= 1
    t.cb = C.pointer(bad)
    assert L.entro_decode(C.byref(t), E.ENTRO_U8, None) == B.ENTRO_ERR_CORRUPT        # codes not canonical
    t.cb = C.pointer(cb)
    t.sub_symbols = 16                                                                # entry points announced, table missing
    assert L.entro_decode(C.byref(t), E.ENTRO_U8, None) == B.ENTRO_ERR_NULL
    t.sub_bits = 20480
    t.sub_symbols = 12
    assert L.entro_decode(C.byref(t), E.ENTRO_U8, None) == B.ENTRO_ERR_SIZE           # segments are not whole pieces
    t.sub_symbols = 1
    assert L.entro_decode(C.byref(t), E.ENTRO_U8, None) == B.ENTRO_ERR_SIZE           # 32 pieces per segment
    t.sub_symbols, t.sub_bits = 0, None
    ws1 = L.entro_workspace_bytes(C.byref(t), 1, E.ENTRO_OP_DECODE)
    st1 = L.entro_plan_staging_bytes(C.byref(t), 1, E.ENTRO_OP_DECODE)
    # the workspace holds what is staged on the host (descriptors, work list) and, behind it, room for the
    # tensor's lookup tables (the wider kind: 2^14 entries of four bytes and the side tables)
    assert 0 < st1 < ws1 and ws1 - st1 >= (1 << 14) * 4 and ws1 % 256 == 0
    two = (B.CTensor * 2)(t, t)
    assert L.entro_workspace_bytes(two, 2, E.ENTRO_OP_DECODE) - ws1 >= (1 << 14) * 4
    plan = B.Plan()
    assert L.entro_plan_init(C.byref(plan), C.byref(t), 1, E.ENTRO_OP_DECODE, E.ENTRO_U8, 4096, 16, None) \
        == B.ENTRO_ERR_CAPACITY
    assert L.entro_plan_run(C.byref(B.Plan()), None) == B.ENTRO_ERR_NULL


@pytest.mark.parametrize("bits,scheme", [(8, 1), (8, 0), (4, 1), (4, 0)])
def test_qparams_from_range_is_the_quantizer_s_first_half(bits, scheme):
    rng = np.random.default_rng(7 + bits + scheme)
    w = (rng.standard_t(4, 20001) * 0.02).astype(np.float32)
    if scheme == 0:
        w = np.abs(w)
    _, s, z = oracle.quantize(w, bits, scheme)
    qp = E.entro_qparams_from_range(float(w.min()), float(w.max()), 0, bits, scheme)
    assert np.float32(qp.scale) == s and qp.zero_point == z and qp.bits == bits and qp.scheme == scheme
    for args, status in [
        ((0.0, 1.0, 1, bits, scheme), B.ENTRO_ERR_NONFINITE),
        ((0.0, float("inf"), 0, bits, scheme), B.ENTRO_ERR_NONFINITE),
        ((2.0, 2.0, 0, bits, 1), B.ENTRO_ERR_RANGE),
        ((-1.0, 1.0, 0, bits, 0), B.ENTRO_ERR_RANGE),
        ((0.0, 1.0, 0, 5, scheme), B.ENTRO_ERR_BITS),
        ((0.0, 1.0, 0, bits, 9), B.ENTRO_ERR_SCHEME),
    ]:
        with pytest.raises(E.EntroError) as e:
            E.entro_qparams_from_range(*args)
        assert e.value.status == status


def test_encoded_bytes_is_the_encoder_s_stream_size():
    for name, sym, chunk in synth.adversarial_symbol_cases(8):
        ln, code, cnt = oracle.codebook_from_symbols(sym, 8)
        cb = E.entro_codebook_from_lengths(ln, 8)
        stream, off = oracle.encode(sym, ln, code, chunk)
        assert E.entro_encoded_bytes(cnt, cb) == stream.size == oracle.stream_bytes(int(off[-1])), name
    cnt = np.zeros(256, np.uint64)
    cnt[255] = 1                                                     # a counted symbol without a code
    ln, _, _ = oracle.codebook_from_symbols(np.array([0, 1, 1], np.uint8), 8)
    assert E.entro_encoded_bytes(cnt, E.entro_codebook_from_lengths(ln, 8)) == 0


def test_device_compression_calls_validate_before_touching_the_gpu():
    L = E.lib()
    qp = B.QParams(1.0, 0, 8, 1)
    assert L.entro_range_device(None, 4, 4096, None) == B.ENTRO_ERR_NULL
    assert L.entro_range_device(4096, 0, 8192, None) == B.ENTRO_ERR_SIZE
    assert L.entro_range_device(4100, 4, 8192, None) == B.ENTRO_ERR_ALIGN
    assert L.entro_quantize_device(4096, 4, C.byref(qp), 8192, None, None) == B.ENTRO_ERR_NULL
    assert L.entro_quantize_device(4096, 4, C.byref(B.QParams(1.0, 0, 5, 1)), 8192, 12288, None) == B.ENTRO_ERR_BITS
    assert L.entro_quantize_device(4096, 4, C.byref(B.QParams(0.0, 0, 8, 1)), 8192, 12288, None) == B.ENTRO_ERR_RANGE
    assert L.entro_quantize_device(4096, 4, C.byref(B.QParams(1.0, 1 << 25, 8, 1)), 8192, 12288, None) == B.ENTRO_ERR_RANGE
    assert L.entro_quantize_device(4096, 4, C.byref(qp), 8193, 12288, None) == B.ENTRO_ERR_ALIGN
    sym = np.arange(16, dtype=np.uint8).repeat(4)
    cb = E.entro_build_codebook(sym, 4)
    assert L.entro_encode_device(4096, 64, C.byref(cb), 32, 8192, 64, 12288, None, None) == B.ENTRO_ERR_NULL
    assert L.entro_encode_device(4096, 64, C.byref(cb), 0, 8192, 64, 12288, 16384, None) == B.ENTRO_ERR_SIZE
    assert L.entro_encode_device(4096, 64, C.byref(cb), (1 << 20) + 1, 8192, 64, 12288, 16384, None) == B.ENTRO_ERR_SIZE
    assert L.entro_encode_device(4096, 64, C.byref(cb), 32, 8192, 40, 12288, 16384, None) == B.ENTRO_ERR_CAPACITY
    assert L.entro_encode_device(4096, 64, C.byref(cb), 32, 8200, 64, 12288, 16384, None) == B.ENTRO_ERR_ALIGN
    bad = B.Codebook.from_buffer_copy(cb)
    bad.code[3] ^= 1
    assert L.entro_encode_device(4096, 64, C.byref(bad), 32, 8192, 64, 12288, 16384, None) == B.ENTRO_ERR_CORRUPT
    assert [E.entro_encode_device_status(v) for v in (0, 1, 2, 4, 3)] == \
        [B.ENTRO_OK, B.ENTRO_ERR_SYMBOL, B.ENTRO_ERR_CAPACITY, B.ENTRO_ERR_SIZE, B.ENTRO_ERR_SYMBOL]


def test_scheme_for_range_takes_the_unsigned_grid_only_where_it_can_hold_the_tensor():
    assert E.entro_scheme_for_range(0.8, 1.2) == E.ENTRO_UNSIGNED          # norm gains
    assert E.entro_scheme_for_range(0.0, 1.0) == E.ENTRO_UNSIGNED
    assert E.entro_scheme_for_range(-0.0, 1.0) == E.ENTRO_UNSIGNED
    assert E.entro_scheme_for_range(-1e-30, 1.0) == E.ENTRO_ASYMMETRIC
    assert E.entro_scheme_for_range(-3.0, -1.0) == E.ENTRO_ASYMMETRIC
    # whatever it picks, the quantizer accepts the tensor
    for w in (np.array([0.8, 1.0, 1.2], np.float32), np.array([-1, 0.5, 2], np.float32)):
        sch = E.entro_scheme_for_range(float(w.min()), float(w.max()))
        q, qp = E.entro_quantize(w, 8, sch)
        qo, s, z = oracle.quantize(w, 8, sch)
        assert np.array_equal(q, qo) and qp.scheme == sch
