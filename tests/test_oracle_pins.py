"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself -- hand-worked values, closed forms, invariants, brute force
on tiny alphabets, or a library routine the step reduces to in a special case.

Paper passages: Eq. 1 / Fig. 2 (quantisation grids), "Huffman weight encoding"
(optimal prefix code), Introduction (alignment with the Shannon bounds,
lossless recovery), "Segmentation for parallel Huffman decoding" (segments
decode independently from known boundaries).
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


# ------------------------------------------------------------------ quantize
def test_quantize_handworked_grids():
    for line in _lines("handworked_quant.txt"):
        head, wtxt, stxt, ztxt, qtxt = [p.strip() for p in line.split("|")]
        scheme_name, bits = head.split()
        scheme = oracle.ASYMMETRIC if scheme_name == "asymmetric" else oracle.UNSIGNED
        w = np.array([float(v) for v in wtxt.split()], np.float32)
        num, den = stxt.split("/")
        q, s, z = oracle.quantize(w, int(bits), scheme)
        assert s == np.float32(np.float32(num) / np.float32(den)), line
        assert z == int(ztxt), line
        assert q.tolist() == [int(v) for v in qtxt.split()], line


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("scheme", [oracle.ASYMMETRIC, oracle.UNSIGNED])
def test_quantize_invariants_and_library_one_liner(bits, scheme):
    rng = np.random.default_rng(11 + bits + scheme)
    w = (rng.standard_t(4, 20000) * 0.02).astype(np.float32)
    if scheme == oracle.UNSIGNED:
        w = np.abs(w)
    Q = (1 << bits) - 1
    q, s, z = oracle.quantize(w, bits, scheme)
    # closed forms, evaluated exactly and then rounded to binary32 once per operation
    lo, hi = Fraction(float(w.min())), Fraction(float(w.max()))
    if scheme == oracle.ASYMMETRIC:
        rng32 = np.float32(float(hi - lo))               # one rounding: the subtraction
        s_ref = np.float32(float(Fraction(float(rng32)) / Q))
        z_ref = int(np.rint(np.float32(float(Fraction(float(-w.min())) / Fraction(float(s_ref))))))
    else:
        s_ref = np.float32(float(hi / Q))
        z_ref = 0
    assert s == s_ref and z == z_ref
    assert q.min() >= 0 and q.max() <= Q
    assert q[np.argmax(w)] == Q
    assert q[np.argmin(w)] == (0 if scheme == oracle.ASYMMETRIC else int(np.rint(w.min() / s)))
    # the step reduces to numpy's rint / clip
    lib = np.clip(np.rint(w / s).astype(np.int64) + z, 0, Q)
    assert np.array_equal(q, lib.astype(np.uint8))
    # reconstruction error at most half a step for every unclamped element
    rec = (q.astype(np.float64) - z) * float(s)
    unclamped = (q > 0) & (q < Q)
    assert np.all(np.abs(rec - w)[unclamped] <= 0.5 * float(s) * (1 + 1e-5))


def test_quantize_errors():
    with pytest.raises(oracle.OracleError) as e:
        oracle.quantize(np.array([1.0, np.nan], np.float32), 8, oracle.ASYMMETRIC)
    assert e.value.code == oracle.ERR_NONFINITE
    with pytest.raises(oracle.OracleError) as e:
        oracle.quantize(np.array([1.0, -0.5], np.float32), 8, oracle.UNSIGNED)
    assert e.value.code == oracle.ERR_RANGE
    with pytest.raises(oracle.OracleError) as e:
        oracle.quantize(np.full(7, 0.25, np.float32), 8, oracle.ASYMMETRIC)
    assert e.value.code == oracle.ERR_RANGE
    with pytest.raises(oracle.OracleError):
        oracle.quantize(np.ones(4, np.float32), 5, oracle.ASYMMETRIC)


def test_quantize_zero_point_may_leave_grid():
    # all-positive tensor under the asymmetric scheme: z = round(-min/s) < 0
    w = np.array([1.0, 1.5, 2.0], np.float32)
    q, s, z = oracle.quantize(w, 8, oracle.ASYMMETRIC)
    # 1.5 / fl32(1/255) is 382.49998 in binary32 (fl32(1/255) lies above 1/255), so it rounds to 382
    mid = int(np.rint(np.float32(float(Fraction(1.5) / Fraction(float(s)))))) + z
    assert s == np.float32(1.0) / np.float32(255.0) and z == -255 and mid == 127
    assert q.tolist() == [0, 127, 255]


# ----------------------------------------------------------- Huffman lengths
def _kraft_exact(ln):
    present = [int(v) for v in ln if v > 0]
    return sum(Fraction(1, 2 ** v) for v in present)


def _py_bruteforce(cnt):
    m = len(cnt)
    if m == 1:
        return cnt[0]
    best = None
    for lens in itertools.product(range(1, m), repeat=m):
        if sum(Fraction(1, 2 ** v) for v in lens) <= 1:
            c = sum(a * b for a, b in zip(cnt, lens))
            best = c if best is None or c < best else best
    return best


def test_huffman_is_optimal_by_brute_force():
    rng = np.random.default_rng(5)
    for m in range(2, 7):
        for trial in range(12 if m < 6 else 4):
            kind = trial % 3
            if kind == 0:
                cnt = rng.integers(1, 50, m)
            elif kind == 1:
                cnt = rng.integers(1, 4, m)              # many ties
            else:
                cnt = (2.0 ** rng.integers(0, 12, m)).astype(np.int64)
            ln = oracle.huffman_lengths(cnt)
            cost = int(np.sum(cnt * ln.astype(np.int64)))
            assert cost == _py_bruteforce([int(c) for c in cnt]), (cnt, ln)
            assert oracle.bruteforce_min_cost(cnt) == cost
            assert _kraft_exact(ln) == 1


def test_c_bruteforce_matches_python_bruteforce_at_7_and_8_symbols():
    rng = np.random.default_rng(6)
    cnt = rng.integers(1, 30, 7)
    assert oracle.bruteforce_min_cost(cnt) == _py_bruteforce([int(c) for c in cnt])
    for _ in range(5):
        cnt = rng.integers(1, 100, 8)
        ln = oracle.huffman_lengths(cnt)
        assert oracle.bruteforce_min_cost(cnt) == int(np.sum(cnt * ln.astype(np.int64)))


# ------------------------------------------------- length-limited codes (extension)
def _py_bruteforce_limited(cnt, max_len):
    m = len(cnt)
    if m == 1:
        return cnt[0]
    best = None
    for lens in itertools.product(range(1, max_len + 1), repeat=m):
        if sum(Fraction(1, 2 ** v) for v in lens) <= 1:
            c = sum(a * b for a, b in zip(cnt, lens))
            best = c if best is None or c < best else best
    return best


def test_limited_lengths_are_optimal_by_brute_force():
    # every length vector up to the limit that satisfies Kraft's inequality, enumerated in Python;
    # the C enumeration for the larger cases is itself checked against the Python one first
    rng = np.random.default_rng(15)
    for m in range(2, 7):
        for trial in range(6):
            cnt = rng.integers(1, 60, m) if trial % 2 else (2.0 ** rng.integers(0, 10, m)).astype(np.int64)
            lo = max(1, math.ceil(math.log2(m)))
            for L in range(lo, min(lo + 3, 5) + 1):
                ln, cost = oracle.limited_lengths(cnt, L)
                assert cost == int(np.sum(cnt * ln.astype(np.int64)))
                assert ln.max() <= L and ln.min() >= 1 and _kraft_exact(ln) <= 1
                assert cost == _py_bruteforce_limited([int(c) for c in cnt], L), (cnt, L, ln)
                assert cost == oracle.bruteforce_min_cost_limited(cnt, L)
    for _ in range(4):
        cnt = rng.integers(1, 1000, 8)
        for L in (3, 4, 6):
            assert oracle.limited_lengths(cnt, L)[1] == oracle.bruteforce_min_cost_limited(cnt, L)


def test_limited_lengths_closed_forms():
    # the example of the dyadic pin: {4,2,1,1} wants lengths {1,2,3,3} (cost 14); limited to 2 bits all four
    # symbols get 2 (cost 16)
    ln, cost = oracle.limited_lengths(np.array([4, 2, 1, 1]), 3)
    assert ln.tolist() == [1, 2, 3, 3] and cost == 14
    ln, cost = oracle.limited_lengths(np.array([4, 2, 1, 1]), 2)
    assert ln.tolist() == [2, 2, 2, 2] and cost == 16
    # as many symbols as the limit has codes: fixed width, whatever the counts
    rng = np.random.default_rng(16)
    for k in (1, 3, 5, 8):
        cnt = rng.integers(1, 10 ** 6, 2 ** k)
        ln, cost = oracle.limited_lengths(cnt, k)
        assert set(ln.tolist()) == {k} and cost == k * int(cnt.sum())
    # more symbols than codes: refused
    with pytest.raises(oracle.OracleError):
        oracle.limited_lengths(np.ones(9, np.int64), 3)
    # absent symbols get no code, a lone symbol one bit
    ln, _ = oracle.limited_lengths(np.array([0, 7, 0, 0]), 5)
    assert ln.tolist() == [0, 1, 0, 0]


def test_limited_lengths_against_unrestricted_huffman():
    # a limit at or above the longest Huffman code changes nothing (same cost); a tighter one costs more,
    # the more the tighter; the cost never drops below the entropy bound
    rng = np.random.default_rng(17)
    for trial in range(6):
        m = int(rng.integers(20, 257))
        cnt = np.zeros(256, np.int64)
        cnt[:m] = (rng.pareto(0.8, m) * 50 + 1).astype(np.int64)
        hl = oracle.huffman_lengths(cnt)
        hcost = int(np.sum(cnt * hl.astype(np.int64)))
        hmax = int(hl.max())
        prev = None
        for L in range(min(hmax, 16), 7, -1):
            ln, cost = oracle.limited_lengths(cnt, L)
            assert ln.max() <= L and _kraft_exact(ln) <= 1 and np.all((ln > 0) == (cnt > 0))
            if L >= hmax:
                assert cost == hcost
            else:
                assert cost >= hcost
            if prev is not None:
                assert cost >= prev
            prev = cost
        n = int(cnt.sum())
        H = -sum(c / n * math.log2(c / n) for c in cnt[cnt > 0])
        assert prev / n >= H - 1e-9


def test_huffman_dyadic_counts_hit_entropy_exactly():
    for k in range(1, 12):
        cnt = [2 ** (k - 1 - i) for i in range(k)] + [1]           # {2^(k-1),...,2,1,1}
        ln = oracle.huffman_lengths(np.array(cnt))
        assert sorted(ln.tolist()) == sorted(list(range(1, k + 1)) + [k])
        assert ln.tolist() == list(range(1, k + 1)) + [k]
        n = sum(cnt)
        H = -sum(c / n * math.log2(c / n) for c in cnt)
        Lbar = sum(c * l for c, l in zip(cnt, ln.tolist())) / n
        assert abs(H - Lbar) < 1e-12


def test_huffman_uniform_counts_give_fixed_width():
    for k in range(1, 9):
        ln = oracle.huffman_lengths(np.full(2 ** k, 7))
        assert np.all(ln == k)


def test_huffman_absent_and_single_symbols():
    cnt = np.zeros(256, np.uint64)
    cnt[17] = 5
    ln = oracle.huffman_lengths(cnt)
    assert ln[17] == 1 and ln.sum() == 1                 # lone symbol: one bit, Kraft sum 1/2
    cnt[200] = 1
    ln = oracle.huffman_lengths(cnt)
    assert ln[17] == 1 and ln[200] == 1 and ln.sum() == 2
    with pytest.raises(oracle.OracleError):
        oracle.huffman_lengths(np.zeros(16, np.uint64))


def test_huffman_fibonacci_depth_and_length_cap():
    fib = [1, 1]
    while len(fib) < 35:
        fib.append(fib[-1] + fib[-2])
    ln = oracle.huffman_lengths(np.array(fib[:33]))      # 33 symbols -> deepest leaf 32
    assert ln.max() == 32 and _kraft_exact(ln) == 1
    with pytest.raises(oracle.OracleError) as e:
        oracle.huffman_lengths(np.array(fib[:34]))       # would need a 33-bit code
    assert e.value.code == oracle.ERR_TOO_LONG


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_entropy_bounds_and_kraft_on_config_shaped_tensors(cfg):
    spec = synth.config_tensors(cfg)[0]
    # a 1M-element slice of the real generator keeps the CPU suite short
    small = synth.TensorSpec(**{**spec.__dict__, "rows": 512, "cols": 2048})
    w = synth.make_tensor(small)
    q, s, z = oracle.quantize(w, small.bits, small.scheme)
    ln, code, cnt = oracle.codebook_from_symbols(q, small.bits)
    n = q.size
    p = cnt[cnt > 0].astype(np.float64) / n
    H = float(-(p * np.log2(p)).sum())
    Lbar = float(np.sum(cnt.astype(np.float64) * ln)) / n
    assert H <= Lbar + 1e-12 and Lbar < H + 1
    assert _kraft_exact(ln) == 1
    # sibling property: the two rarest present symbols share the maximal length
    present = np.flatnonzero(cnt)
    order = present[np.argsort(cnt[present], kind="stable")]
    assert ln[order[0]] == ln.max()
    assert np.sum(ln == ln.max()) >= 2
    # more frequent never longer
    for a, b in zip(order[:-1], order[1:]):
        if cnt[a] < cnt[b]:
            assert ln[a] >= ln[b]


# ----------------------------------------------------------- canonical codes
def test_canonical_handworked():
    rows = _lines("handworked_stream.txt")
    ln = np.array([int(v) for v in rows[0].split()], np.uint8)
    want = [int(v, 2) for v in rows[1].split()]
    code = oracle.canonical_codes(ln)
    assert code.tolist() == want


def _bitstr(code, ln):
    return format(int(code), "b").zfill(int(ln))


def test_canonical_prefix_free_and_consecutive():
    rng = np.random.default_rng(9)
    cnt = rng.integers(0, 1000, 256) * (rng.random(256) < 0.6)
    cnt[3] = 10 ** 6
    ln = oracle.huffman_lengths(cnt)
    code = oracle.canonical_codes(ln)
    words = {s: _bitstr(code[s], ln[s]) for s in range(256) if ln[s]}
    for a, b in itertools.permutations(words, 2):
        assert not words[b].startswith(words[a])
    for L in range(1, 33):
        syms = [s for s in range(256) if ln[s] == L]
        vals = [int(code[s]) for s in syms]
        assert vals == list(range(vals[0], vals[0] + len(vals))) if vals else True
    # numerically increasing with (length, symbol) when left-justified
    order = sorted(words, key=lambda s: (ln[s], s))
    just = [int(code[s]) << (32 - int(ln[s])) for s in order]
    assert just == sorted(just) and len(set(just)) == len(just)


def test_canonical_rejects_oversubscribed_lengths():
    with pytest.raises(oracle.OracleError):
        oracle.canonical_codes(np.array([1, 1, 1], np.uint8))


# -------------------------------------------------------------------- encode
def test_encode_handworked_stream():
    rows = _lines("handworked_stream.txt")
    ln = np.array([int(v) for v in rows[0].split()], np.uint8)
    code = np.array([int(v, 2) for v in rows[1].split()], np.uint32)
    sym = np.array([int(v) for v in rows[2].split()], np.uint8)
    want_bytes = [int(v, 16) for v in rows[3].split()]
    want_off = [int(v) for v in rows[4].split()]
    stream, off = oracle.encode(sym, ln, code, 2)
    assert stream[:2].tolist() == want_bytes
    assert off.tolist() == want_off
    assert not stream[2:].any() and stream.size == 32 and stream.size % 16 == 0
    assert oracle.decode(stream, off, sym.size, 2, ln, code).tolist() == sym.tolist()


def test_encode_uniform_alphabet_is_plain_bit_packing():
    rng = np.random.default_rng(3)
    for k in (1, 2, 3, 4, 8):
        A = 2 ** k
        sym = np.concatenate([np.arange(A), rng.integers(0, A, 5000)]).astype(np.uint8)
        cnt = np.full(A, 1, np.uint64)                   # force the fixed-width code
        ln = oracle.huffman_lengths(cnt)
        code = oracle.canonical_codes(ln)
        assert code.tolist() == list(range(A))
        stream, off = oracle.encode(sym, ln, code, 512)
        bits = ((sym[:, None] >> np.arange(k - 1, -1, -1)) & 1).astype(np.uint8).ravel()
        packed = np.packbits(bits, bitorder="little")
        assert np.array_equal(stream[: packed.size], packed)
        assert not stream[packed.size:].any()
        assert off.tolist() == [min(i * 512, sym.size) * k for i in range(off.size)]


def test_encode_sizes_offsets_and_padding():
    for name, sym, chunk in synth.adversarial_symbol_cases(8):
        ln, code, cnt = oracle.codebook_from_symbols(sym, 8)
        stream, off = oracle.encode(sym, ln, code, chunk)
        total = int(np.sum(cnt * ln.astype(np.uint64)))
        assert int(off[-1]) == total, name
        per_sym = ln[sym].astype(np.int64)
        starts = np.concatenate([[0], np.cumsum(per_sym)])[::chunk]
        assert off[:-1].tolist() == starts[: off.size - 1].tolist(), name
        assert off.size == -(-sym.size // chunk) + 1
        nbytes = -(-total // 8)
        assert stream.size == -(-nbytes // 16) * 16 + 16 and not stream[nbytes:].any(), name
        if total % 8:
            assert stream[nbytes - 1] >> (total % 8) == 0, name
    with pytest.raises(oracle.OracleError) as e:            # a symbol without a code
        ln = np.array([1, 1, 0, 0], np.uint8)
        oracle.encode(np.array([0, 2], np.uint8), ln, oracle.canonical_codes(ln), 4)
    assert e.value.code == oracle.ERR_SYMBOL


# -------------------------------------------------------------------- decode
@pytest.mark.parametrize("bits", [4, 8])
def test_round_trip_identity_on_adversarial_streams(bits):
    for name, sym, chunk in synth.adversarial_symbol_cases(bits):
        ln, code, _ = oracle.codebook_from_symbols(sym, bits)
        stream, off = oracle.encode(sym, ln, code, chunk)
        out = oracle.decode(stream, off, sym.size, chunk, ln, code)
        assert np.array_equal(out, sym), name
    # the deep case really is deep
    cases = {n: s for n, s, _ in synth.adversarial_symbol_cases(8)}
    ln, _, _ = oracle.codebook_from_symbols(cases["fibonacci_deep"], 8)
    assert ln.max() == 28          # (not 32: the case caps its counts; 32-bit codes come from given lengths elsewhere)


def test_round_trip_identity_config1():
    spec = synth.config_tensors(1)[0]
    w = synth.make_tensor(spec)
    q, s, z = oracle.quantize(w, 8, oracle.ASYMMETRIC)
    ln, code, _ = oracle.codebook_from_symbols(q, 8)
    stream, off = oracle.encode(q, ln, code, 4096)
    assert off.size == 1025
    assert np.array_equal(oracle.decode(stream, off, q.size, 4096, ln, code), q)


def test_segments_decode_independently_and_in_any_order():
    rng = np.random.default_rng(21)
    sym = np.minimum(rng.geometric(0.3, 50000) - 1, 255).astype(np.uint8)
    chunk = 1000
    ln, code, _ = oracle.codebook_from_symbols(sym, 8)
    stream, off = oracle.encode(sym, ln, code, chunk)
    n_chunks = off.size - 1
    out = np.full(sym.size, 255, np.uint8)
    for k in rng.permutation(n_chunks):
        before = out.copy()
        oracle.decode_chunks(stream, off, sym.size, chunk, ln, code, int(k), 1, out)
        lo, hi = k * chunk, min((k + 1) * chunk, sym.size)
        assert np.array_equal(out[lo:hi], sym[lo:hi])
        before[lo:hi] = out[lo:hi]
        assert np.array_equal(before, out)               # nothing else was touched
    assert np.array_equal(out, sym)


# ------------------------------------------------- entry points inside a segment
def test_sub_index_handworked():
    rows = _lines("handworked_sub_index.txt")
    ln = np.array([int(v) for v in rows[0].split()], np.uint8)
    sym = np.array([int(v) for v in rows[1].split()], np.uint8)
    want_bits = [int(v) for v in rows[2].split()]
    want_off = [int(v) for v in rows[3].split()]
    want_starts = [int(v) for v in rows[4].split()]
    code = oracle.canonical_codes(ln)
    stream, off = oracle.encode(sym, ln, code, 4)
    assert off.tolist() == want_off
    sub = oracle.sub_index(sym, ln, 4, 2)
    assert sub.tolist() == want_bits
    starts = [int(off[j // 2]) + int(sub[(j // 2) * 2:j].sum()) for j in range(3)]
    assert starts == want_starts
    for j in range(3):                                   # every piece decodes on its own
        out = oracle.decode_subs(stream, off, sub, sym.size, 4, 2, ln, code, j, 1, np.full(5, 9, np.uint8))
        assert out[2 * j:2 * j + 2].tolist() == sym[2 * j:2 * j + 2].tolist()
        assert (np.delete(out, range(2 * j, min(2 * j + 2, 5))) == 9).all()


@pytest.mark.parametrize("chunk,sub,n", [(4096, 256, 70000), (1024, 64, 10000 + 37), (512, 512, 3000), (96, 32, 1000)])
def test_sub_index_agrees_with_a_finer_segmentation(chunk, sub, n):
    """The entry points of pieces of `sub` symbols are the segment offsets of the same symbols encoded with segments
    of `sub` symbols (a path through encode that does not know of pieces), the pieces of a segment add up to the
    segment, and decoding from the entry points gives the symbols."""
    rng = np.random.default_rng(chunk + sub)
    sym = np.minimum(rng.geometric(0.25, n) - 1, 255).astype(np.uint8)
    ln, code, _ = oracle.codebook_from_symbols(sym, 8)
    stream, off = oracle.encode(sym, ln, code, chunk)
    _, off_fine = oracle.encode(sym, ln, code, sub)
    bits = oracle.sub_index(sym, ln, chunk, sub)
    per = chunk // sub
    n_sub = (n + sub - 1) // sub
    assert bits.size == n_sub
    starts = np.array([int(off[j // per]) + int(bits[(j // per) * per:j].astype(np.uint64).sum()) for j in range(n_sub)])
    assert np.array_equal(starts, off_fine[:-1].astype(np.int64))
    for c in range(off.size - 1):
        assert int(bits[c * per:(c + 1) * per].astype(np.uint64).sum()) == int(off[c + 1] - off[c])
    lens = ln.astype(np.int64)[sym]
    assert bits.tolist() == [int(lens[j * sub:(j + 1) * sub].sum()) for j in range(n_sub)]
    out = np.full(n, 255, np.uint8)
    for j in rng.permutation(n_sub)[:40]:
        oracle.decode_subs(stream, off, bits, n, chunk, sub, ln, code, int(j), 1, out)
        assert np.array_equal(out[j * sub:(j + 1) * sub], sym[j * sub:(j + 1) * sub])
    assert np.array_equal(oracle.decode_subs(stream, off, bits, n, chunk, sub, ln, code, 0, n_sub), sym)


def test_sub_index_errors():
    sym = np.zeros(100, np.uint8)
    ln = np.zeros(256, np.uint8)
    ln[0] = 1
    with pytest.raises(oracle.OracleError):
        oracle.sub_index(sym, ln, 48, 32)                # segments are not a whole number of pieces
    ln32 = np.zeros(256, np.uint8)
    ln32[:2] = [1, 32]
    with pytest.raises(oracle.OracleError) as e:         # 2048 codes of 32 bits do not fit a 16-bit entry
        oracle.sub_index(np.ones(4096, np.uint8), ln32, 4096, 2048)
    assert e.value.code == oracle.ERR_TOO_LONG


def test_histogram_is_a_bincount():
    rng = np.random.default_rng(8)
    for bits in (8, 4):
        q = rng.integers(0, 1 << bits, 100001).astype(np.uint8)
        q[q == 3] = 5                                    # an absent symbol
        assert np.array_equal(oracle.histogram(q, bits), np.bincount(q, minlength=1 << bits).astype(np.uint64))
    with pytest.raises(oracle.OracleError):
        oracle.histogram(np.array([16], np.uint8), 4)


def test_pack_u4_layout():
    q = np.array([1, 2, 3, 4, 15], np.uint8)
    assert oracle.pack_u4(q).tolist() == [0x21, 0x43, 0x0F]
    rng = np.random.default_rng(2)
    q = rng.integers(0, 16, 1001).astype(np.uint8)
    p = oracle.pack_u4(q)
    assert np.array_equal(p[:500] & 15, q[0:1000:2]) and np.array_equal(p[:500] >> 4, q[1:1000:2])
    assert p[500] == q[1000]


# ------------------------------------------------------------------- dequant
def test_dequant_closed_forms_and_library_routines():
    s, z = np.float32(0.0123456), 143
    q = np.arange(256, dtype=np.uint8)
    f = oracle.dequant_f32(q, s, z)
    assert f[z] == 0.0 and not np.signbit(f[z])
    assert np.array_equal(f, (q.astype(np.int32) - z).astype(np.float32) * s)     # numpy binary32 product
    exact = [Fraction(int(v) - z) * Fraction(float(s)) for v in q]
    assert all(np.float32(float(e)) == v for e, v in zip(exact, f))               # single correct rounding
    assert np.unique(f).size == 256
    b = oracle.dequant_bf16(q, s, z)
    t = torch.from_numpy(f.copy()).bfloat16().view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(b, t)
    # z outside the grid
    f2 = oracle.dequant_f32(np.array([0, 255], np.uint8), np.float32(0.5), -255)
    assert f2.tolist() == [127.5, 255.0]


def test_bf16_round_half_even():
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1.0 and 1+2^-7: ties to even -> 1.0
    s = np.float32(1.0 + 2.0 ** -8)
    assert synth.bf16_bits_to_f32(oracle.dequant_bf16(np.array([1], np.uint8), s, 0))[0] == 1.0
    s = np.float32(1.0 + 3 * 2.0 ** -8)                  # halfway, odd below -> rounds up to 1+2^-6
    assert synth.bf16_bits_to_f32(oracle.dequant_bf16(np.array([1], np.uint8), s, 0))[0] == 1.0 + 2.0 ** -6


# ---------------------------------------------------------------------- gemv
def test_gemv_against_definitions():
    rng = np.random.default_rng(4)
    rows, cols = 37, 300
    q = rng.integers(0, 256, rows * cols).astype(np.uint8)
    s, z = np.float32(0.0173), 131
    W = oracle.dequant_f32(q, s, z).astype(np.float64).reshape(rows, cols)
    # unit vectors pick columns exactly
    for j in (0, 17, cols - 1):
        e = np.zeros(cols, np.float32)
        e[j] = 1.0
        y64, y32 = oracle.gemv(q, rows, cols, s, z, synth.f32_to_bf16_bits(e))
        assert np.array_equal(y64, W[:, j]) and np.array_equal(y32.astype(np.float64), W[:, j])
    # all-ones gives row sums; a random bf16 x matches numpy's fp64 matmul
    ones = synth.f32_to_bf16_bits(np.ones(cols, np.float32))
    y64, _ = oracle.gemv(q, rows, cols, s, z, ones)
    assert np.allclose(y64, W.sum(axis=1), rtol=1e-12, atol=1e-12)
    xb = synth.make_x_bf16(0, 0, cols)
    x = synth.bf16_bits_to_f32(xb).astype(np.float64)
    y64, y32 = oracle.gemv(q, rows, cols, s, z, xb)
    assert np.allclose(y64, W @ x, rtol=1e-12, atol=1e-12)
    assert np.allclose(y32, y64, rtol=1e-4, atol=1e-4)
    # linearity in x (exactly representable combination)
    xb2 = synth.make_x_bf16(0, 1, cols)
    x2 = synth.bf16_bits_to_f32(xb2)
    comb = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(xb) * 2)           # 2*x is exact in bf16
    ya, _ = oracle.gemv(q, rows, cols, s, z, comb)
    assert np.allclose(ya, 2 * y64, rtol=1e-13)
    # a transposed operand would fail this: non-square with distinct row/col structure
    qT = q.reshape(rows, cols).T.copy().ravel()
    yT, _ = oracle.gemv(qT, cols, rows, s, z, synth.make_x_bf16(0, 2, rows))
    xr = synth.bf16_bits_to_f32(synth.make_x_bf16(0, 2, rows)).astype(np.float64)
    assert np.allclose(yT, W.T @ xr, rtol=1e-12, atol=1e-12)
