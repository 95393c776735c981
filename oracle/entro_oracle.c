/*
 * CPU oracle for the EntroLLM hot path  --  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, scalar, single-threaded C.  Only the tests, the smoke check and
 * the benchmark's CPU-baseline leg may call it; the GPU library never does and
 * shares no code, table or helper with it.
 *
 * What each routine follows (EntroLLM, arxiv 2505.02380):
 *   quantize        Proposed Method, "Mixed Quantization Scheme", Eq. 1 and the
 *                   grids of Fig. 2 (unsigned and asymmetric, one (s, z) per
 *                   tensor).  Readings where the text is silent are listed next
 *                   to the function.
 *   huffman_lengths "Huffman weight encoding": a binary tree grown by merging,
 *                   again and again, the two least frequent nodes; a symbol's
 *                   code length is its leaf depth.
 *   canonical_codes The code VALUES are not fixed by the paper (only lengths
 *                   matter for optimality); the stream format uses the
 *                   canonical assignment described at the function.
 *   encode          "Huffman weight encoding" + "Segmentation for parallel
 *                   Huffman decoding": codes appended in flat tensor order, the
 *                   start bit of every fixed-symbol-count segment recorded.
 *   decode          the serial definition (Fig. 3, top): walk an explicit
 *                   binary tree one bit at a time, for each segment on its own
 *                   starting from the segment's recorded boundary.
 *   sub_index       an extension of the same segmentation: stream positions
 *                   recorded inside a segment as well (16-bit piece lengths), and
 *                   the decode of single pieces from those entry points.
 *   dequant / gemv  the inverse grid map (q - z) * s and the batch-1 linear
 *                   layer y = W x of the token-generation phase ("Latency
 *                   Reduction from Huffman Coding").
 *
 * Parity pins live in tests/test_oracle_pins.py (closed forms, brute force on
 * tiny alphabets, Kraft equality, entropy bounds, library one-liners).  The
 * paper prints no worked bitstream, so absolute compressed sizes are pinned
 * only by those invariants ("parity unpinned" against printed values).
 *
 * Stream format (a choice of this build, mirrored independently by the GPU
 * library): bit k of a stream is (stream[k >> 3] >> (k & 7)) & 1; a code of
 * length L is written first-bit-first (its most significant bit lands on the
 * lowest stream position); segments follow each other with no alignment.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_SYMBOLS 256
#define ORACLE_MAX_LEN 32

enum { OR_OK = 0, OR_ERR_ARG = 1, OR_ERR_NONFINITE = 2, OR_ERR_RANGE = 3,
       OR_ERR_SYMBOL = 4, OR_ERR_TOO_LONG = 5, OR_ERR_CAPACITY = 6, OR_ERR_CORRUPT = 7 };

/* ------------------------------------------------------------------ quantize
 * Eq. 1 with Q = 2^bits - 1, all arithmetic in IEEE binary32, rounding to
 * nearest with ties to even (the paper's rounding bracket names no tie rule):
 *   unsigned    s = max / Q              z = 0
 *   asymmetric  s = (max - min) / Q      z = rint(-min / s)
 *   q = clamp(rint(w / s) + z, 0, Q)
 * Eq. 1's right-hand form subtracts z before the division; here z is the
 * integer zero-point of Fig. 2(c), added after rounding, which is the reading
 * under which (q - z) * s inverts the map.  The clamp is needed because
 * rint(max/s) + rint(-min/s) can overshoot Q by one.
 * Errors: non-finite input; negative input under the unsigned scheme; a
 * constant tensor (s would be 0).
 */
int oracle_quantize(const float *w, uint64_t n, int bits, int scheme,
                    uint8_t *q, float *s_out, int32_t *z_out)
{
    if (!w || !q || !s_out || !z_out || n == 0) return OR_ERR_ARG;
    if (bits != 4 && bits != 8) return OR_ERR_ARG;
    if (scheme != 0 && scheme != 1) return OR_ERR_ARG;
    const int32_t Q = (1 << bits) - 1;
    float lo = w[0], hi = w[0];
    for (uint64_t i = 0; i < n; ++i) {
        if (!isfinite(w[i])) return OR_ERR_NONFINITE;
        if (w[i] < lo) lo = w[i];
        if (w[i] > hi) hi = w[i];
    }
    volatile float s;
    int32_t z;
    if (scheme == 0) {
        if (lo < 0.0f) return OR_ERR_RANGE;
        if (!(hi > 0.0f)) return OR_ERR_RANGE;
        s = hi / (float)Q;
        z = 0;
    } else {
        if (!(hi > lo)) return OR_ERR_RANGE;
        volatile float range = hi - lo;
        s = range / (float)Q;
        volatile float zr = -lo / s;
        z = (int32_t)rintf(zr);
    }
    if (!(s > 0.0f) || !isfinite(s)) return OR_ERR_RANGE;
    for (uint64_t i = 0; i < n; ++i) {
        volatile float t = w[i] / s;
        int64_t v = (int64_t)rintf(t) + (int64_t)z;
        if (v < 0) v = 0;
        if (v > Q) v = Q;
        q[i] = (uint8_t)v;
    }
    *s_out = s;
    *z_out = z;
    return OR_OK;
}

int oracle_histogram(const uint8_t *q, uint64_t n, int bits, uint64_t *cnt)
{
    if (!q || !cnt || (bits != 4 && bits != 8)) return OR_ERR_ARG;
    const int A = 1 << bits;
    memset(cnt, 0, sizeof(uint64_t) * (size_t)A);
    for (uint64_t i = 0; i < n; ++i) {
        if (q[i] >= A) return OR_ERR_SYMBOL;
        cnt[q[i]]++;
    }
    return OR_OK;
}

/* ------------------------------------------------------------ Huffman tree
 * Leaves = symbols with a non-zero count, in symbol order.  Repeat: take the
 * two live nodes of smallest weight (ties: the node created earlier first,
 * leaves counting as created in symbol order before any merged node), replace
 * them by a parent whose weight is their sum.  A symbol's length is its depth.
 * Absent symbols get length 0 (no code).  A lone present symbol gets length 1.
 * Several optimal length vectors can exist; only their cost is unique.
 */
int oracle_huffman_lengths(const uint64_t *cnt, int nsym, uint8_t *len)
{
    if (!cnt || !len || nsym < 1 || nsym > ORACLE_MAX_SYMBOLS) return OR_ERR_ARG;
    uint64_t weight[2 * ORACLE_MAX_SYMBOLS];
    int parent[2 * ORACLE_MAX_SYMBOLS];
    int alive[2 * ORACLE_MAX_SYMBOLS];
    int leaf_of[ORACLE_MAX_SYMBOLS];
    int nodes = 0;
    for (int s = 0; s < nsym; ++s) {
        len[s] = 0;
        leaf_of[s] = -1;
        if (cnt[s] > 0) {
            weight[nodes] = cnt[s];
            parent[nodes] = -1;
            alive[nodes] = 1;
            leaf_of[s] = nodes;
            nodes++;
        }
    }
    if (nodes == 0) return OR_ERR_ARG;
    if (nodes == 1) {
        for (int s = 0; s < nsym; ++s) if (leaf_of[s] >= 0) len[s] = 1;
        return OR_OK;
    }
    int live = nodes;
    while (live > 1) {
        int a = -1, b = -1;                 /* a = smallest, b = second smallest */
        for (int i = 0; i < nodes; ++i) {
            if (!alive[i]) continue;
            if (a < 0 || weight[i] < weight[a]) { b = a; a = i; }
            else if (b < 0 || weight[i] < weight[b]) { b = i; }
        }
        weight[nodes] = weight[a] + weight[b];
        parent[nodes] = -1;
        alive[nodes] = 1;
        parent[a] = nodes;
        parent[b] = nodes;
        alive[a] = alive[b] = 0;
        nodes++;
        live--;
    }
    for (int s = 0; s < nsym; ++s) {
        if (leaf_of[s] < 0) continue;
        int d = 0;
        for (int v = leaf_of[s]; parent[v] >= 0; v = parent[v]) d++;
        if (d > ORACLE_MAX_LEN) return OR_ERR_TOO_LONG;
        len[s] = (uint8_t)d;
    }
    return OR_OK;
}

/* Canonical assignment: present symbols ordered by (length, symbol); the first
 * gets code 0; each next one gets (previous + 1) shifted left by the growth in
 * length.  Code values are read as `len`-bit integers, most significant bit
 * first.  Fails if the lengths over-subscribe the code space. */
int oracle_canonical_codes(const uint8_t *len, int nsym, uint32_t *code)
{
    if (!len || !code || nsym < 1 || nsym > ORACLE_MAX_SYMBOLS) return OR_ERR_ARG;
    uint64_t next = 0;
    int prev_len = 0;
    int any = 0;
    for (int L = 1; L <= ORACLE_MAX_LEN; ++L) {
        for (int s = 0; s < nsym; ++s) {
            if (len[s] != L) continue;
            if (any) next = (next + 1) << (L - prev_len);
            if (next >> L) return OR_ERR_CORRUPT;      /* Kraft sum above 1 */
            code[s] = (uint32_t)next;
            prev_len = L;
            any = 1;
        }
    }
    for (int s = 0; s < nsym; ++s) {
        if (len[s] > ORACLE_MAX_LEN) return OR_ERR_TOO_LONG;
        if (len[s] == 0) code[s] = 0;
    }
    return any ? OR_OK : OR_ERR_ARG;
}

/* ------------------------------------------------------------------ encode */
static void put_bit(uint8_t *stream, uint64_t k, int bit)
{
    if (bit) stream[k >> 3] |= (uint8_t)(1u << (k & 7));
}

/* Size in bytes of an encoded stream holding `total_bits`: whole bytes, then
 * zero bytes up to a multiple of 16, then 16 more zero bytes. */
uint64_t oracle_stream_bytes(uint64_t total_bits)
{
    uint64_t b = (total_bits + 7) / 8;
    b = (b + 15) / 16 * 16;
    return b + 16;
}

/* offsets has ceil(n / chunk_symbols) + 1 entries; offsets[k] is the stream
 * bit at which symbol k*chunk_symbols starts, the last entry the total. */
int oracle_encode(const uint8_t *q, uint64_t n, const uint8_t *len, const uint32_t *code,
                  int nsym, uint32_t chunk_symbols, uint8_t *stream, uint64_t stream_cap,
                  uint64_t *stream_bytes, uint64_t *offsets)
{
    if (!q || !len || !code || !stream || !stream_bytes || !offsets) return OR_ERR_ARG;
    if (n == 0 || chunk_symbols == 0) return OR_ERR_ARG;
    uint64_t total = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (q[i] >= nsym || len[q[i]] == 0) return OR_ERR_SYMBOL;
        total += len[q[i]];
    }
    uint64_t need = oracle_stream_bytes(total);
    if (need > stream_cap) return OR_ERR_CAPACITY;
    memset(stream, 0, need);
    uint64_t pos = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (i % chunk_symbols == 0) offsets[i / chunk_symbols] = pos;
        int L = len[q[i]];
        uint32_t c = code[q[i]];
        for (int b = L - 1; b >= 0; --b) put_bit(stream, pos++, (int)((c >> b) & 1u));
    }
    offsets[(n + chunk_symbols - 1) / chunk_symbols] = pos;
    *stream_bytes = need;
    return OR_OK;
}

/* ------------------------------------------------------------------ decode */
typedef struct { int32_t child[2]; int32_t symbol; } tree_node;   /* symbol < 0: inner */

static int build_tree(const uint8_t *len, const uint32_t *code, int nsym, tree_node *t, int cap)
{
    int used = 1;
    t[0].child[0] = t[0].child[1] = -1;
    t[0].symbol = -1;
    for (int s = 0; s < nsym; ++s) {
        if (len[s] == 0) continue;
        int v = 0;
        for (int b = len[s] - 1; b >= 0; --b) {
            int bit = (int)((code[s] >> b) & 1u);
            if (t[v].symbol >= 0) return -1;               /* a code is a prefix of another */
            if (t[v].child[bit] < 0) {
                if (used >= cap) return -1;
                t[used].child[0] = t[used].child[1] = -1;
                t[used].symbol = -1;
                t[v].child[bit] = used++;
            }
            v = t[v].child[bit];
        }
        if (t[v].symbol >= 0 || t[v].child[0] >= 0 || t[v].child[1] >= 0) return -1;
        t[v].symbol = s;
    }
    return used;
}

static int get_bit(const uint8_t *stream, uint64_t k)
{
    return (stream[k >> 3] >> (k & 7)) & 1;
}

/* Decode segments [first_chunk, first_chunk + num_chunks) into out, which is
 * indexed by absolute symbol position (out[i] for symbol i of the tensor). */
int oracle_decode_chunks(const uint8_t *stream, uint64_t stream_bytes, const uint64_t *offsets,
                         uint64_t n, uint32_t chunk_symbols, const uint8_t *len,
                         const uint32_t *code, int nsym, uint64_t first_chunk,
                         uint64_t num_chunks, uint8_t *out)
{
    if (!stream || !offsets || !len || !code || !out || n == 0 || chunk_symbols == 0)
        return OR_ERR_ARG;
    const uint64_t n_chunks = (n + chunk_symbols - 1) / chunk_symbols;
    if (first_chunk + num_chunks > n_chunks) return OR_ERR_ARG;
    const int cap = 2 * ORACLE_MAX_SYMBOLS * ORACLE_MAX_LEN;
    tree_node *t = (tree_node *)malloc(sizeof(tree_node) * (size_t)cap);
    if (!t) return OR_ERR_ARG;
    if (build_tree(len, code, nsym, t, cap) < 0) { free(t); return OR_ERR_CORRUPT; }
    const uint64_t limit_bits = stream_bytes * 8;
    int rc = OR_OK;
    for (uint64_t k = first_chunk; k < first_chunk + num_chunks && rc == OR_OK; ++k) {
        uint64_t pos = offsets[k];
        uint64_t lo = k * (uint64_t)chunk_symbols;
        uint64_t hi = lo + chunk_symbols < n ? lo + chunk_symbols : n;
        for (uint64_t i = lo; i < hi; ++i) {
            int v = 0;
            while (t[v].symbol < 0) {
                if (pos >= limit_bits) { rc = OR_ERR_CORRUPT; break; }
                v = t[v].child[get_bit(stream, pos++)];
                if (v < 0) { rc = OR_ERR_CORRUPT; break; }
            }
            if (rc != OR_OK) break;
            out[i] = (uint8_t)t[v].symbol;
        }
    }
    free(t);
    return rc;
}

int oracle_decode(const uint8_t *stream, uint64_t stream_bytes, const uint64_t *offsets,
                  uint64_t n, uint32_t chunk_symbols, const uint8_t *len, const uint32_t *code,
                  int nsym, uint8_t *out)
{
    if (n == 0 || chunk_symbols == 0) return OR_ERR_ARG;
    return oracle_decode_chunks(stream, stream_bytes, offsets, n, chunk_symbols, len, code, nsym,
                                0, (n + chunk_symbols - 1) / chunk_symbols, out);
}

/* ------------------------------------------------- entry points inside a segment
 * An extension of "Segmentation for parallel Huffman decoding" (segments with known
 * boundaries decode independently, Fig. 3): inside a segment the stream position
 * is recorded every `sub_symbols` symbols as well, so that a piece of a segment
 * can be decoded on its own.  chunk_symbols must be a multiple of sub_symbols.
 * sub_bits[j], j = 0 .. ceil(n / sub_symbols) - 1, is the number of stream bits
 * that piece j (symbols j*sub_symbols .. (j+1)*sub_symbols - 1) occupies, so
 * piece j starts at its segment's offset plus the sub_bits of the pieces in
 * front of it in the same segment.  A piece longer than 65535 bits does not fit
 * the 16-bit entry (OR_ERR_TOO_LONG). */
int oracle_sub_index(const uint8_t *q, uint64_t n, const uint8_t *len, int nsym,
                     uint32_t chunk_symbols, uint32_t sub_symbols, uint16_t *sub_bits)
{
    if (!q || !len || !sub_bits || n == 0 || chunk_symbols == 0 || sub_symbols == 0) return OR_ERR_ARG;
    if (chunk_symbols % sub_symbols != 0) return OR_ERR_ARG;
    uint64_t bits = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (q[i] >= nsym || len[q[i]] == 0) return OR_ERR_SYMBOL;
        bits += len[q[i]];
        if ((i + 1) % sub_symbols == 0 || i + 1 == n) {
            if (bits > 65535u) return OR_ERR_TOO_LONG;
            sub_bits[i / sub_symbols] = (uint16_t)bits;
            bits = 0;
        }
    }
    return OR_OK;
}

/* Decode pieces [first_sub, first_sub + num_subs), each on its own from its
 * entry point, into out (indexed by absolute symbol position). */
int oracle_decode_subs(const uint8_t *stream, uint64_t stream_bytes, const uint64_t *offsets,
                       const uint16_t *sub_bits, uint64_t n, uint32_t chunk_symbols,
                       uint32_t sub_symbols, const uint8_t *len, const uint32_t *code, int nsym,
                       uint64_t first_sub, uint64_t num_subs, uint8_t *out)
{
    if (!stream || !offsets || !sub_bits || !len || !code || !out || n == 0) return OR_ERR_ARG;
    if (chunk_symbols == 0 || sub_symbols == 0 || chunk_symbols % sub_symbols != 0) return OR_ERR_ARG;
    const uint64_t per_chunk = chunk_symbols / sub_symbols;
    const uint64_t n_subs = (n + sub_symbols - 1) / sub_symbols;
    if (first_sub + num_subs > n_subs) return OR_ERR_ARG;
    const int cap = 2 * ORACLE_MAX_SYMBOLS * ORACLE_MAX_LEN;
    tree_node *t = (tree_node *)malloc(sizeof(tree_node) * (size_t)cap);
    if (!t) return OR_ERR_ARG;
    if (build_tree(len, code, nsym, t, cap) < 0) { free(t); return OR_ERR_CORRUPT; }
    const uint64_t limit_bits = stream_bytes * 8;
    int rc = OR_OK;
    for (uint64_t j = first_sub; j < first_sub + num_subs && rc == OR_OK; ++j) {
        const uint64_t chunk = j / per_chunk;
        uint64_t pos = offsets[chunk];
        for (uint64_t i = chunk * per_chunk; i < j; ++i) pos += sub_bits[i];
        const uint64_t lo = j * (uint64_t)sub_symbols;
        const uint64_t hi = lo + sub_symbols < n ? lo + sub_symbols : n;
        for (uint64_t i = lo; i < hi; ++i) {
            int v = 0;
            while (t[v].symbol < 0) {
                if (pos >= limit_bits) { rc = OR_ERR_CORRUPT; break; }
                v = t[v].child[get_bit(stream, pos++)];
                if (v < 0) { rc = OR_ERR_CORRUPT; break; }
            }
            if (rc != OR_OK) break;
            out[i] = (uint8_t)t[v].symbol;
        }
    }
    free(t);
    return rc;
}

/* Two 4-bit symbols per byte: symbol 2i in the low nibble, 2i+1 in the high
 * nibble; an odd count leaves the last high nibble zero.  out has (n+1)/2 bytes. */
void oracle_pack_u4(const uint8_t *q, uint64_t n, uint8_t *out)
{
    for (uint64_t i = 0; i < (n + 1) / 2; ++i) {
        uint8_t lo = q[2 * i] & 15u;
        uint8_t hi = (2 * i + 1 < n) ? (q[2 * i + 1] & 15u) : 0u;
        out[i] = (uint8_t)(lo | (hi << 4));
    }
}

/* ----------------------------------------------------------------- dequant
 * w = (q - z) * s: the difference in integers, converted exactly to binary32,
 * then a single binary32 multiplication. */
void oracle_dequant_f32(const uint8_t *q, uint64_t n, float s, int32_t z, float *out)
{
    for (uint64_t i = 0; i < n; ++i) {
        volatile float d = (float)((int32_t)q[i] - z);
        volatile float p = d * s;
        out[i] = p;
    }
}

static uint16_t bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);   /* NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* bfloat16 = the binary32 product rounded to nearest, ties to even. */
void oracle_dequant_bf16(const uint8_t *q, uint64_t n, float s, int32_t z, uint16_t *out)
{
    for (uint64_t i = 0; i < n; ++i) {
        volatile float d = (float)((int32_t)q[i] - z);
        volatile float p = d * s;
        out[i] = bf16_rne(p);
    }
}

/* -------------------------------------------------------------------- gemv
 * y[r] = sum_j w[r][j] * x[j], W row-major [rows][cols], w the binary32
 * dequantised weight, x bfloat16 widened exactly.  y64: every product and the
 * running sum in binary64, j ascending (the reference).  y32 (optional): the
 * same loop with a binary32 running sum, to show what sequential fp32
 * accumulation gives. */
void oracle_gemv(const uint8_t *q, uint64_t rows, uint64_t cols, float s, int32_t z,
                 const uint16_t *x_bf16, double *y64, float *y32)
{
    for (uint64_t r = 0; r < rows; ++r) {
        double acc = 0.0;
        volatile float acc32 = 0.0f;
        for (uint64_t j = 0; j < cols; ++j) {
            volatile float d = (float)((int32_t)q[r * cols + j] - z);
            volatile float w = d * s;
            uint32_t xb = (uint32_t)x_bf16[j] << 16;
            float xf;
            memcpy(&xf, &xb, 4);
            acc += (double)w * (double)xf;
            volatile float p32 = w * xf;
            acc32 = acc32 + p32;
        }
        y64[r] = acc;
        if (y32) y32[r] = acc32;
    }
}

/* ------------------------------------------------------------- brute force
 * Smallest sum(cnt[i] * len[i]) over ALL prefix-code length vectors for m <= 8
 * symbols with positive counts: every assignment of lengths 1..m-1 (a longer
 * code never helps with m leaves) whose Kraft sum is at most 1. */
static void brute_rec(const uint64_t *cnt, int m, int i, uint64_t kraft_num, int maxlen,
                      uint64_t cost, uint64_t *best)
{
    /* kraft_num counts units of 2^-maxlen */
    if (kraft_num > ((uint64_t)1 << maxlen)) return;
    if (cost >= *best) return;
    if (i == m) { *best = cost; return; }
    for (int L = 1; L <= maxlen; ++L)
        brute_rec(cnt, m, i + 1, kraft_num + ((uint64_t)1 << (maxlen - L)), maxlen,
                  cost + cnt[i] * (uint64_t)L, best);
}

uint64_t oracle_bruteforce_min_cost(const uint64_t *cnt, int m)
{
    if (m < 1 || m > 8) return 0;
    if (m == 1) return cnt[0];
    uint64_t best = UINT64_MAX;
    brute_rec(cnt, m, 0, 0, m - 1, 0, &best);
    return best;
}

/* ------------------------------------------------- length-limited prefix codes
 * An extension in the direction the paper's conclusions name as future work
 * (hardware-aware optimisation of the coder): the prefix code with the smallest
 * sum(cnt[i] * len[i]) among those whose codes are at most max_len bits long, so
 * that a decoder's single-level table holds every code.
 *
 * This is the definition written out, not a construction: every assignment of
 * lengths 1..max_len to the symbols with a positive count whose Kraft sum
 * sum(2^-len) is at most 1 is the length vector of a prefix code, and the
 * minimum over all of them is taken by dynamic programming over the Kraft budget
 * in units of 2^-max_len: best[i][u] = min over len of best[i-1][u - 2^(max_len
 * - len)] + cnt[i] * len.  max_len <= 16 keeps the table small.
 * len_out gets one optimal length vector (0 for absent symbols); returns 0, or 1
 * for bad arguments (more symbols than 2^max_len codes, no symbol at all). */
int oracle_limited_lengths(const uint64_t *cnt, int nsym, int max_len, uint8_t *len_out, uint64_t *cost_out)
{
    if (!cnt || !len_out || nsym < 1 || nsym > 256 || max_len < 1 || max_len > 16) return 1;
    int idx[256], m = 0;
    for (int s = 0; s < nsym; ++s) { len_out[s] = 0; if (cnt[s]) idx[m++] = s; }
    if (m == 0 || ((uint64_t)m > ((uint64_t)1 << max_len))) return 1;
    if (m == 1) { len_out[idx[0]] = 1; if (cost_out) *cost_out = cnt[idx[0]]; return 0; }
    const uint32_t U = (uint32_t)1 << max_len;
    uint64_t *prev = malloc(sizeof(uint64_t) * (U + 1)), *cur = malloc(sizeof(uint64_t) * (U + 1));
    uint8_t *choice = malloc((size_t)m * (U + 1));
    if (!prev || !cur || !choice) { free(prev); free(cur); free(choice); return 1; }
    for (uint32_t u = 0; u <= U; ++u) prev[u] = 0;                 /* no symbol placed: cost 0 at any budget */
    for (int i = 0; i < m; ++i) {
        const uint64_t c = cnt[idx[i]];
        for (uint32_t u = 0; u <= U; ++u) {
            uint64_t best = UINT64_MAX;
            uint8_t bl = 0;
            for (int l = 1; l <= max_len; ++l) {
                const uint32_t need = (uint32_t)1 << (max_len - l);
                if (need > u || prev[u - need] == UINT64_MAX) continue;
                const uint64_t v = prev[u - need] + c * (uint64_t)l;
                if (v < best) { best = v; bl = (uint8_t)l; }
            }
            cur[u] = best;
            choice[(size_t)i * (U + 1) + u] = bl;
        }
        uint64_t *t = prev; prev = cur; cur = t;
    }
    /* prev[u]: cheapest way to place all symbols within budget exactly-or-under u (budgets are "at most":
     * prev of an earlier row is defined for every u, so spare budget is simply left unused) */
    if (prev[U] == UINT64_MAX) { free(prev); free(cur); free(choice); return 1; }
    if (cost_out) *cost_out = prev[U];
    uint32_t u = U;
    for (int i = m - 1; i >= 0; --i) {
        const uint8_t l = choice[(size_t)i * (U + 1) + u];
        len_out[idx[i]] = l;
        u -= (uint32_t)1 << (max_len - l);
    }
    free(prev); free(cur); free(choice);
    return 0;
}

/* The same minimum by plain enumeration, for m <= 8 symbols with positive counts. */
uint64_t oracle_bruteforce_min_cost_limited(const uint64_t *cnt, int m, int max_len)
{
    if (m < 1 || m > 8 || max_len < 1 || max_len > 12) return 0;
    if (m == 1) return cnt[0];
    uint64_t best = UINT64_MAX;
    brute_rec(cnt, m, 0, 0, max_len, 0, &best);
    return best;
}
