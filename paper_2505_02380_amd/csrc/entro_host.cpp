// Host side of libentro: quantisation, Huffman code construction, encoding.
//
// These steps run offline, before the GPU hot path (EntroLLM, Proposed Method:
// "Mixed Quantization Scheme" with Eq. 1 / Fig. 2, "Huffman weight encoding",
// "Segmentation for parallel Huffman decoding").  They are support code for
// the decoders in entro_device.hip and are written for throughput on the host
// (threads over ranges) so that multi-gigabyte synthetic weight sets can be
// prepared in seconds.
#include "entro.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

namespace {

unsigned worker_count(uint64_t n, uint64_t grain) {
    unsigned hw = std::thread::hardware_concurrency();
    if (hw == 0) hw = 1;
    if (const char *e = std::getenv("ENTRO_HOST_THREADS")) {
        int v = std::atoi(e);
        if (v > 0) hw = static_cast<unsigned>(v);
    }
    uint64_t want = (n + grain - 1) / grain;
    if (want < 1) want = 1;
    return static_cast<unsigned>(std::min<uint64_t>(hw, want));
}

// Run f(part, begin, end) over [0, n) split into contiguous parts.
template <class F>
void parallel_ranges(uint64_t n, uint64_t grain, F f) {
    unsigned parts = worker_count(n, grain);
    if (parts <= 1) {
        f(0u, uint64_t{0}, n);
        return;
    }
    std::vector<std::thread> th;
    th.reserve(parts);
    uint64_t per = (n + parts - 1) / parts;
    for (unsigned p = 0; p < parts; ++p) {
        uint64_t b = std::min<uint64_t>(n, per * p), e = std::min<uint64_t>(n, per * (p + 1));
        th.emplace_back([=] { f(p, b, e); });
    }
    for (auto &t : th) t.join();
}

bool bits_ok(int bits) { return bits == 4 || bits == 8; }

// Optimal prefix-code lengths by the two-queue construction: leaves sorted by
// count feed one queue, merged nodes (created in non-decreasing weight order)
// the other; the two lightest fronts are merged until one node is left.
entro_status huffman_lengths(const uint64_t *counts, int nsym, uint8_t *len) {
    struct Node { uint64_t w; int parent; };
    std::vector<int> order;
    for (int s = 0; s < nsym; ++s) {
        len[s] = 0;
        if (counts[s]) order.push_back(s);
    }
    const int m = static_cast<int>(order.size());
    if (m == 0) return ENTRO_ERR_SIZE;
    if (m == 1) {
        len[order[0]] = 1;
        return ENTRO_OK;
    }
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return counts[a] < counts[b]; });
    std::vector<Node> nodes(2 * m - 1);
    for (int i = 0; i < m; ++i) nodes[i] = {counts[order[i]], -1};
    int leaf = 0, inner = m, made = m;
    auto pop = [&]() {
        // prefer a leaf on ties: keeps the tree shallow
        if (leaf < m && (inner >= made || nodes[leaf].w <= nodes[inner].w)) return leaf++;
        return inner++;
    };
    while (made < 2 * m - 1) {
        int a = pop();
        int b = pop();
        nodes[made] = {nodes[a].w + nodes[b].w, -1};
        nodes[a].parent = made;
        nodes[b].parent = made;
        ++made;
    }
    // depth of every node from the root downwards (parents have larger indices)
    std::vector<int> depth(2 * m - 1, 0);
    for (int i = 2 * m - 3; i >= 0; --i) depth[i] = depth[nodes[i].parent] + 1;
    for (int i = 0; i < m; ++i) {
        if (depth[i] > ENTRO_MAX_CODE_LEN) return ENTRO_ERR_CODE_TOO_LONG;
        len[order[i]] = static_cast<uint8_t>(depth[i]);
    }
    return ENTRO_OK;
}

// Cheapest prefix-code lengths under a length limit, by package-merge (Larmore and
// Hirschberg): at every level from the limit up to 1 the leaves are merged, by
// weight, with the pairs ("packages") of the level below; the 2m - 2 lightest
// items of the top level are kept, and a symbol's length is the number of kept
// items its leaf is part of.  A package is a weight and, per leaf, how often it
// holds it.
entro_status limited_lengths(const uint64_t *counts, int nsym, int max_len, uint8_t *len) {
    if (max_len < 1 || max_len > ENTRO_MAX_CODE_LEN) return ENTRO_ERR_SIZE;
    std::vector<int> order;
    for (int s = 0; s < nsym; ++s) {
        len[s] = 0;
        if (counts[s]) order.push_back(s);
    }
    const int m = static_cast<int>(order.size());
    if (m == 0) return ENTRO_ERR_SIZE;
    if (m == 1) {
        len[order[0]] = 1;
        return ENTRO_OK;
    }
    if (max_len < 31 && (uint64_t{1} << max_len) < static_cast<uint64_t>(m)) return ENTRO_ERR_CODE_TOO_LONG;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return counts[a] < counts[b]; });
    struct Item {
        unsigned __int128 w;            // sums of up to 2^31 counts of up to 2^64: more than 64 bits
        std::vector<uint8_t> holds;     // per leaf (in sorted order): times this item holds it
    };
    auto leaf_items = [&]() {
        std::vector<Item> v(m);
        for (int i = 0; i < m; ++i) {
            v[i].w = counts[order[i]];
            v[i].holds.assign(m, 0);
            v[i].holds[i] = 1;
        }
        return v;
    };
    std::vector<Item> level = leaf_items();                         // the deepest level: leaves only
    for (int depth = max_len - 1; depth >= 1; --depth) {
        // packages of the level below: its items paired up in weight order (an odd one out is dropped)
        std::vector<Item> packages;
        for (size_t i = 0; i + 1 < level.size(); i += 2) {
            Item p;
            p.w = level[i].w + level[i + 1].w;
            p.holds = level[i].holds;
            for (int j = 0; j < m; ++j) p.holds[j] = static_cast<uint8_t>(p.holds[j] + level[i + 1].holds[j]);
            packages.push_back(std::move(p));
        }
        std::vector<Item> leaves = leaf_items(), merged;
        merged.reserve(leaves.size() + packages.size());
        size_t a = 0, b = 0;
        while (a < leaves.size() || b < packages.size()) {
            // a leaf first on equal weight: keeps codes short for the heavier symbols
            if (b >= packages.size() || (a < leaves.size() && leaves[a].w <= packages[b].w)) merged.push_back(std::move(leaves[a++]));
            else merged.push_back(std::move(packages[b++]));
        }
        level.swap(merged);
    }
    std::vector<int> depth_of(m, 0);
    for (int i = 0; i < 2 * m - 2; ++i)
        for (int j = 0; j < m; ++j) depth_of[j] += level[i].holds[j];
    for (int j = 0; j < m; ++j) {
        if (depth_of[j] < 1 || depth_of[j] > max_len) return ENTRO_ERR_CODE_TOO_LONG;   // cannot happen
        len[order[j]] = static_cast<uint8_t>(depth_of[j]);
    }
    return ENTRO_OK;
}

entro_status assign_canonical(entro_codebook *cb) {
    const int nsym = 1 << cb->bits;
    uint32_t per_len[ENTRO_MAX_CODE_LEN + 2] = {0};
    int used = 0, max_len = 0;
    for (int s = 0; s < ENTRO_MAX_SYMBOLS; ++s) {
        if (s >= nsym) {
            if (cb->len[s]) return ENTRO_ERR_SYMBOL;
            cb->code[s] = 0;
            continue;
        }
        int l = cb->len[s];
        if (l > ENTRO_MAX_CODE_LEN) return ENTRO_ERR_CODE_TOO_LONG;
        if (l) {
            per_len[l]++;
            ++used;
            max_len = std::max(max_len, l);
        }
        cb->code[s] = 0;
    }
    if (used == 0) return ENTRO_ERR_SIZE;
    // first code of each length; reject over-subscribed length sets
    uint64_t next[ENTRO_MAX_CODE_LEN + 2] = {0};
    uint64_t code = 0;
    for (int l = 1; l <= max_len; ++l) {
        code = (code + per_len[l - 1]) << 1;
        next[l] = code;
        if (code + per_len[l] > (uint64_t{1} << l)) return ENTRO_ERR_CORRUPT;
    }
    for (int s = 0; s < nsym; ++s)
        if (int l = cb->len[s]) cb->code[s] = static_cast<uint32_t>(next[l]++);
    cb->n_used = used;
    cb->max_len = max_len;
    cb->reserved = 0;
    return ENTRO_OK;
}

// Append-only little-endian bit writer over a zeroed byte range.  The first
// and last byte it touches may be shared with a neighbouring writer, so those
// are merged with an atomic OR; everything in between is stored plainly.
class BitWriter {
public:
    BitWriter(uint8_t *base, uint64_t start_bit)
        : base_(base), byte_(start_bit >> 3), acc_(0), fill_(static_cast<unsigned>(start_bit & 7)),
          first_(true) {}
    // `code` read as a len-bit integer goes out most significant bit first
    void put(uint32_t code, unsigned len) {
        uint64_t rev = reverse_bits(code, len);
        acc_ |= rev << fill_;
        fill_ += len;
        while (fill_ >= 8) {
            emit(static_cast<uint8_t>(acc_));
            acc_ >>= 8;
            fill_ -= 8;
        }
    }
    void finish() {
        if (fill_) or_byte(byte_, static_cast<uint8_t>(acc_));
        fill_ = 0;
    }

private:
    static uint64_t reverse_bits(uint32_t v, unsigned len) {
        v = ((v >> 1) & 0x55555555u) | ((v & 0x55555555u) << 1);
        v = ((v >> 2) & 0x33333333u) | ((v & 0x33333333u) << 2);
        v = ((v >> 4) & 0x0f0f0f0fu) | ((v & 0x0f0f0f0fu) << 4);
        v = ((v >> 8) & 0x00ff00ffu) | ((v & 0x00ff00ffu) << 8);
        v = (v >> 16) | (v << 16);
        return len ? static_cast<uint64_t>(v) >> (32 - len) : 0;
    }
    void or_byte(uint64_t at, uint8_t v) { __atomic_fetch_or(base_ + at, v, __ATOMIC_RELAXED); }
    void emit(uint8_t v) {
        if (first_) {
            or_byte(byte_, v);
            first_ = false;
        } else {
            base_[byte_] = v;
        }
        ++byte_;
    }
    uint8_t *base_;
    uint64_t byte_;
    uint64_t acc_;
    unsigned fill_;
    bool first_;
};

uint64_t padded_bytes(uint64_t total_bits) {
    uint64_t b = (total_bits + 7) / 8;
    b = (b + 15) / 16 * 16;
    return b + 16;
}

}  // namespace

extern "C" {

entro_scheme entro_scheme_for_range(float min, float max) {
    return (min >= 0.0f && max > 0.0f) ? ENTRO_UNSIGNED : ENTRO_ASYMMETRIC;
}

entro_status entro_qparams_from_range(float min, float max, uint32_t nonfinite, int bits, entro_scheme scheme,
                                      entro_qparams *qp) {
    if (!qp) return ENTRO_ERR_NULL;
    if (!bits_ok(bits)) return ENTRO_ERR_BITS;
    if (scheme != ENTRO_UNSIGNED && scheme != ENTRO_ASYMMETRIC) return ENTRO_ERR_SCHEME;
    if (nonfinite || !std::isfinite(min) || !std::isfinite(max)) return ENTRO_ERR_NONFINITE;
    const float Q = static_cast<float>((1 << bits) - 1);
    float s;
    int32_t z;
    if (scheme == ENTRO_UNSIGNED) {
        if (min < 0.0f || !(max > 0.0f)) return ENTRO_ERR_RANGE;
        s = max / Q;
        z = 0;
    } else {
        if (!(max > min)) return ENTRO_ERR_RANGE;
        s = (max - min) / Q;
        if (!(s > 0.0f) || !std::isfinite(s)) return ENTRO_ERR_RANGE;
        z = static_cast<int32_t>(std::nearbyintf(-min / s));
    }
    if (!(s > 0.0f) || !std::isfinite(s)) return ENTRO_ERR_RANGE;
    qp->scale = s;
    qp->zero_point = z;
    qp->bits = bits;
    qp->scheme = scheme;
    return ENTRO_OK;
}

entro_status entro_quantize(const float *w, uint64_t n, int bits, entro_scheme scheme, uint8_t *q,
                            entro_qparams *qp) {
    if (!w || !q || !qp) return ENTRO_ERR_NULL;
    if (!bits_ok(bits)) return ENTRO_ERR_BITS;
    if (scheme != ENTRO_UNSIGNED && scheme != ENTRO_ASYMMETRIC) return ENTRO_ERR_SCHEME;
    if (n == 0) return ENTRO_ERR_SIZE;

    const unsigned parts = worker_count(n, 1u << 20);
    std::vector<float> lo(parts, w[0]), hi(parts, w[0]);
    std::vector<char> bad(parts, 0);
    parallel_ranges(n, 1u << 20, [&](unsigned p, uint64_t b, uint64_t e) {
        float l = w[b < n ? b : 0], h = l;
        bool nonfinite = false;
        for (uint64_t i = b; i < e; ++i) {
            float v = w[i];
            nonfinite |= !std::isfinite(v);
            l = v < l ? v : l;
            h = v > h ? v : h;
        }
        lo[p] = l;
        hi[p] = h;
        bad[p] = nonfinite;
    });
    float mn = lo[0], mx = hi[0];
    for (unsigned p = 0; p < parts; ++p) {
        if (bad[p]) return ENTRO_ERR_NONFINITE;
        mn = std::min(mn, lo[p]);
        mx = std::max(mx, hi[p]);
    }
    entro_status st = entro_qparams_from_range(mn, mx, 0, bits, scheme, qp);
    if (st != ENTRO_OK) return st;
    const float s = qp->scale;
    const int32_t z = qp->zero_point;
    const int32_t Qi = (1 << bits) - 1;
    parallel_ranges(n, 1u << 20, [&](unsigned, uint64_t b, uint64_t e) {
        for (uint64_t i = b; i < e; ++i) {
            // true division, nearest-even rounding (default FP environment)
            int64_t v = static_cast<int64_t>(std::nearbyintf(w[i] / s)) + z;
            v = v < 0 ? 0 : (v > Qi ? Qi : v);
            q[i] = static_cast<uint8_t>(v);
        }
    });
    return ENTRO_OK;
}

entro_status entro_codebook_from_lengths(const uint8_t *len, int bits, entro_codebook *cb) {
    if (!len || !cb) return ENTRO_ERR_NULL;
    if (!bits_ok(bits)) return ENTRO_ERR_BITS;
    std::memset(cb, 0, sizeof(*cb));
    cb->bits = bits;
    std::memcpy(cb->len, len, static_cast<size_t>(1) << bits);
    return assign_canonical(cb);
}

entro_status entro_codebook_from_counts(const uint64_t *counts, int bits, entro_codebook *cb) {
    if (!counts || !cb) return ENTRO_ERR_NULL;
    if (!bits_ok(bits)) return ENTRO_ERR_BITS;
    std::memset(cb, 0, sizeof(*cb));
    cb->bits = bits;
    entro_status st = huffman_lengths(counts, 1 << bits, cb->len);
    if (st != ENTRO_OK) return st;
    return assign_canonical(cb);
}

entro_status entro_codebook_from_counts_limited(const uint64_t *counts, int bits, int max_len, entro_codebook *cb) {
    if (!counts || !cb) return ENTRO_ERR_NULL;
    if (!bits_ok(bits)) return ENTRO_ERR_BITS;
    std::memset(cb, 0, sizeof(*cb));
    cb->bits = bits;
    entro_status st = limited_lengths(counts, 1 << bits, max_len, cb->len);
    if (st != ENTRO_OK) return st;
    return assign_canonical(cb);
}

static entro_status histogram_of(const uint8_t *q, uint64_t n, int bits, uint64_t *counts);

entro_status entro_build_codebook_limited(const uint8_t *q, uint64_t n, int bits, int max_len, entro_codebook *cb) {
    if (!q || !cb) return ENTRO_ERR_NULL;
    if (!bits_ok(bits)) return ENTRO_ERR_BITS;
    if (n == 0) return ENTRO_ERR_SIZE;
    uint64_t counts[256];
    entro_status st = histogram_of(q, n, bits, counts);
    if (st != ENTRO_OK) return st;
    return entro_codebook_from_counts_limited(counts, bits, max_len, cb);
}

entro_status entro_build_codebook(const uint8_t *q, uint64_t n, int bits, entro_codebook *cb) {
    if (!q || !cb) return ENTRO_ERR_NULL;
    if (!bits_ok(bits)) return ENTRO_ERR_BITS;
    if (n == 0) return ENTRO_ERR_SIZE;
    uint64_t counts[256];
    entro_status st = histogram_of(q, n, bits, counts);
    if (st != ENTRO_OK) return st;
    return entro_codebook_from_counts(counts, bits, cb);
}

// Symbol counts of q, on all host threads.
static entro_status histogram_of(const uint8_t *q, uint64_t n, int bits, uint64_t *counts) {
    const unsigned parts = worker_count(n, 1u << 22);
    std::vector<uint64_t> hist(static_cast<size_t>(parts) * 256, 0);
    parallel_ranges(n, 1u << 22, [&](unsigned p, uint64_t b, uint64_t e) {
        // four interleaved tables hide the store-to-load dependency on repeated symbols
        uint64_t h[4][256] = {};
        uint64_t i = b;
        for (; i + 4 <= e; i += 4) {
            h[0][q[i]]++;
            h[1][q[i + 1]]++;
            h[2][q[i + 2]]++;
            h[3][q[i + 3]]++;
        }
        for (; i < e; ++i) h[0][q[i]]++;
        uint64_t *dst = &hist[static_cast<size_t>(p) * 256];
        for (int s = 0; s < 256; ++s) dst[s] = h[0][s] + h[1][s] + h[2][s] + h[3][s];
    });
    for (int s = 0; s < 256; ++s) counts[s] = 0;
    for (unsigned p = 0; p < parts; ++p)
        for (int s = 0; s < 256; ++s) counts[s] += hist[static_cast<size_t>(p) * 256 + s];
    for (int s = 1 << bits; s < 256; ++s)
        if (counts[s]) return ENTRO_ERR_SYMBOL;
    return ENTRO_OK;
}

uint64_t entro_num_chunks(uint64_t n, uint32_t chunk_symbols) {
    return chunk_symbols ? (n + chunk_symbols - 1) / chunk_symbols : 0;
}

uint64_t entro_encode_bound(uint64_t n, const entro_codebook *cb) {
    if (!cb || n == 0 || cb->max_len < 1 || cb->max_len > ENTRO_MAX_CODE_LEN) return 0;
    return padded_bytes(n * static_cast<uint64_t>(cb->max_len));
}

uint64_t entro_encoded_bytes(const uint64_t *counts, const entro_codebook *cb) {
    if (!counts || !cb || !bits_ok(cb->bits)) return 0;
    uint64_t bits = 0;
    for (int s = 0; s < (1 << cb->bits); ++s) {
        if (counts[s] && !cb->len[s]) return 0;
        bits += counts[s] * cb->len[s];
    }
    return padded_bytes(bits);
}

entro_status entro_encode(const uint8_t *q, uint64_t n, const entro_codebook *cb,
                          uint32_t chunk_symbols, uint8_t *stream, uint64_t stream_cap,
                          uint64_t *stream_bytes, uint64_t *offsets) {
    if (!q || !cb || !stream || !stream_bytes || !offsets) return ENTRO_ERR_NULL;
    if (!bits_ok(cb->bits)) return ENTRO_ERR_BITS;
    if (n == 0 || chunk_symbols == 0) return ENTRO_ERR_SIZE;
    const uint64_t n_chunks = entro_num_chunks(n, chunk_symbols);
    const int nsym = 1 << cb->bits;
    uint8_t len[256];
    for (int s = 0; s < 256; ++s) len[s] = s < nsym ? cb->len[s] : 0;

    // pass 1: bits per segment, and a check that every symbol has a code
    std::atomic<int> missing{0};
    parallel_ranges(n_chunks, 64, [&](unsigned, uint64_t cb0, uint64_t cb1) {
        for (uint64_t c = cb0; c < cb1; ++c) {
            uint64_t lo = c * chunk_symbols, hi = std::min<uint64_t>(n, lo + chunk_symbols);
            uint64_t bits_here = 0;
            bool miss = false;
            for (uint64_t i = lo; i < hi; ++i) {
                unsigned l = len[q[i]];
                miss |= (l == 0);
                bits_here += l;
            }
            if (miss) missing.store(1, std::memory_order_relaxed);
            offsets[c + 1] = bits_here;
        }
    });
    if (missing.load()) return ENTRO_ERR_SYMBOL;
    offsets[0] = 0;
    for (uint64_t c = 0; c < n_chunks; ++c) offsets[c + 1] += offsets[c];
    const uint64_t total = offsets[n_chunks];
    const uint64_t need = padded_bytes(total);
    if (need > stream_cap) return ENTRO_ERR_CAPACITY;
    if (need >= (uint64_t{1} << 32)) return ENTRO_ERR_SIZE;

    // pass 2: every worker writes a contiguous run of segments into the zeroed stream
    parallel_ranges(need, 1u << 22, [&](unsigned, uint64_t b, uint64_t e) { std::memset(stream + b, 0, e - b); });
    parallel_ranges(n_chunks, 64, [&](unsigned, uint64_t cb0, uint64_t cb1) {
        if (cb0 >= cb1) return;
        BitWriter bw(stream, offsets[cb0]);
        uint64_t lo = cb0 * chunk_symbols, hi = std::min<uint64_t>(n, cb1 * static_cast<uint64_t>(chunk_symbols));
        for (uint64_t i = lo; i < hi; ++i) bw.put(cb->code[q[i]], len[q[i]]);
        bw.finish();
    });
    *stream_bytes = need;
    return ENTRO_OK;
}

entro_status entro_sub_index(const uint8_t *q, uint64_t n, const entro_codebook *cb, uint32_t chunk_symbols,
                             uint32_t sub_symbols, uint16_t *sub_bits) {
    if (!q || !cb || !sub_bits) return ENTRO_ERR_NULL;
    if (!bits_ok(cb->bits)) return ENTRO_ERR_BITS;
    if (n == 0 || chunk_symbols == 0 || sub_symbols == 0 || chunk_symbols % sub_symbols != 0) return ENTRO_ERR_SIZE;
    const uint32_t per = chunk_symbols / sub_symbols;
    if (per > ENTRO_MAX_SUB_PER_CHUNK || (per & (per - 1u)) != 0) return ENTRO_ERR_SIZE;
    const int nsym = 1 << cb->bits;
    uint8_t len[256];
    for (int s = 0; s < 256; ++s) len[s] = s < nsym ? cb->len[s] : 0;
    const uint64_t n_sub = entro_num_chunks(n, sub_symbols);
    std::atomic<int> bad{0};           // 1: a symbol without a code, 2: a piece too long for 16 bits
    parallel_ranges(n_sub, 256, [&](unsigned, uint64_t j0, uint64_t j1) {
        for (uint64_t j = j0; j < j1; ++j) {
            const uint64_t lo = j * sub_symbols, hi = std::min<uint64_t>(n, lo + sub_symbols);
            uint64_t bits_here = 0;
            bool miss = false;
            for (uint64_t i = lo; i < hi; ++i) {
                const unsigned l = len[q[i]];
                miss |= (l == 0);
                bits_here += l;
            }
            if (miss) bad.store(1, std::memory_order_relaxed);
            else if (bits_here > 65535u) bad.store(2, std::memory_order_relaxed);
            sub_bits[j] = static_cast<uint16_t>(bits_here);
        }
    });
    if (bad.load() == 1) return ENTRO_ERR_SYMBOL;
    if (bad.load() == 2) return ENTRO_ERR_CODE_TOO_LONG;
    return ENTRO_OK;
}

entro_status entro_check_offsets(const uint64_t *offsets, uint64_t n, uint32_t chunk_symbols,
                                 uint64_t stream_bytes, const entro_codebook *cb) {
    if (!offsets || !cb) return ENTRO_ERR_NULL;
    if (n == 0 || chunk_symbols == 0) return ENTRO_ERR_SIZE;
    if (cb->max_len < 1 || cb->max_len > ENTRO_MAX_CODE_LEN) return ENTRO_ERR_CORRUPT;
    int min_len = ENTRO_MAX_CODE_LEN;
    for (int s = 0; s < (1 << cb->bits); ++s)
        if (cb->len[s]) min_len = std::min<int>(min_len, cb->len[s]);
    const uint64_t n_chunks = entro_num_chunks(n, chunk_symbols);
    if (offsets[0] != 0) return ENTRO_ERR_CORRUPT;
    for (uint64_t c = 0; c < n_chunks; ++c) {
        if (offsets[c + 1] < offsets[c]) return ENTRO_ERR_CORRUPT;
        uint64_t syms = std::min<uint64_t>(chunk_symbols, n - c * chunk_symbols);
        uint64_t span = offsets[c + 1] - offsets[c];
        if (span > syms * static_cast<uint64_t>(cb->max_len)) return ENTRO_ERR_CORRUPT;
        if (span < syms * static_cast<uint64_t>(min_len)) return ENTRO_ERR_CORRUPT;
    }
    if (stream_bytes < 32 || stream_bytes % 16) return ENTRO_ERR_CORRUPT;
    if ((offsets[n_chunks] + 7) / 8 > stream_bytes - 16) return ENTRO_ERR_CORRUPT;
    return ENTRO_OK;
}

double entro_bits_saved(int bits, double mean_code_len) { return bits - mean_code_len; }

double entro_theoretical_speedup(int bits, double mean_code_len) {
    return mean_code_len > 0.0 ? bits / mean_code_len : 0.0;
}

const char *entro_status_string(entro_status s) {
    switch (s) {
        case ENTRO_OK: return "ok";
        case ENTRO_ERR_NULL: return "null pointer";
        case ENTRO_ERR_BITS: return "bits must be 4 or 8";
        case ENTRO_ERR_SCHEME: return "unknown scheme or output type not valid for this call";
        case ENTRO_ERR_SIZE: return "bad size";
        case ENTRO_ERR_NONFINITE: return "non-finite weight";
        case ENTRO_ERR_RANGE: return "weights outside the range the scheme can represent";
        case ENTRO_ERR_SYMBOL: return "symbol out of range or without a code";
        case ENTRO_ERR_CODE_TOO_LONG: return "code longer than 32 bits";
        case ENTRO_ERR_CAPACITY: return "buffer too small";
        case ENTRO_ERR_CORRUPT: return "inconsistent codebook or offsets";
        case ENTRO_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case ENTRO_ERR_DEVICE: return "HIP error";
    }
    return "unknown status";
}

}  // extern "C"
