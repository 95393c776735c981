// Device side of libentro: segment-parallel Huffman decode for gfx950 with
// fused dequantisation and a fused batch-1 matrix-vector product.
//
// EntroLLM ("Segmentation for parallel Huffman decoding", Fig. 3) cuts the
// encoded parameter space into segments with known boundaries and decodes
// them independently; here a segment is a fixed number of symbols and one
// GPU lane owns one segment, so a 256-lane workgroup decodes 256 consecutive
// segments of one tensor with one shared set of lookup tables in LDS.
#include "entro.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

namespace {

constexpr int kWG = 256;            // lanes (= segments) per workgroup
constexpr int kL1 = 11;             // bits resolved by the first-level table
constexpr uint32_t kL1Mask = (1u << kL1) - 1u;
constexpr int kBatch = 3;           // symbols decoded per 64-bit refill: 64 - 31 >= 3 * kL1
constexpr uint32_t kMaxChunkSymbols = 1u << 20;

// What the kernels read about one tensor.  Lives in kernel arguments (single
// tensor calls) or in the workspace table (batched calls).
struct DevTensor {
    const uint8_t *stream;
    const uint64_t *offsets;
    void *out;
    const uint16_t *x;
    float *partials;            // GEMV: head/tail partial sums, 2 per segment
    uint64_t n;
    uint32_t stream_bytes;
    uint32_t chunk_symbols;
    uint32_t n_chunks;
    uint32_t rows;
    uint32_t cols;
    uint32_t bits;
    float scale;
    int32_t zero_point;
    uint32_t max_len;
    uint32_t need_fix;
    uint8_t len[256];
};

struct WorkItem {
    uint32_t tensor;
    uint32_t first;             // first segment (main kernels) or first row (second-stage sum)
};

enum Mode { kModeU8 = 0, kModeU4 = 1, kModeF32 = 2, kModeBF16 = 3, kModeGemvF32 = 4, kModeGemvBF16 = 5 };

// LDS tables of one workgroup.  First-level entry: symbol | len << 8 | payload << 16,
// len == 0 marks a prefix whose code is longer than kL1 bits.
struct Tables {
    uint32_t lut[1 << kL1];
    uint32_t cnt[ENTRO_MAX_CODE_LEN + 2];
    uint32_t first[ENTRO_MAX_CODE_LEN + 2];
    uint32_t offs[ENTRO_MAX_CODE_LEN + 2];
    uint8_t sorted[256];
    uint8_t lens[256];
};

__device__ __forceinline__ uint32_t bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float dequant(uint32_t sym, int32_t z, float s) {
    return static_cast<float>(static_cast<int32_t>(sym) - z) * s;
}

template <int MODE>
__device__ __forceinline__ uint32_t make_entry(uint32_t sym, uint32_t len, int32_t z, float s) {
    uint32_t e = sym | (len << 8);
    if (MODE == kModeBF16) e |= bf16_bits(dequant(sym, z, s)) << 16;
    return e;
}

// Canonical code tables and the first-level lookup table, built from the 256
// (or 16) code lengths by the whole workgroup.
template <int MODE>
__device__ void build_tables(const DevTensor &t, Tables &tb) {
    const int tid = threadIdx.x;
    const uint32_t l = t.len[tid];
    tb.lens[tid] = static_cast<uint8_t>(l);
    if (tid < ENTRO_MAX_CODE_LEN + 2) tb.cnt[tid] = 0;
    const uint32_t filler = make_entry<MODE>(0, 1, t.zero_point, t.scale);
    for (int i = tid; i < (1 << kL1); i += kWG) tb.lut[i] = filler;
    __syncthreads();
    if (l) atomicAdd(&tb.cnt[l], 1u);
    __syncthreads();
    if (tid == 0) {
        uint64_t code = 0;
        uint32_t off = 0;
        for (int b = 1; b <= ENTRO_MAX_CODE_LEN; ++b) {
            code = (code + (b > 1 ? tb.cnt[b - 1] : 0u)) << 1;
            tb.first[b] = static_cast<uint32_t>(code);
            tb.offs[b] = off;
            off += tb.cnt[b];
        }
    }
    __syncthreads();
    if (l) {
        uint32_t rank = 0;
        for (int s = 0; s < tid; ++s) rank += (tb.lens[s] == l);
        const uint32_t code = tb.first[l] + rank;
        tb.sorted[tb.offs[l] + rank] = static_cast<uint8_t>(tid);
        if (l <= kL1) {
            const uint32_t rev = __brev(code) >> (32 - l);        // first code bit -> bit 0
            const uint32_t e = make_entry<MODE>(tid, l, t.zero_point, t.scale);
            for (uint32_t i = rev; i < (1u << kL1); i += (1u << l)) tb.lut[i] = e;
        } else {
            const uint32_t prefix = code >> (l - kL1);
            tb.lut[__brev(prefix) >> (32 - kL1)] = 0;             // long-code marker
        }
    }
    __syncthreads();
}

// 64 stream bits starting at the dword that holds bit `p` (relative to byte
// `base`), shifted so that bit p is bit 0: at least 33 valid bits.  The read
// is clamped to the last 8 bytes of the (padded) stream.
__device__ __forceinline__ uint64_t load_bits(const uint8_t *stream, uint32_t base, uint32_t p,
                                              uint32_t last_off) {
    uint32_t off = base + ((p >> 5) << 2);
    off = off < last_off ? off : last_off;
    const uint32_t *w = reinterpret_cast<const uint32_t *>(stream + off);
    const uint64_t v = static_cast<uint64_t>(w[0]) | (static_cast<uint64_t>(w[1]) << 32);
    return v >> (p & 31u);
}

// Second level: canonical search over the lengths above kL1.  `window` holds
// the next 32 stream bits, first bit in bit 0.
template <int MODE>
__device__ __noinline__ uint32_t decode_long(const Tables &tb, uint32_t window, uint32_t max_len,
                                             int32_t z, float s) {
    const uint32_t v = __brev(window);
    for (uint32_t l = kL1 + 1; l <= max_len; ++l) {
        const uint32_t d = (v >> (32 - l)) - tb.first[l];
        if (d < tb.cnt[l]) return make_entry<MODE>(tb.sorted[tb.offs[l] + d], l, z, s);
    }
    return make_entry<MODE>(0, 1, z, s);     // not a code (corrupt stream): keep moving
}

// Per-lane reader of one segment.
struct Reader {
    const uint8_t *stream;
    uint32_t base;       // dword-aligned byte offset of the segment start
    uint32_t last_off;   // stream_bytes - 8
    uint32_t p;          // bit position relative to base
    uint64_t buf;
};

template <int MODE>
__device__ __forceinline__ uint32_t next_symbol(Reader &r, const Tables &tb, const DevTensor &t) {
    uint32_t e = tb.lut[static_cast<uint32_t>(r.buf) & kL1Mask];
    if (__builtin_expect((e & 0xff00u) == 0, 0)) {
        const uint64_t w = load_bits(r.stream, r.base, r.p, r.last_off);
        e = decode_long<MODE>(tb, static_cast<uint32_t>(w), t.max_len, t.zero_point, t.scale);
        r.p += (e >> 8) & 0xffu;
        r.buf = load_bits(r.stream, r.base, r.p, r.last_off);
    } else {
        const uint32_t len = (e >> 8) & 0xffu;
        r.buf >>= len;
        r.p += len;
    }
    return e;
}

template <int MODE> struct OutTraits;
template <> struct OutTraits<kModeU8> { static constexpr int group = 16; static constexpr int ebits = 8; };
template <> struct OutTraits<kModeU4> { static constexpr int group = 32; static constexpr int ebits = 4; };
template <> struct OutTraits<kModeF32> { static constexpr int group = 4; static constexpr int ebits = 32; };
template <> struct OutTraits<kModeBF16> { static constexpr int group = 8; static constexpr int ebits = 16; };

// Decode one segment and write it in the output type of MODE.
template <int MODE>
__device__ __forceinline__ void decode_segment(const DevTensor &t, const Tables &tb, uint32_t k) {
    constexpr int G = OutTraits<MODE>::group;
    const uint32_t C = t.chunk_symbols;
    const uint64_t first_sym = static_cast<uint64_t>(k) * C;
    const uint64_t left = t.n - first_sym;
    const uint32_t nsym = left < C ? static_cast<uint32_t>(left) : C;
    const uint64_t off_bits = t.offsets[k];
    Reader r;
    r.stream = t.stream;
    r.last_off = t.stream_bytes - 8u;
    r.base = static_cast<uint32_t>(off_bits >> 3) & ~3u;
    r.p = static_cast<uint32_t>(off_bits - (static_cast<uint64_t>(r.base) << 3));
    r.buf = 0;

    // 16-byte stores need every segment to start on a 16-byte boundary
    const bool vec_ok = ((static_cast<uint64_t>(C) * OutTraits<MODE>::ebits) & 127u) == 0;
    uint8_t *out8 = static_cast<uint8_t *>(t.out);
    uint32_t i = 0;
    if (vec_ok) {
        uint4 *dst = reinterpret_cast<uint4 *>(out8 + ((first_sym * OutTraits<MODE>::ebits) >> 3));
        for (; i + G <= nsym; i += G) {
            uint32_t v[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < G; ++j) {
                if (j % kBatch == 0) r.buf = load_bits(r.stream, r.base, r.p, r.last_off);
                const uint32_t e = next_symbol<MODE>(r, tb, t);
                if (MODE == kModeU8) v[j >> 2] |= (e & 0xffu) << ((j & 3) * 8);
                if (MODE == kModeU4) v[j >> 3] |= (e & 0xfu) << ((j & 7) * 4);
                if (MODE == kModeBF16) v[j >> 1] |= (j & 1) ? (e & 0xffff0000u) : (e >> 16);
                if (MODE == kModeF32) v[j] = __float_as_uint(dequant(e & 0xffu, t.zero_point, t.scale));
            }
            *dst++ = make_uint4(v[0], v[1], v[2], v[3]);
        }
    }
    // ragged tail, or segments that are not 16-byte aligned: element by element
    uint32_t pending = 0;     // low nibble waiting for its partner (packed 4-bit)
    for (; i < nsym; ++i) {
        r.buf = load_bits(r.stream, r.base, r.p, r.last_off);
        const uint32_t e = next_symbol<MODE>(r, tb, t);
        const uint64_t idx = first_sym + i;
        if (MODE == kModeU8) out8[idx] = static_cast<uint8_t>(e);
        if (MODE == kModeU4) {
            if (idx & 1) out8[idx >> 1] = static_cast<uint8_t>(pending | ((e & 0xfu) << 4));
            else pending = e & 0xfu;
        }
        if (MODE == kModeBF16) reinterpret_cast<uint16_t *>(t.out)[idx] = static_cast<uint16_t>(e >> 16);
        if (MODE == kModeF32) reinterpret_cast<float *>(t.out)[idx] = dequant(e & 0xffu, t.zero_point, t.scale);
    }
    if (MODE == kModeU4 && (nsym & 1)) out8[(first_sym + nsym - 1) >> 1] = static_cast<uint8_t>(pending);
}

// Decode one segment straight into dot products with x.  A segment covers one
// or more row fragments; complete rows are stored, a leading / trailing
// incomplete fragment goes to the segment's head / tail partial.
template <int MODE>
__device__ __forceinline__ void gemv_segment(const DevTensor &t, const Tables &tb, uint32_t k) {
    const uint32_t C = t.chunk_symbols;
    const uint64_t first_sym = static_cast<uint64_t>(k) * C;
    const uint64_t left = t.n - first_sym;
    const uint32_t nsym = left < C ? static_cast<uint32_t>(left) : C;
    const uint64_t off_bits = t.offsets[k];
    Reader r;
    r.stream = t.stream;
    r.last_off = t.stream_bytes - 8u;
    r.base = static_cast<uint32_t>(off_bits >> 3) & ~3u;
    r.p = static_cast<uint32_t>(off_bits - (static_cast<uint64_t>(r.base) << 3));
    r.buf = 0;

    uint32_t row = static_cast<uint32_t>(first_sym / t.cols);
    uint32_t col = static_cast<uint32_t>(first_sym - static_cast<uint64_t>(row) * t.cols);
    const uint32_t start_col = col;
    bool first_fragment = true;
    float acc = 0.0f;
    float head = 0.0f, tail = 0.0f;
    for (uint32_t i = 0; i < nsym; ++i) {
        if (i % kBatch == 0) r.buf = load_bits(r.stream, r.base, r.p, r.last_off);
        const uint32_t e = next_symbol<MODE>(r, tb, t);
        const float xv = __uint_as_float(static_cast<uint32_t>(t.x[col]) << 16);
        acc = fmaf(static_cast<float>(static_cast<int32_t>(e & 0xffu) - t.zero_point), xv, acc);
        if (++col == t.cols) {
            if (first_fragment && start_col != 0) {
                head = acc;                                  // row began in an earlier segment
            } else {
                const float y = acc * t.scale;
                if (MODE == kModeGemvF32) reinterpret_cast<float *>(t.out)[row] = y;
                else reinterpret_cast<uint16_t *>(t.out)[row] = static_cast<uint16_t>(bf16_bits(y));
            }
            first_fragment = false;
            acc = 0.0f;
            col = 0;
            ++row;
        }
    }
    if (col != 0) {                                          // row continues in the next segment
        if (first_fragment) head = acc;
        else tail = acc;
    }
    if (t.need_fix) {
        t.partials[2 * static_cast<uint64_t>(k)] = head;
        t.partials[2 * static_cast<uint64_t>(k) + 1] = tail;
    }
}

template <int MODE>
__device__ __forceinline__ void run_item(const DevTensor &t, uint32_t first_chunk, Tables &tb) {
    build_tables<MODE>(t, tb);
    const uint32_t k = first_chunk + threadIdx.x;
    if (k >= t.n_chunks) return;
    if constexpr (MODE == kModeGemvF32 || MODE == kModeGemvBF16) gemv_segment<MODE>(t, tb, k);
    else decode_segment<MODE>(t, tb, k);
}

template <int MODE>
__global__ __launch_bounds__(kWG) void k_single(const DevTensor t) {
    __shared__ Tables tb;
    run_item<MODE>(t, blockIdx.x * kWG, tb);
}

template <int MODE>
__global__ __launch_bounds__(kWG) void k_batch(const DevTensor *__restrict__ tensors,
                                               const WorkItem *__restrict__ items) {
    __shared__ Tables tb;
    const WorkItem it = items[blockIdx.x];
    run_item<MODE>(tensors[it.tensor], it.first, tb);
}

// Second stage of the GEMV: rows that straddle segments are summed in segment order.
template <int MODE>
__device__ __forceinline__ void fix_row(const DevTensor &t, uint32_t row) {
    if (row >= t.rows) return;
    const uint64_t lo = static_cast<uint64_t>(row) * t.cols;
    const uint64_t hi = lo + t.cols - 1;
    const uint32_t k_lo = static_cast<uint32_t>(lo / t.chunk_symbols);
    const uint32_t k_hi = static_cast<uint32_t>(hi / t.chunk_symbols);
    if (k_lo == k_hi) return;                                 // whole row inside one segment: already stored
    float acc = 0.0f;
    for (uint32_t k = k_lo; k <= k_hi; ++k) {
        const uint32_t first_row = static_cast<uint32_t>((static_cast<uint64_t>(k) * t.chunk_symbols) / t.cols);
        acc += t.partials[2 * static_cast<uint64_t>(k) + (first_row == row ? 0 : 1)];
    }
    const float y = acc * t.scale;
    if (MODE == kModeGemvF32) reinterpret_cast<float *>(t.out)[row] = y;
    else reinterpret_cast<uint16_t *>(t.out)[row] = static_cast<uint16_t>(bf16_bits(y));
}

template <int MODE>
__global__ __launch_bounds__(kWG) void k_fix_single(const DevTensor t) {
    fix_row<MODE>(t, blockIdx.x * kWG + threadIdx.x);
}

template <int MODE>
__global__ __launch_bounds__(kWG) void k_fix_batch(const DevTensor *__restrict__ tensors,
                                                   const WorkItem *__restrict__ items) {
    const WorkItem it = items[blockIdx.x];
    fix_row<MODE>(tensors[it.tensor], it.first + threadIdx.x);
}

// ------------------------------------------------------------------ host glue
thread_local std::string g_last_error;

bool hip_ok(hipError_t e, const char *what) {
    if (e == hipSuccess) return true;
    g_last_error = std::string(what) + ": " + hipGetErrorString(e);
    return false;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool dtype_ok(entro_op op, entro_dtype d, int bits) {
    if (op == ENTRO_OP_DECODE) return d == ENTRO_U8 || (d == ENTRO_U4_PACKED && bits == 4);
    return d == ENTRO_F32 || d == ENTRO_BF16;
}

// Re-derive the canonical codes from the lengths and compare: the kernels
// rebuild the code from lengths alone, so the two must agree.
entro_status check_codebook(const entro_codebook *cb) {
    if (!cb) return ENTRO_ERR_NULL;
    if (cb->bits != 4 && cb->bits != 8) return ENTRO_ERR_BITS;
    entro_codebook ref;
    entro_status st = entro_codebook_from_lengths(cb->len, cb->bits, &ref);
    if (st != ENTRO_OK) return st == ENTRO_ERR_SIZE ? ENTRO_ERR_CORRUPT : st;
    for (int s = 0; s < (1 << cb->bits); ++s)
        if (ref.code[s] != cb->code[s]) return ENTRO_ERR_CORRUPT;
    for (int s = (1 << cb->bits); s < ENTRO_MAX_SYMBOLS; ++s)
        if (cb->len[s]) return ENTRO_ERR_CORRUPT;
    if (ref.max_len != cb->max_len) return ENTRO_ERR_CORRUPT;
    return ENTRO_OK;
}

entro_status fill_dev_tensor(const entro_tensor *t, entro_op op, entro_dtype d, DevTensor *dt) {
    if (!t || !t->stream || !t->offsets || !t->out || !t->cb) return ENTRO_ERR_NULL;
    entro_status st = check_codebook(t->cb);
    if (st != ENTRO_OK) return st;
    const int bits = t->cb->bits;
    if (!dtype_ok(op, d, bits)) return ENTRO_ERR_SCHEME;
    if (t->n == 0 || t->chunk_symbols == 0 || t->chunk_symbols > kMaxChunkSymbols) return ENTRO_ERR_SIZE;
    if (d == ENTRO_U4_PACKED && (t->chunk_symbols & 1u)) return ENTRO_ERR_SIZE;
    if (t->stream_bytes < 32 || (t->stream_bytes & 15u) || t->stream_bytes >= (uint64_t{1} << 32))
        return ENTRO_ERR_SIZE;
    const uint64_t n_chunks = entro_num_chunks(t->n, t->chunk_symbols);
    if (n_chunks >= (uint64_t{1} << 32) - kWG) return ENTRO_ERR_SIZE;
    if (!aligned16(t->stream) || !aligned16(t->offsets) || !aligned16(t->out)) return ENTRO_ERR_ALIGN;
    if (op != ENTRO_OP_DECODE && t->qp.bits != bits) return ENTRO_ERR_BITS;
    if (op == ENTRO_OP_GEMV) {
        if (!t->x) return ENTRO_ERR_NULL;
        if (!aligned16(t->x)) return ENTRO_ERR_ALIGN;
        if (t->rows == 0 || t->cols == 0 || static_cast<uint64_t>(t->rows) * t->cols != t->n)
            return ENTRO_ERR_SIZE;
    }
    std::memset(dt, 0, sizeof(*dt));
    dt->stream = static_cast<const uint8_t *>(t->stream);
    dt->offsets = t->offsets;
    dt->out = t->out;
    dt->x = static_cast<const uint16_t *>(t->x);
    dt->n = t->n;
    dt->stream_bytes = static_cast<uint32_t>(t->stream_bytes);
    dt->chunk_symbols = t->chunk_symbols;
    dt->n_chunks = static_cast<uint32_t>(n_chunks);
    dt->rows = t->rows;
    dt->cols = t->cols;
    dt->bits = static_cast<uint32_t>(bits);
    dt->scale = t->qp.scale;
    dt->zero_point = t->qp.zero_point;
    dt->max_len = static_cast<uint32_t>(t->cb->max_len);
    dt->need_fix = (op == ENTRO_OP_GEMV && (t->chunk_symbols % t->cols) != 0) ? 1u : 0u;
    std::memcpy(dt->len, t->cb->len, 256);
    return ENTRO_OK;
}

int mode_of(entro_op op, entro_dtype d) {
    if (op == ENTRO_OP_GEMV) return d == ENTRO_F32 ? kModeGemvF32 : kModeGemvBF16;
    switch (d) {
        case ENTRO_U8: return kModeU8;
        case ENTRO_U4_PACKED: return kModeU4;
        case ENTRO_F32: return kModeF32;
        default: return kModeBF16;
    }
}

template <class F>
void dispatch_mode(int mode, F f) {
    switch (mode) {
        case kModeU8: f(std::integral_constant<int, kModeU8>{}); break;
        case kModeU4: f(std::integral_constant<int, kModeU4>{}); break;
        case kModeF32: f(std::integral_constant<int, kModeF32>{}); break;
        case kModeBF16: f(std::integral_constant<int, kModeBF16>{}); break;
        case kModeGemvF32: f(std::integral_constant<int, kModeGemvF32>{}); break;
        default: f(std::integral_constant<int, kModeGemvBF16>{}); break;
    }
}

entro_status launch_single(const entro_tensor *t, entro_op op, entro_dtype d, float *partials,
                           void *hip_stream) {
    DevTensor dt;
    entro_status st = fill_dev_tensor(t, op, d, &dt);
    if (st != ENTRO_OK) return st;
    dt.partials = partials;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const unsigned grid = (dt.n_chunks + kWG - 1) / kWG;
    const int mode = mode_of(op, d);
    dispatch_mode(mode, [&](auto m) { hipLaunchKernelGGL(k_single<decltype(m)::value>, dim3(grid), dim3(kWG), 0, s, dt); });
    if (!hip_ok(hipGetLastError(), "launch decode kernel")) return ENTRO_ERR_DEVICE;
    if (dt.need_fix) {
        const unsigned g2 = (dt.rows + kWG - 1) / kWG;
        if (mode == kModeGemvF32) hipLaunchKernelGGL(k_fix_single<kModeGemvF32>, dim3(g2), dim3(kWG), 0, s, dt);
        else hipLaunchKernelGGL(k_fix_single<kModeGemvBF16>, dim3(g2), dim3(kWG), 0, s, dt);
        if (!hip_ok(hipGetLastError(), "launch row-sum kernel")) return ENTRO_ERR_DEVICE;
    }
    return ENTRO_OK;
}

uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

struct Layout {
    uint64_t off_tensors, off_items, off_fix, off_partials, total;
    uint32_t n_items, n_fix;
};

// Workspace layout shared by entro_workspace_bytes and entro_plan_init.
bool plan_layout(const entro_tensor *ts, uint32_t count, entro_op op, Layout *L) {
    uint64_t items = 0, fix = 0, partial_floats = 0;
    for (uint32_t i = 0; i < count; ++i) {
        if (ts[i].chunk_symbols == 0 || ts[i].n == 0) return false;
        const uint64_t nc = entro_num_chunks(ts[i].n, ts[i].chunk_symbols);
        items += (nc + kWG - 1) / kWG;
        if (op == ENTRO_OP_GEMV && ts[i].cols && (ts[i].chunk_symbols % ts[i].cols) != 0) {
            fix += (static_cast<uint64_t>(ts[i].rows) + kWG - 1) / kWG;
            partial_floats += 2 * nc;
        }
    }
    if (items >= (uint64_t{1} << 31) || fix >= (uint64_t{1} << 31)) return false;
    L->n_items = static_cast<uint32_t>(items);
    L->n_fix = static_cast<uint32_t>(fix);
    L->off_tensors = 0;
    L->off_items = align_up(sizeof(DevTensor) * static_cast<uint64_t>(count), 256);
    L->off_fix = L->off_items + align_up(sizeof(WorkItem) * items, 256);
    L->off_partials = L->off_fix + align_up(sizeof(WorkItem) * fix, 256);
    L->total = L->off_partials + align_up(sizeof(float) * partial_floats, 256);
    return true;
}

}  // namespace

extern "C" {

const char *entro_last_device_error(void) { return g_last_error.c_str(); }

entro_status entro_decode(const entro_tensor *t, entro_dtype out_type, void *hip_stream) {
    return launch_single(t, ENTRO_OP_DECODE, out_type, nullptr, hip_stream);
}

entro_status entro_decode_dequant(const entro_tensor *t, entro_dtype out_type, void *hip_stream) {
    return launch_single(t, ENTRO_OP_DEQUANT, out_type, nullptr, hip_stream);
}

uint64_t entro_gemv_workspace_bytes(const entro_tensor *t) {
    if (!t || t->chunk_symbols == 0 || t->cols == 0) return 0;
    if ((t->chunk_symbols % t->cols) == 0) return 0;
    return align_up(2 * sizeof(float) * entro_num_chunks(t->n, t->chunk_symbols), 256);
}

entro_status entro_decode_gemv(const entro_tensor *t, entro_dtype y_type, void *workspace,
                               uint64_t workspace_bytes, void *hip_stream) {
    if (!t) return ENTRO_ERR_NULL;
    const uint64_t need = entro_gemv_workspace_bytes(t);
    if (need) {
        if (!workspace) return ENTRO_ERR_NULL;
        if (workspace_bytes < need) return ENTRO_ERR_CAPACITY;
        if (!aligned16(workspace)) return ENTRO_ERR_ALIGN;
    }
    return launch_single(t, ENTRO_OP_GEMV, y_type, static_cast<float *>(workspace), hip_stream);
}

uint64_t entro_workspace_bytes(const entro_tensor *ts, uint32_t count, entro_op op) {
    Layout L;
    if (!ts || count == 0 || !plan_layout(ts, count, op, &L)) return 0;
    return L.total;
}

entro_status entro_plan_init(entro_plan *plan, const entro_tensor *ts, uint32_t count, entro_op op,
                             entro_dtype out_type, void *workspace, uint64_t workspace_bytes,
                             void *hip_stream) {
    if (!plan || !ts || !workspace) return ENTRO_ERR_NULL;
    if (count == 0) return ENTRO_ERR_SIZE;
    if (op != ENTRO_OP_DECODE && op != ENTRO_OP_DEQUANT && op != ENTRO_OP_GEMV) return ENTRO_ERR_SCHEME;
    if (!aligned16(workspace)) return ENTRO_ERR_ALIGN;
    Layout L;
    if (!plan_layout(ts, count, op, &L)) return ENTRO_ERR_SIZE;
    if (workspace_bytes < L.total) return ENTRO_ERR_CAPACITY;

    std::vector<unsigned char> host(L.off_partials, 0);
    DevTensor *dts = reinterpret_cast<DevTensor *>(host.data() + L.off_tensors);
    WorkItem *items = reinterpret_cast<WorkItem *>(host.data() + L.off_items);
    WorkItem *fix = reinterpret_cast<WorkItem *>(host.data() + L.off_fix);
    uint64_t n_items = 0, n_fix = 0, partial_floats = 0;
    float *partials_base = reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + L.off_partials);
    for (uint32_t i = 0; i < count; ++i) {
        entro_status st = fill_dev_tensor(&ts[i], op, out_type, &dts[i]);
        if (st != ENTRO_OK) return st;
        for (uint32_t c = 0; c < dts[i].n_chunks; c += kWG) items[n_items++] = WorkItem{i, c};
        if (dts[i].need_fix) {
            dts[i].partials = partials_base + partial_floats;
            partial_floats += 2 * static_cast<uint64_t>(dts[i].n_chunks);
            for (uint32_t r = 0; r < dts[i].rows; r += kWG) fix[n_fix++] = WorkItem{i, r};
        }
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (!hip_ok(hipMemcpyAsync(workspace, host.data(), host.size(), hipMemcpyHostToDevice, s), "copy plan table"))
        return ENTRO_ERR_DEVICE;
    // the staging vector dies with this call, so wait for the copy
    if (!hip_ok(hipStreamSynchronize(s), "wait for plan table")) return ENTRO_ERR_DEVICE;
    plan->workspace = workspace;
    plan->workspace_bytes = workspace_bytes;
    plan->op = op;
    plan->out = out_type;
    plan->count = count;
    plan->n_items = L.n_items;
    plan->n_fix = L.n_fix;
    plan->flags = 0;
    plan->off_tensors = L.off_tensors;
    plan->off_items = L.off_items;
    plan->off_partials = L.off_partials;
    plan->off_fix = L.off_fix;
    return ENTRO_OK;
}

entro_status entro_plan_run(const entro_plan *plan, void *hip_stream) {
    if (!plan || !plan->workspace) return ENTRO_ERR_NULL;
    if (plan->n_items == 0) return ENTRO_ERR_SIZE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const unsigned char *ws = static_cast<const unsigned char *>(plan->workspace);
    const DevTensor *dts = reinterpret_cast<const DevTensor *>(ws + plan->off_tensors);
    const WorkItem *items = reinterpret_cast<const WorkItem *>(ws + plan->off_items);
    const WorkItem *fix = reinterpret_cast<const WorkItem *>(ws + plan->off_fix);
    const int mode = mode_of(static_cast<entro_op>(plan->op), static_cast<entro_dtype>(plan->out));
    dispatch_mode(mode, [&](auto m) {
        hipLaunchKernelGGL(k_batch<decltype(m)::value>, dim3(plan->n_items), dim3(kWG), 0, s, dts, items);
    });
    if (!hip_ok(hipGetLastError(), "launch batched decode kernel")) return ENTRO_ERR_DEVICE;
    if (plan->n_fix) {
        if (mode == kModeGemvF32) hipLaunchKernelGGL(k_fix_batch<kModeGemvF32>, dim3(plan->n_fix), dim3(kWG), 0, s, dts, fix);
        else hipLaunchKernelGGL(k_fix_batch<kModeGemvBF16>, dim3(plan->n_fix), dim3(kWG), 0, s, dts, fix);
        if (!hip_ok(hipGetLastError(), "launch batched row-sum kernel")) return ENTRO_ERR_DEVICE;
    }
    return ENTRO_OK;
}

static entro_status run_batch(const entro_tensor *ts, uint32_t count, entro_op op, entro_dtype d,
                              void *workspace, uint64_t workspace_bytes, void *hip_stream) {
    entro_plan plan;
    entro_status st = entro_plan_init(&plan, ts, count, op, d, workspace, workspace_bytes, hip_stream);
    if (st != ENTRO_OK) return st;
    return entro_plan_run(&plan, hip_stream);
}

entro_status entro_decode_batch(const entro_tensor *ts, uint32_t count, entro_dtype out_type,
                                void *workspace, uint64_t workspace_bytes, void *hip_stream) {
    return run_batch(ts, count, ENTRO_OP_DECODE, out_type, workspace, workspace_bytes, hip_stream);
}

entro_status entro_decode_dequant_batch(const entro_tensor *ts, uint32_t count, entro_dtype out_type,
                                        void *workspace, uint64_t workspace_bytes, void *hip_stream) {
    return run_batch(ts, count, ENTRO_OP_DEQUANT, out_type, workspace, workspace_bytes, hip_stream);
}

entro_status entro_decode_gemv_batch(const entro_tensor *ts, uint32_t count, entro_dtype y_type,
                                     void *workspace, uint64_t workspace_bytes, void *hip_stream) {
    return run_batch(ts, count, ENTRO_OP_GEMV, y_type, workspace, workspace_bytes, hip_stream);
}

}  // extern "C"
