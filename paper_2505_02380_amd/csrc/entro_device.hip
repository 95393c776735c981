// Device side of libentro: segment-parallel Huffman decode for gfx950 with
// fused dequantisation and a fused batch-1 matrix-vector product.
//
// EntroLLM ("Segmentation for parallel Huffman decoding", Fig. 3) cuts the
// encoded parameter space into segments with known boundaries and decodes
// them independently; here a segment is a fixed number of symbols and one
// GPU lane owns one segment, so a workgroup of W lanes decodes W consecutive
// segments of one tensor with one shared set of lookup tables in LDS.
//
// Data flow of the decode / dequant kernels, per lane:
//   HBM --128-byte lines (GEMV: 64)--> registers --between output blocks--> 128-byte ring in LDS
//   ring --three dwords--> 63-bit window --14 bits--> first-level table (LDS,
//   16-bit entries: length | symbol) --shift by the entry--> next code ...
//   four symbols --one aligned dword--> the lane's row of the wave's LDS tile
//   tile rows --dequantise / pack, row-wise--> HBM,
// so that every global store instruction of a wave covers whole rows (the GEMV
// has no tile: a lane multiplies its four symbols into x as they come).  All 64
// lanes of a wave decode in step, four symbols per window: no lane waits for
// another, nothing is written to LDS at an odd address, and a flush happens
// after a fixed number of groups.  The symbol loop has no branch per lookup; a
// lane that meets a code too long for the first-level table stops moving for the
// rest of its group, and the wave then finishes that group for it with the
// second-level table or a canonical search.
#include "entro.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <type_traits>
#include <vector>

// Partial sums of entro_decode_gemv_static: two floats per segment.  Every GPU the library runs on holds
// its own copy of this array until the process ends.  In host code the name stands for the symbol only;
// the array's address on a device comes from hipGetSymbolAddress (static_scratch below).
static __device__ __align__(256) float scratch[2 * ENTRO_STATIC_GEMV_MAX_SEGMENTS];

namespace {

constexpr int kL1 = 14;                  // stream bits that index the first-level table
constexpr uint32_t kL1Mask = (1u << kL1) - 1u;
constexpr int kL2Cap = 512;              // second-level entries (all long prefixes together)
constexpr int kL2MaxBits = 6;            // the second level resolves codes of up to kL1 + 6 = 20 bits
constexpr int kL2MaxPrefixes = 32;       // more long prefixes than this: second level unused (32 blocks of 16 fill it)
constexpr int kSingleBits = 9;             // pair tables: index bits of the table of single codes
constexpr uint32_t kUnit = 64;           // segments a wavefront decodes at a time: one per lane
constexpr int kGroup = 4;                // symbols per ring read: 63 valid bits >= 4 * 14
constexpr uint32_t kTailShift = 4;       // a stretch's last round is drawn with lanes up to 2^this times finer
constexpr int kTripGroups = 4;           // ring reads between two checks of the ring's fill
constexpr int kScalarProbes = 2;         // scalar reader: symbols per 64-bit load, 33 valid bits >= 2 * kL1
constexpr int kRingBits = 1024;          // a lane's ring: two 64-byte lines (eight 16-byte blocks)
constexpr int kRingDwords = kRingBits / 32 + 2;   // and two mirror dwords
constexpr int kRing2Bits = 512;          // the short ring: four blocks
constexpr int kRing2Dwords = kRing2Bits / 32 + 2;
constexpr int kGroupBits = kGroup * kL1;           // most stream bits a group takes through the first level
constexpr int kTripBits = (kTripGroups - 1) * kGroupBits + 64;   // a trip's last ring read ends this far past its start
constexpr uint32_t kMaxChunkSymbols = 1u << 20;
static_assert(kGroup * kL1 <= 63 && kGroup == 4, "a group packs four symbol bytes into one dword");

// What the kernels read about one tensor.  Lives in kernel arguments (single
// tensor calls) or in the workspace table (batched calls).
struct DevTensor {
    const uint8_t *stream;
    const uint64_t *offsets;
    void *out;
    const uint16_t *x;
    float *partials;            // GEMV: head/tail partial sums, 2 per segment
    const uint16_t *sub;        // entry points inside the segments: stream bits of every piece (or null)
    void *tables;               // batched launches: the tensor's lookup tables as k_tables left them (or null: build them)
    uint64_t n;
    uint32_t stream_bytes;
    uint32_t chunk_symbols;     // symbols one lane decodes: a piece, where the tensor has entry points, else a segment
    uint32_t n_chunks;          // and how many of those the tensor has
    uint32_t sub_shift;         // log2 of lanes per segment (0: a lane takes a whole segment)
    uint32_t sub_merge;         // log2 of the pieces of the entry-point table that one lane takes
    uint32_t rows;
    uint32_t cols;
    uint32_t bits;
    float scale;
    int32_t zero_point;
    uint32_t max_len;
    uint32_t need_fix;
    uint32_t row_lanes;         // GEMV: lanes per matrix row where a wavefront sums its rows by itself (0: not so)
    uint32_t fine;              // batched launches: index of the same tensor's description with finer lanes (0: none)
    uint32_t fine_shift;        // log2 of how many of those lanes make one of this description's
    uint8_t len[256];
};

struct WorkItem {
    uint32_t tensor;
    uint32_t first;             // first segment (main kernels) or first row (second-stage sum)
};

// The P modes are the byte, fp32 and bf16 outputs and the GEMV of launches whose tensors all hold
// 4-bit symbols: they decode two symbols per lookup, like the packed output.
// The W modes are the GEMV on wide tables (8-bit symbols, zero-point within [-1, 256]): gemv_direct2.
enum Mode { kModeU8 = 0, kModeU4 = 1, kModeF32 = 2, kModeBF16 = 3, kModeGemvF32 = 4, kModeGemvBF16 = 5,
            kModeU8P = 6, kModeF32P = 7, kModeBF16P = 8, kModeGemvF32P = 9, kModeGemvBF16P = 10,
            kModeGemvF32W = 11, kModeGemvBF16W = 12 };
constexpr bool gemv_f32(int mode) { return mode == kModeGemvF32 || mode == kModeGemvF32P || mode == kModeGemvF32W; }
constexpr bool is_gemv(int mode) {
    return gemv_f32(mode) || mode == kModeGemvBF16 || mode == kModeGemvBF16P || mode == kModeGemvBF16W;
}
constexpr bool wide_gemv(int mode) { return mode == kModeGemvF32W || mode == kModeGemvBF16W; }
// the output format of a mode
constexpr int base_mode(int mode) { return mode == kModeU8P ? kModeU8 : mode == kModeF32P ? kModeF32 : mode == kModeBF16P ? kModeBF16 : mode; }

// Per output mode: symbols of a lane that one flush takes, bytes of its tile row
// (one per table lookup: a symbol, or two 4-bit symbols already packed), waves
// per workgroup (what fits into the 160 KB of LDS), tile bytes one lane consumes
// per flush pass (a 16-byte store for all but fp32) and bytes that a row becomes
// in memory.  The host glue sizes its launches with the same numbers.  The GEMV
// has no tile (only spb, the symbols between two ring refills, and waves count).
template <int MODE> struct Cfg;
template <> struct Cfg<kModeU8> { static constexpr int spb = 64, row = 64, waves = 14, piece = 16, out_row = 64; };
template <> struct Cfg<kModeU4> { static constexpr int spb = 128, row = 64, waves = 14, piece = 16, out_row = 64; };
template <> struct Cfg<kModeF32> { static constexpr int spb = 64, row = 64, waves = 16, piece = 8, out_row = 256; };
template <> struct Cfg<kModeBF16> { static constexpr int spb = 64, row = 64, waves = 16, piece = 8, out_row = 128; };
template <> struct Cfg<kModeGemvF32> { static constexpr int spb = 64, row = 64, waves = 14, piece = 8, out_row = 0; };
template <> struct Cfg<kModeGemvBF16> { static constexpr int spb = 64, row = 64, waves = 14, piece = 8, out_row = 0; };
template <> struct Cfg<kModeGemvF32P> { static constexpr int spb = 128, row = 64, waves = 14, piece = 8, out_row = 0; };
template <> struct Cfg<kModeGemvBF16P> { static constexpr int spb = 128, row = 64, waves = 14, piece = 8, out_row = 0; };
template <> struct Cfg<kModeGemvF32W> { static constexpr int spb = 64, row = 64, waves = 16, piece = 8, out_row = 0; };
template <> struct Cfg<kModeGemvBF16W> { static constexpr int spb = 64, row = 64, waves = 16, piece = 8, out_row = 0; };
template <> struct Cfg<kModeU8P> { static constexpr int spb = 128, row = 64, waves = 14, piece = 16, out_row = 128; };
template <> struct Cfg<kModeF32P> { static constexpr int spb = 128, row = 64, waves = 14, piece = 8, out_row = 512; };
template <> struct Cfg<kModeBF16P> { static constexpr int spb = 128, row = 64, waves = 14, piece = 8, out_row = 256; };
// Packed 4-bit output decodes two symbols per lookup, and so do the P modes.
template <int MODE> constexpr bool kPairMode = MODE == kModeU4 || MODE == kModeU8P || MODE == kModeF32P || MODE == kModeBF16P ||
                                               MODE == kModeGemvF32P || MODE == kModeGemvBF16P;

// Lookup tables of one workgroup (LDS).
// Entry (16 bits): bits 0..5 the code's length, bits 8..15 its symbol, so that an
// entry serves as a 64-bit shift amount as it stands.
// First level: indexed by the next kL1 stream bits.  A zero length marks a prefix
// whose code is longer than kL1 bits (a lane that looks one up does not move);
// the whole low byte is zero then, bits 8..10 are the depth of the prefix's block
// in the second level (7: it has none) and bits 11..15 the block's start in units
// of sixteen entries.
// Second level: per long prefix a block indexed by the following `depth` stream
// bits; zero there sends the lane to the canonical search
// (first / cnt / offs / sorted).
// Pair tables (packed 4-bit output): a first-level entry holds the next TWO codes
// where both fit into the kL1 index bits, their lengths added up and the two
// symbols packed the way the output wants them (first one in the low nibble); a
// zero entry otherwise.  There is no second level then; lut2 starts with a
// table of single codes up to kSingleBits long instead, for what the pair table
// leaves out and for the element-by-element paths.
struct alignas(16) TablesTail {
    uint16_t lut2[kL2Cap];
    uint32_t cnt[ENTRO_MAX_CODE_LEN + 2];
    uint32_t first[ENTRO_MAX_CODE_LEN + 2];
    uint32_t offs[ENTRO_MAX_CODE_LEN + 2];
    uint32_t pdepth[kL2MaxPrefixes];     // per long prefix: bits its second-level block resolves
    uint32_t pbase[kL2MaxPrefixes];      // and where the block starts (a multiple of 16)
    uint32_t first_prefix;               // smallest kL1-bit prefix of a long code; 2^kL1 if level 2 is unused
    uint32_t long_start;                 // the same, but kept when level 2 is unused
    uint32_t pad[2];
    uint8_t sorted[256];
};
// E: the first level's entry.  16 bits: as described above.  32 bits (the GEMV's wide tables): the same in the
// low half and, in the high half, the value the symbol contributes, ready for use: bf16(symbol - zero_point),
// which is exact (an integer of at most 256 in magnitude), so that the product needs neither a conversion
// nor a subtraction per symbol.  A window that is to index 32-bit entries carries two stale low bits.
template <class E>
struct alignas(16) TablesT : TablesTail {
    static constexpr uint32_t stale = sizeof(E) == 2 ? 1u : 2u;
    E lut[1 << kL1];
};
using Tables = TablesT<uint16_t>;
using Tables32 = TablesT<uint32_t>;

// Per-wave LDS: the lanes' stream rings and their output rows.
// The ring is stored dword-major (dword d of lane l at d * 64 + l): whatever
// dword each lane reads, lane l stays on bank l % 32.  A tile row holds the ROW
// symbol bytes a lane decodes between two flushes.  Rows have no padding; row r
// is rotated by tile_rot(r) dwords instead, which spreads over all banks both
// the writes (all lanes write the same dword of their rows at the same time) and
// the row-wise reads of the flush.
template <int ROW>
struct alignas(256) WaveMem {
    static constexpr int row_dwords = ROW / 4;
    static_assert(row_dwords == 16 || row_dwords == 32, "the rotation below is made for these");
    uint32_t ring[kRing2Dwords * 64];
    uint32_t tile[64 * row_dwords];
    // rows of 16 dwords alternate between the two halves of the 32 banks, so pairs of rows share a rotation
    static __device__ __forceinline__ uint32_t tile_rot(uint32_t row) { return row_dwords == 16 ? row >> 1 : row; }
    // where dword j of row `row` lives
    static __device__ __forceinline__ uint32_t tile_at(uint32_t row, uint32_t j) {
        return row * row_dwords + ((j + tile_rot(row)) & (row_dwords - 1));
    }
};

// Per-wave LDS of the kernels that use the short ring: 64 bytes of stream per lane and rows of 32
// symbol bytes.  Row r is rotated by 2 * ((r >> 2) & 3) dwords, which keeps its dword pairs aligned
// and spreads rows four apart (which start on the same bank) over the banks.
struct alignas(256) WaveMem2 {
    static constexpr int row_dwords = 8;
    uint32_t ring[18 * 64];
    uint32_t tile[64 * row_dwords];
    static __device__ __forceinline__ uint32_t tile_at(uint32_t row, uint32_t j) {
        return row * row_dwords + ((j + 2u * ((row >> 2) & 3u)) & (row_dwords - 1));
    }
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef const u32x4 __attribute__((address_space(1))) *global_u4_ptr;
typedef u32x4 __attribute__((address_space(1))) *global_u4_wptr;
typedef u32x2 __attribute__((address_space(1))) *global_u2_wptr;
// LDS pointers with the address space spelled out: the accesses compile to plain
// ds_ instructions with 32-bit addresses
typedef volatile uint32_t __attribute__((address_space(3))) *lds_v32;
typedef const uint32_t __attribute__((address_space(3))) *lds_p32;

__device__ __forceinline__ uint32_t bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float dequant(uint32_t sym, int32_t z, float s) {
    return static_cast<float>(static_cast<int32_t>(sym) - z) * s;
}

__device__ __forceinline__ uint32_t pack_entry(uint32_t sym, uint32_t len) { return len | (sym << 8); }
__device__ __forceinline__ uint32_t entry_len(uint32_t e) { return e & 0x3fu; }
__device__ __forceinline__ uint32_t entry_sym(uint32_t e) { return (e >> 8) & 0xffu; }

// The eight 4-bit symbols of four pair bytes, one per byte, in order.
__device__ __forceinline__ void unpack_nibbles(uint32_t d, uint32_t &lo, uint32_t &hi) {
    const uint32_t even = d & 0x0f0f0f0fu, odd = (d >> 4) & 0x0f0f0f0fu;   // symbols 0, 2, 4, 6 and 1, 3, 5, 7
    lo = __builtin_amdgcn_perm(odd, even, 0x05010400u);
    hi = __builtin_amdgcn_perm(odd, even, 0x07030602u);
}

__device__ __forceinline__ void wave_sync_lds() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Canonical code tables and both lookup levels, built from the 256 (or 16)
// code lengths by the whole workgroup of WG >= 256 lanes (four waves hold the
// symbols).  `wcnt` is scratch of 4 * 33 words.
template <int WG, bool PAIR, class TB>
__device__ __forceinline__ void build_tables(const DevTensor &t, TB &tb, uint32_t *wcnt) {
    static_assert(WG >= 256, "one lane per symbol");
    const uint32_t tid = threadIdx.x;
    const uint32_t wave = tid >> 6;
    const uint32_t l = tid < 256 ? t.len[tid] : 0u;
    if (tid < kL2MaxPrefixes) tb.pdepth[tid] = 0;
    for (uint32_t i = tid; i < kL2Cap; i += WG) tb.lut2[i] = 0;
    // symbols of each length per wave, and every symbol's place among those of its length in its wave
    uint32_t rank = 0;
    if (tid < 256) {
        for (uint32_t b = 1; b <= ENTRO_MAX_CODE_LEN; ++b) {
            const uint64_t m = __builtin_amdgcn_ballot_w64(l == b);
            if (l == b) rank = __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(m >> 32), __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(m), 0u));
            if ((tid & 63u) == 0) wcnt[wave * (ENTRO_MAX_CODE_LEN + 1) + b] = static_cast<uint32_t>(__builtin_popcountll(m));
        }
    }
    __syncthreads();
    if (tid >= 1 && tid <= ENTRO_MAX_CODE_LEN + 1) {
        // lane b: symbols shorter than b, and the first code of length b = sum over j < b of cnt[j] * 2^(b - j)
        const uint32_t b = tid;
        uint64_t code = 0;
        uint32_t off = 0, mine = 0;
        for (uint32_t j = 1; j <= b && j <= ENTRO_MAX_CODE_LEN; ++j) {
            const uint32_t c = wcnt[j] + wcnt[(ENTRO_MAX_CODE_LEN + 1) + j] + wcnt[2 * (ENTRO_MAX_CODE_LEN + 1) + j] +
                               wcnt[3 * (ENTRO_MAX_CODE_LEN + 1) + j];
            if (j < b) {
                code += static_cast<uint64_t>(c) << (b - j);
                off += c;
            } else {
                mine = c;
            }
        }
        tb.cnt[b] = b <= ENTRO_MAX_CODE_LEN ? mine : 0u;
        tb.first[b] = static_cast<uint32_t>(code);
        tb.offs[b] = off;
    }
    if (tid == 0) { tb.cnt[0] = 0; tb.first[0] = 0; tb.offs[0] = 0; }
    __syncthreads();
    if (tid == 0) {
        // canonical codes grow with length, so the long codes own the kL1-bit prefixes from the
        // first long code's on
        uint32_t first_prefix = 1u << kL1;
        for (uint32_t b = kL1 + 1; b <= ENTRO_MAX_CODE_LEN; ++b)
            if (tb.cnt[b]) {
                first_prefix = tb.first[b] >> (b - kL1);
                break;
            }
        tb.long_start = first_prefix;
        if ((1u << kL1) - first_prefix > static_cast<uint32_t>(kL2MaxPrefixes)) first_prefix = 1u << kL1;
        tb.first_prefix = first_prefix;
    }
    __syncthreads();
    uint32_t code = 0;
    const uint32_t first_prefix = tb.first_prefix;
    const bool have_l2 = !PAIR && first_prefix < (1u << kL1);
    if (l) {
        for (uint32_t w = 0; w < wave; ++w) rank += wcnt[w * (ENTRO_MAX_CODE_LEN + 1) + l];
        code = tb.first[l] + rank;
        tb.sorted[tb.offs[l] + rank] = static_cast<uint8_t>(tid);
        if (l > kL1 && have_l2) atomicMax(&tb.pdepth[(code >> (l - kL1)) - first_prefix], l - kL1);
    }
    __syncthreads();
    if (tid == 0 && have_l2) {
        // every long prefix gets a block of 2^min(depth, cap) entries; lower the cap until all fit
        const uint32_t n_prefix = (1u << kL1) - first_prefix;
        uint32_t cap = kL2MaxBits;
        for (;;) {
            uint32_t total = 0;
            for (uint32_t q = 0; q < n_prefix; ++q) {
                const uint32_t d = tb.pdepth[q] < cap ? tb.pdepth[q] : cap;
                total += d < 4 ? 16u : 1u << d;
            }
            if (total <= static_cast<uint32_t>(kL2Cap) || cap == 0) break;
            --cap;
        }
        uint32_t base = 0;
        for (uint32_t q = 0; q < n_prefix; ++q) {
            const uint32_t d = tb.pdepth[q] < cap ? tb.pdepth[q] : cap;
            tb.pdepth[q] = d;
            tb.pbase[q] = base;
            base += d < 4 ? 16u : 1u << d;
        }
    }
    __syncthreads();
    // second level: every long symbol fills the slots of its block that start with its code
    if (l > kL1 && have_l2) {
        const uint32_t extra = l - kL1;
        const uint32_t prefix = code >> extra;
        const uint32_t depth = tb.pdepth[prefix - first_prefix];
        const uint32_t base = tb.pbase[prefix - first_prefix];
        if (extra <= depth) {
            const uint16_t e = static_cast<uint16_t>(pack_entry(tid, l));
            const uint32_t suffix = code & ((1u << extra) - 1u);
            const uint32_t rev = __brev(suffix) >> (32 - extra);
            for (uint32_t i = rev; i < (1u << depth); i += (1u << extra)) tb.lut2[base + i] = e;
        }
        // longer codes keep the zero entry: canonical search
    }
    // first level: every lane resolves its share of the index values by a canonical search whose
    // limits sit in scalar registers
    const uint32_t long_start = tb.long_start;
    uint32_t fb[kL1 + 1], cb[kL1 + 1], ob[kL1 + 1];
#pragma unroll
    for (int b = 1; b <= kL1; ++b) {
        fb[b] = __builtin_amdgcn_readfirstlane(tb.first[b]);
        cb[b] = __builtin_amdgcn_readfirstlane(tb.cnt[b]);
        ob[b] = __builtin_amdgcn_readfirstlane(tb.offs[b]);
    }
    if constexpr (PAIR) {
        // single codes of up to kSingleBits bits; zero: longer, or no code at all
        for (uint32_t i = tid; i < (1u << kSingleBits); i += WG) {
            const uint32_t v = __brev(i) >> (32 - kSingleBits);
            uint32_t len = 0, idx = 0;
#pragma unroll
            for (int b = 1; b <= kSingleBits; ++b) {
                const uint32_t d = (v >> (kSingleBits - b)) - fb[b];
                const bool hit = d < cb[b];
                len = hit ? static_cast<uint32_t>(b) : len;
                idx = hit ? ob[b] + d : idx;
            }
            tb.lut2[i] = static_cast<uint16_t>(len ? pack_entry(tb.sorted[idx], len) : 0u);
        }
    }
    for (uint32_t i = tid; i < (1u << kL1); i += WG) {
        const uint32_t v = __brev(i) >> (32 - kL1);               // the index bits in code order
        uint32_t len = 0, idx = 0;
#pragma unroll
        for (int b = 1; b <= kL1; ++b) {
            const uint32_t d = (v >> (kL1 - b)) - fb[b];
            const bool hit = d < cb[b];                           // at most one length matches
            len = hit ? static_cast<uint32_t>(b) : len;
            idx = hit ? ob[b] + d : idx;
        }
        if constexpr (PAIR) {
            // the first code as below (an index that starts no code moves one bit and gives symbol 0),
            // then the code that the remaining index bits spell, if they hold all of it
            uint32_t s0 = 0, l0 = 0;
            if (len) { s0 = tb.sorted[idx]; l0 = len; }
            else if (v < long_start) l0 = 1;
            uint32_t e = 0;
            if (l0) {
                const uint32_t v2 = (v << l0) & kL1Mask;            // zeros behind the bits that are left
                uint32_t len1 = 0, idx1 = 0;
#pragma unroll
                for (int b = 1; b <= kL1; ++b) {
                    const uint32_t d = (v2 >> (kL1 - b)) - fb[b];
                    const bool hit = d < cb[b];
                    len1 = hit ? static_cast<uint32_t>(b) : len1;
                    idx1 = hit ? ob[b] + d : idx1;
                }
                if (len1 && l0 + len1 <= static_cast<uint32_t>(kL1)) e = pack_entry(s0 | (static_cast<uint32_t>(tb.sorted[idx1]) << 4), l0 + len1);
            }
            tb.lut[i] = static_cast<std::remove_reference_t<decltype(tb.lut[0])>>(e);
            continue;
        }
        // no match: the start of a longer code (the entry says where its second-level block is),
        // or, where a lone symbol leaves half of the code space unused, of none: symbol 0, one bit
        uint32_t e = pack_entry(0, 1);
        if (v >= long_start) {
            e = 7u << 8;
            if (v >= first_prefix) e = (tb.pdepth[v - first_prefix] << 8) | ((tb.pbase[v - first_prefix] >> 4) << 11);
        }
        if (len) {
            e = pack_entry(tb.sorted[idx], len);
            if constexpr (sizeof(tb.lut[0]) == 4)       // wide entry: the centred symbol as bf16 in the high half
                e |= __float_as_uint(static_cast<float>(static_cast<int32_t>(tb.sorted[idx]) - t.zero_point)) & 0xffff0000u;
        }
        tb.lut[i] = static_cast<std::remove_reference_t<decltype(tb.lut[0])>>(e);
    }
    __syncthreads();
}

// Canonical search over the lengths from `from` on.  `window` holds the next 32
// stream bits, first bit in bit 0.
__device__ __noinline__ uint32_t decode_canonical(const TablesTail &tb, uint32_t window, uint32_t from, uint32_t max_len) {
    const uint32_t v = __brev(window);
    for (uint32_t l = from; l <= max_len; ++l) {
        const uint32_t d = (v >> (32 - l)) - tb.first[l];
        if (d < tb.cnt[l]) return pack_entry(tb.sorted[tb.offs[l] + d], l);
    }
    return pack_entry(0, 1);        // not a code (corrupt stream): keep moving
}

// The code at the start of `window`, which the first level answered with the
// miss entry `miss`: second level (needs kL1 + kL2MaxBits valid bits).  Zero if
// the code is longer still.
__device__ __forceinline__ uint32_t lookup_l2(const TablesTail &tb, uint32_t miss, uint32_t window) {
    const uint32_t depth = (miss >> 8) & 7u;
    if (depth > static_cast<uint32_t>(kL2MaxBits)) return 0;
    return tb.lut2[(((miss >> 11) << 4) + __builtin_amdgcn_ubfe(window, kL1, depth)) & (kL2Cap - 1)];
}

// The same with the canonical search behind it; `window` holds the next 32 stream bits.
__device__ __forceinline__ uint32_t decode_long(const TablesTail &tb, uint32_t miss, uint32_t window, uint32_t max_len) {
    uint32_t e = lookup_l2(tb, miss, window);
    if (__builtin_expect(e == 0, 0)) e = decode_canonical(tb, window, kL1 + 1, max_len);
    return e;
}

// Pair tables: the single code at the start of `window` (the next 32 stream bits).
__device__ __forceinline__ uint32_t single_entry(const TablesTail &tb, uint32_t window, uint32_t max_len) {
    uint32_t e = tb.lut2[window & ((1u << kSingleBits) - 1u)];
    if (__builtin_expect(e == 0, 0)) e = decode_canonical(tb, window, kSingleBits + 1, max_len);
    return e;
}

// Stream bit at which a lane's piece k starts: the segment's offset, plus the lengths of the pieces in
// front of it in the same segment where the tensor has entry points inside its segments.
__device__ __forceinline__ uint64_t seg_start(const DevTensor &t, uint32_t k) {
    const uint32_t sh = t.sub_shift;
    if (sh == 0) return t.offsets[k];
    const uint32_t c = k >> sh;
    const uint32_t before = (k - (c << sh)) << t.sub_merge;          // pieces of the segment in front of the lane's
    const uint16_t *sb = t.sub + (static_cast<uint64_t>(c) << (sh + t.sub_merge));
    uint32_t add = 0;
#pragma unroll
    for (uint32_t i = 0; i + 1 < ENTRO_MAX_SUB_PER_CHUNK; ++i)
        if (i < before) add += sb[i];
    return t.offsets[c] + add;
}

// ---------------------------------------------------------------- scalar reader
// Reads straight from global memory, one symbol per lookup; used for segments
// whose size does not fit the row path and for shorter last segments.

// 64 stream bits starting at the dword that holds absolute stream bit `pos`,
// shifted so that bit pos is bit 0: at least 33 valid bits.  The read is
// clamped to the last 8 bytes of the (padded) stream.
__device__ __forceinline__ uint64_t load_bits(const uint8_t *stream, uint64_t pos, uint32_t last_off) {
    uint32_t off = static_cast<uint32_t>(pos >> 5) << 2;
    off = off < last_off ? off : last_off;
    const uint32_t *w = reinterpret_cast<const uint32_t *>(stream + off);
    const uint64_t v = static_cast<uint64_t>(w[0]) | (static_cast<uint64_t>(w[1]) << 32);
    return v >> (static_cast<uint32_t>(pos) & 31u);
}

struct ScalarReader {
    const uint8_t *stream;
    uint32_t last_off;   // stream_bytes - 8
    uint64_t pos;        // absolute stream bit
    uint64_t buf;
};

// The next symbol's entry from the scalar reader; r.buf must hold kL1 valid bits.
// With pair tables the table of single codes answers.
template <bool PAIR, class TB>
__device__ __forceinline__ uint32_t next_entry(ScalarReader &r, const TB &tb, uint32_t max_len) {
    uint32_t e = PAIR ? tb.lut2[static_cast<uint32_t>(r.buf) & ((1u << kSingleBits) - 1u)]
                      : tb.lut[static_cast<uint32_t>(r.buf) & kL1Mask];
    if (__builtin_expect(entry_len(e) == 0, 0)) {
        const uint32_t window = static_cast<uint32_t>(load_bits(r.stream, r.pos, r.last_off));
        e = PAIR ? decode_canonical(tb, window, kSingleBits + 1, max_len) : decode_long(tb, e, window, max_len);
        r.pos += entry_len(e);
        r.buf = load_bits(r.stream, r.pos, r.last_off);
    } else {
        r.buf >>= entry_len(e);
        r.pos += entry_len(e);
    }
    return e;
}

template <int MODE> struct OutTraits;
template <> struct OutTraits<kModeU8> { static constexpr int ebits = 8; };
template <> struct OutTraits<kModeU4> { static constexpr int ebits = 4; };
template <> struct OutTraits<kModeF32> { static constexpr int ebits = 32; };
template <> struct OutTraits<kModeBF16> { static constexpr int ebits = 16; };
template <> struct OutTraits<kModeU8P> { static constexpr int ebits = 8; };
template <> struct OutTraits<kModeF32P> { static constexpr int ebits = 32; };
template <> struct OutTraits<kModeBF16P> { static constexpr int ebits = 16; };

// nsym symbols, element by element: the stream from absolute bit `pos` on holds the tensor's symbols
// first_sym, first_sym + 1, ... (first_sym is even for packed 4-bit output).
template <int MODE, class TB>
__device__ void decode_scalar_from(const DevTensor &t, const TB &tb, uint64_t pos, uint64_t first_sym, uint32_t nsym) {
    ScalarReader r;
    r.stream = t.stream;
    r.last_off = t.stream_bytes - 8u;
    r.pos = pos;
    r.buf = 0;
    const uint32_t max_len = t.max_len;
    const int32_t z = t.zero_point;
    const float s = t.scale;
    uint8_t *out8 = static_cast<uint8_t *>(t.out);
    uint32_t pending = 0;     // low nibble waiting for its partner (packed 4-bit)
    for (uint32_t i = 0; i < nsym; ++i) {
        if (i % kScalarProbes == 0) r.buf = load_bits(r.stream, r.pos, r.last_off);
        const uint32_t sym = entry_sym(next_entry<kPairMode<MODE>>(r, tb, max_len));
        const uint64_t idx = first_sym + i;
        constexpr int OUT = base_mode(MODE);
        if (OUT == kModeU8) out8[idx] = static_cast<uint8_t>(sym);
        if (OUT == kModeU4) {
            if (idx & 1) out8[idx >> 1] = static_cast<uint8_t>(pending | ((sym & 0xfu) << 4));
            else pending = sym & 0xfu;
        }
        if (OUT == kModeBF16) reinterpret_cast<uint16_t *>(t.out)[idx] = static_cast<uint16_t>(bf16_bits(dequant(sym, z, s)));
        if (OUT == kModeF32) reinterpret_cast<float *>(t.out)[idx] = dequant(sym, z, s);
    }
    if (MODE == kModeU4 && (nsym & 1)) out8[(first_sym + nsym - 1) >> 1] = static_cast<uint8_t>(pending);
}

// All nsym symbols of segment k, element by element.
template <int MODE, class TB>
__device__ void decode_scalar(const DevTensor &t, const TB &tb, uint32_t k, uint32_t nsym) {
    decode_scalar_from<MODE>(t, tb, seg_start(t, k), static_cast<uint64_t>(k) * t.chunk_symbols, nsym);
}

// ------------------------------------------------------------------ ring reader
// The long ring (gemv_direct, i.e. the GEMV of tensors that do not fit the wide tables; the
// other kernels use the short ring below).  Each lane keeps up to 128 bytes of its segment
// in a ring in LDS (eight 16-byte blocks, block j in slot j & 7) and the line that follows
// the ring's contents in registers: a lane asks memory for a whole line at a time (LB
// blocks; gemv_direct takes 64 bytes).  Dwords
// 32 and 33 of the lane's ring mirror dwords 0 and 1, so a three-dword read
// starting in the last ring dwords needs no wrap.
// Positions are bits relative to line 0, the line in which the segment starts.  The lane tracks q = p - 1, p being its position: a window read at bit
// q carries one stale low bit, which makes bits 1..14 the first-level table's
// byte offset of the code that starts at p.
// Registers move into the ring only between blocks of output (ring_topup), two
// blocks at a time, at the point where the wave's previous stores have long been
// written: a wait for the line then does not wait for stores.  A lane whose codes
// are so long that the ring runs dry in between loads its ring afresh.
// LB: blocks per line, 8 (128 bytes) or 4 (64 bytes).
template <int LB>
struct RingReader {
    static_assert(LB == 4 || LB == 8, "a line is a half or a whole 128-byte memory line");
    static constexpr uint32_t line_bytes = 16u * LB;
    const uint8_t *stream;
    lds_v32 ring;          // this lane's dword 0; dword d is ring[d * 64]
    uint32_t start64;      // byte offset of line 0 (a multiple of the line size)
    uint32_t last_blk;     // stream_bytes - 16
    uint32_t q;            // p - 1
    uint32_t end;          // the ring holds the stream up to here; a multiple of 256, at most kRingBits past p's block
    u32x4 nx[LB];          // the line at `end`; its pairs of blocks in front of `end` are in the ring already
};

__device__ __forceinline__ u32x4 load_block(const uint8_t *stream, uint32_t off, uint32_t last_blk) {
    off = off < last_blk ? off : last_blk;
    return *(global_u4_ptr)(stream + off);
}

// Line `line` into the registers; blocks past the end of the stream repeat its
// last block (nothing decodes them).
template <int LB>
__device__ __forceinline__ void load_line(RingReader<LB> &r, uint32_t line) {
    const uint32_t base = r.start64 + line * RingReader<LB>::line_bytes;
#pragma unroll
    for (int i = 0; i < LB; ++i) r.nx[i] = load_block(r.stream, base + 16u * i, r.last_blk);
}

// Block `blk` (16 bytes, counted from line 0) into its slot.
template <int LB>
__device__ __forceinline__ void ring_store(RingReader<LB> &r, uint32_t blk, const u32x4 v) {
    const uint32_t slot = blk & 7u;
    lds_v32 dst = r.ring + slot * 256u;
    dst[0] = v.x; dst[64] = v.y; dst[128] = v.z; dst[192] = v.w;
    if (slot == 0) { r.ring[32 * 64] = v.x; r.ring[33 * 64] = v.y; }
}

// Fill the ring with the 128 bytes from the 64-byte half line that holds absolute
// stream bit `pos` on, and ask for the line that holds what comes next (with
// 128-byte lines and p in the second half of line 0 that is line 1, whose first
// half is in the ring then).  RARE: the loads are a loop, to stay small where
// this is inlined into paths that hardly ever run.
template <bool RARE, int LB>
__device__ __forceinline__ void ring_fill(RingReader<LB> &r, uint64_t pos) {
    r.start64 = static_cast<uint32_t>(pos >> 3) & ~(RingReader<LB>::line_bytes - 1u);
    r.q = static_cast<uint32_t>(pos - (static_cast<uint64_t>(r.start64) << 3)) - 1u;
    const uint32_t first = ((r.q + 1u) >> 9) * 4u;                  // first block of the half line that holds p
    r.end = kRingBits + first * 128u;
    if (RARE) {
#pragma unroll 1
        for (uint32_t b = 0; b < 8; ++b) ring_store(r, first + b, load_block(r.stream, r.start64 + 16u * (first + b), r.last_blk));
    } else {
#pragma unroll
        for (uint32_t b = 0; b < 8; ++b) ring_store(r, first + b, load_block(r.stream, r.start64 + 16u * (first + b), r.last_blk));
    }
    load_line(r, r.end / (128u * LB));
}

template <int LB>
__device__ __forceinline__ void ring_load(RingReader<LB> &r, uint64_t pos) { ring_fill<false>(r, pos); }

// A ring read at q takes the dword that holds bit q and the two after it: it
// stays inside the ring's contents while q + 64 < end.
template <int LB>
__device__ __forceinline__ bool ring_short(const RingReader<LB> &r, uint32_t ahead) { return r.q + ahead + 64u >= r.end; }

// Rare: a lane whose codes are so long that the ring ran dry starts it afresh at p.
template <int LB>
__device__ __forceinline__ void ring_reload(RingReader<LB> &r) {
    ring_fill<true>(r, (static_cast<uint64_t>(r.start64) << 3) + r.q + 1u);
}

// Move what the registers hold into the blocks p has left behind, two blocks at
// a time while two slots are free; after the line's last pair, ask for the next
// line.
template <int LB>
__device__ __forceinline__ void ring_topup(RingReader<LB> &r) {
    const uint32_t pblk = ((r.q + 1u) >> 7) << 7;                    // start of the block that holds p
#pragma unroll
    for (uint32_t pair = 0; pair < LB / 2; ++pair) {
        if (((r.end >> 8) & (LB / 2 - 1u)) == pair && r.end - pblk <= kRingBits - 256u) {
            ring_store(r, r.end >> 7, r.nx[2 * pair]);
            ring_store(r, (r.end >> 7) + 1u, r.nx[2 * pair + 1]);
            r.end += 256u;
            if (pair == LB / 2 - 1) load_line(r, r.end / (128u * LB));
        }
    }
}

// The stream from bit q = p - 1 on: 63 valid bits above the stale one.
template <int LB>
__device__ __forceinline__ uint64_t ring_read(const RingReader<LB> &r) {
    // a plain (not volatile) pointer: the compiler may fetch two of the dwords with one instruction
    const lds_p32 src = (lds_p32)(r.ring + ((r.q >> 5) & 31u) * 64u);
    const uint32_t w0 = src[0], w1 = src[64], w2 = src[128];
    const uint32_t lo = __builtin_amdgcn_alignbit(w1, w0, r.q);     // uses q & 31
    const uint32_t hi = __builtin_amdgcn_alignbit(w2, w1, r.q);
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

// ------------------------------------------------------------- short ring reader
// The same reader with half the LDS, for the kernels whose wavefront count is what limits them
// (a lane's chain of dependent table lookups is bound by LDS latency, so the number of lanes a
// compute unit keeps decoding is its throughput, and LDS is what limits that number): a ring of
// four 16-byte blocks per lane (block j in slot j & 3, dwords 16 and 17 mirror dwords 0 and 1)
// and registers moving into the ring after every 32 symbols instead of 64.  The registers still
// hold a whole 128-byte line (asking memory for 64 bytes at a time reads every line twice).  Block
// i of a line goes to slot i & 3, so the moves are four statically addressed steps, each taken by
// the lanes whose next block belongs into that slot and whose slot is free.  A lane asks for its
// next line when the last block of the current one has moved; it is used from the next boundary
// on, one wait for the whole wavefront.
struct Ring2 {
    const uint8_t *stream;
    lds_v32 ring;          // this lane's dword 0; dword d is ring[d * 64]
    uint32_t start64;      // byte offset of line 0 (a multiple of 128)
    uint32_t last_blk;     // stream_bytes - 16
    uint32_t stale;        // stale low bits of a window: 1 for tables of 16-bit entries, 2 for 32-bit entries
    uint32_t q;            // p - stale, in bits from line 0
    uint32_t end;          // the ring holds the stream up to here; a multiple of 128, at most kRing2Bits past p's block
    u32x4 nx[8];           // the line that holds block end >> 7
};

template <int SLOT>
__device__ __forceinline__ void ring2_store(Ring2 &r, const u32x4 v) {
    lds_v32 dst = r.ring + SLOT * 256;
    dst[0] = v.x; dst[64] = v.y; dst[128] = v.z; dst[192] = v.w;
    if (SLOT == 0) { r.ring[16 * 64] = v.x; r.ring[17 * 64] = v.y; }
}

__device__ __forceinline__ void ring2_load_line(Ring2 &r, uint32_t line) {
    const uint32_t base = r.start64 + line * 128u;
#pragma unroll
    for (int i = 0; i < 8; ++i) r.nx[i] = load_block(r.stream, base + 16u * i, r.last_blk);
}

// Fill the ring with the four blocks from the one that holds absolute stream bit `pos` on and ask
// for the line that holds the block after them (line 0 again, if they end inside it).
template <bool RARE>
__device__ __forceinline__ void ring2_fill(Ring2 &r, uint64_t pos) {
    r.start64 = static_cast<uint32_t>(pos >> 3) & ~127u;
    r.q = static_cast<uint32_t>(pos - (static_cast<uint64_t>(r.start64) << 3)) - r.stale;
    const uint32_t first = (r.q + r.stale) >> 7;                     // 0..7
    r.end = (first + 4u) * 128u;
    if (RARE) {
#pragma unroll 1
        for (uint32_t b = first; b < first + 4u; ++b) {
            const u32x4 v = load_block(r.stream, r.start64 + 16u * b, r.last_blk);
            lds_v32 dst = r.ring + (b & 3u) * 256u;
            dst[0] = v.x; dst[64] = v.y; dst[128] = v.z; dst[192] = v.w;
            if ((b & 3u) == 0) { r.ring[16 * 64] = v.x; r.ring[17 * 64] = v.y; }
        }
    } else {
        u32x4 v[4];
#pragma unroll
        for (uint32_t b = 0; b < 4; ++b) v[b] = load_block(r.stream, r.start64 + 16u * (first + b), r.last_blk);
#pragma unroll
        for (uint32_t b = 0; b < 4; ++b) {
            lds_v32 dst = r.ring + ((first + b) & 3u) * 256u;
            dst[0] = v[b].x; dst[64] = v[b].y; dst[128] = v[b].z; dst[192] = v[b].w;
            if (((first + b) & 3u) == 0) { r.ring[16 * 64] = v[b].x; r.ring[17 * 64] = v[b].y; }
        }
    }
    ring2_load_line(r, r.end >> 10);
}

__device__ __forceinline__ bool ring_short(const Ring2 &r, uint32_t ahead) { return r.q + ahead + 64u >= r.end; }

__device__ __forceinline__ void ring_reload(Ring2 &r) {
    ring2_fill<true>(r, (static_cast<uint64_t>(r.start64) << 3) + r.q + r.stale);
}

template <int J>
__device__ __forceinline__ void ring2_step(Ring2 &r, uint32_t pblk, bool &wants_line) {
    if (((r.end >> 7) & 3u) == J && r.end - pblk <= kRing2Bits - 128u) {
        const bool upper = (r.end >> 9) & 1u;                        // the line's second half
        u32x4 v;
        v.x = upper ? r.nx[J + 4].x : r.nx[J].x;
        v.y = upper ? r.nx[J + 4].y : r.nx[J].y;
        v.z = upper ? r.nx[J + 4].z : r.nx[J].z;
        v.w = upper ? r.nx[J + 4].w : r.nx[J].w;
        ring2_store<J>(r, v);
        r.end += 128u;
        if (J == 3 && upper) wants_line = true;
    }
}

// Between two half blocks of output: registers into the slots p has left behind, then the request for the
// next line by the lanes whose registers are used up.
__device__ __forceinline__ void ring2_topup(Ring2 &r) {
    const uint32_t pblk = ((r.q + r.stale) >> 7) << 7;
    bool wants_line = false;
    ring2_step<0>(r, pblk, wants_line);
    ring2_step<1>(r, pblk, wants_line);
    ring2_step<2>(r, pblk, wants_line);
    ring2_step<3>(r, pblk, wants_line);
    if (wants_line) ring2_load_line(r, r.end >> 10);
}

__device__ __forceinline__ uint64_t ring_read(const Ring2 &r) {
    const lds_p32 src = (lds_p32)(r.ring + ((r.q >> 5) & 15u) * 64u);
    const uint32_t w0 = src[0], w1 = src[64], w2 = src[128];
    const uint32_t lo = __builtin_amdgcn_alignbit(w1, w0, r.q);
    const uint32_t hi = __builtin_amdgcn_alignbit(w2, w1, r.q);
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

// The first-level entry at this byte offset (an index shifted left by the table's number of stale bits).
template <class TB>
__device__ __forceinline__ uint32_t lut_at(const TB &tb, uint32_t byte_off) {
    typedef std::remove_const_t<std::remove_reference_t<decltype(tb.lut[0])>> E;
    return *reinterpret_cast<const E *>(reinterpret_cast<const char *>(tb.lut) + byte_off);
}

// The rest of a group for the lanes that met a code longer than kL1 bits.  e0..e3
// are the group's entries (from the long code on they all are its miss entry),
// w is the window as it stopped in front of the long code, `packed` the symbols in
// front of it (and junk behind).  The long code comes out of the second level
// with the bits still in the window (at least 63 - 3 * 14 of them; it needs 20)
// or, failing that, out of the canonical search; the symbols behind it are
// looked up one by one, each with a window of its own.
// With pair tables a miss is a pair that the index bits do not hold in full: its
// two codes, and whatever pair after it misses again, come from the table of
// single codes, every one with a window of its own.
template <bool PAIR, class Reader, class TB>
__device__ __forceinline__ uint32_t careful_group(Reader &r, const TB &tb, uint32_t max_len, uint32_t e0,
                                                  uint32_t e1, uint32_t e2, uint32_t e3, uint64_t w, uint32_t packed) {
    const uint32_t l0 = entry_len(e0), l1 = entry_len(e1), l2 = entry_len(e2);
    const uint32_t at = l0 == 0 ? 0u : l1 == 0 ? 1u : l2 == 0 ? 2u : 3u;     // place of the long code
    r.q += l0 + l1 + l2;                                                   // its entries add nothing
    if constexpr (PAIR) {
        packed = __builtin_amdgcn_ubfe(packed, 0, 8u * at);
#pragma unroll 1
        for (uint32_t i = at; i < static_cast<uint32_t>(kGroup); ++i) {
            if (ring_short(r, 0)) ring_reload(r);
            uint32_t e = lut_at(tb, static_cast<uint32_t>(ring_read(r)) & (kL1Mask << TB::stale));
            if (entry_len(e) == 0) {
                const uint32_t a = single_entry(tb, static_cast<uint32_t>(ring_read(r) >> TB::stale), max_len);
                r.q += entry_len(a);
                if (ring_short(r, 0)) ring_reload(r);
                const uint32_t b = single_entry(tb, static_cast<uint32_t>(ring_read(r) >> TB::stale), max_len);
                r.q += entry_len(b);
                e = ((entry_sym(a) & 0xfu) | ((entry_sym(b) & 0xfu) << 4)) << 8;
            } else {
                r.q += entry_len(e);
            }
            packed |= entry_sym(e) << (8u * i);
        }
        if (ring_short(r, kTripBits - 64)) ring_reload(r);
        return packed;
    }
    uint32_t e = lookup_l2(tb, e3, static_cast<uint32_t>(w >> TB::stale));
    if (__builtin_expect(e == 0, 0)) {
        if (ring_short(r, 0)) ring_reload(r);
        e = decode_canonical(tb, static_cast<uint32_t>(ring_read(r) >> TB::stale), kL1 + 1, max_len);
    }
    packed = __builtin_amdgcn_ubfe(packed, 0, 8u * at) | (entry_sym(e) << (8u * at));
    r.q += entry_len(e);
    if (at < static_cast<uint32_t>(kGroup) - 1u) {
        // the symbols behind it: one fresh window holds them all unless another long code turns up
        if (ring_short(r, 0)) ring_reload(r);
        uint64_t wi = ring_read(r);
#pragma unroll
        for (uint32_t i = 1; i < static_cast<uint32_t>(kGroup); ++i) {
            if (i > at) {
                e = lut_at(tb, static_cast<uint32_t>(wi) & (kL1Mask << TB::stale));
                if (__builtin_expect(entry_len(e) == 0, 0)) {
                    if (ring_short(r, 0)) ring_reload(r);
                    wi = ring_read(r);
                    e = decode_long(tb, e, static_cast<uint32_t>(wi >> TB::stale), max_len);
                    r.q += entry_len(e);
                    if (ring_short(r, 0)) ring_reload(r);
                    wi = ring_read(r);
                } else {
                    wi >>= entry_len(e);
                    r.q += entry_len(e);
                }
                packed |= entry_sym(e) << (8u * i);
            }
        }
    }
    // the groups that follow in this trip count on the usual margin
    if (ring_short(r, kTripBits - 64)) ring_reload(r);
    return packed;
}

// One group: a fresh window and kGroup table lookups without a branch; every
// entry is the shift amount that moves the window to the next code.  A lane that
// meets a code longer than kL1 bits stops moving (its later lookups see the same
// bits and give the same entry of length zero); if the wave has such a lane, the
// rest of its group is decoded with more care.  Returns the group's four symbols,
// first one lowest.
template <bool PAIR, class Reader, class TB>
__device__ __forceinline__ uint32_t ring_group(Reader &r, const TB &tb, uint32_t max_len) {
    uint64_t w = ring_read(r);
    const uint32_t e0 = lut_at(tb, static_cast<uint32_t>(w) & (kL1Mask << TB::stale));
    w >>= (e0 & 63u);
    const uint32_t e1 = lut_at(tb, static_cast<uint32_t>(w) & (kL1Mask << TB::stale));
    w >>= (e1 & 63u);
    const uint32_t e2 = lut_at(tb, static_cast<uint32_t>(w) & (kL1Mask << TB::stale));
    w >>= (e2 & 63u);
    const uint32_t e3 = lut_at(tb, static_cast<uint32_t>(w) & (kL1Mask << TB::stale));
    // byte 1 of each entry, in order
    uint32_t packed = __builtin_amdgcn_perm(e1, e0, 0x0c0c0501u) | __builtin_amdgcn_perm(e3, e2, 0x05010c0cu);
    uint32_t q_next = r.q + ((e0 + e1 + e2 + e3) & 0xffu);            // lengths add up in the low byte (<= 56)
    const bool miss = (e3 & 0xffu) == 0;                              // a miss entry's low byte is zero
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(miss) != 0, 0)) {
        if (miss) {
            packed = careful_group<PAIR>(r, tb, max_len, e0, e1, e2, e3, w, packed);
            q_next = r.q;
        }
    }
    r.q = q_next;
    return packed;
}

// ring_group on wide tables, for the GEMV: returns the four symbols' values (symbol - zero_point as bf16, two per
// dword, first one lowest) instead of the symbols.
template <class Reader>
__device__ __forceinline__ u32x2 ring_group_wide(Reader &r, const Tables32 &tb, uint32_t max_len, float zf) {
    constexpr uint32_t kMask = kL1Mask << Tables32::stale;
    uint64_t w = ring_read(r);
    const uint32_t e0 = lut_at(tb, static_cast<uint32_t>(w) & kMask);
    w >>= (e0 & 63u);
    const uint32_t e1 = lut_at(tb, static_cast<uint32_t>(w) & kMask);
    w >>= (e1 & 63u);
    const uint32_t e2 = lut_at(tb, static_cast<uint32_t>(w) & kMask);
    w >>= (e2 & 63u);
    const uint32_t e3 = lut_at(tb, static_cast<uint32_t>(w) & kMask);
    // the high halves of the entries, in order
    u32x2 vals = {__builtin_amdgcn_perm(e1, e0, 0x07060302u), __builtin_amdgcn_perm(e3, e2, 0x07060302u)};
    uint32_t q_next = r.q + ((e0 + e1 + e2 + e3) & 0xffu);
    const bool miss = (e3 & 0xffu) == 0;
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(miss) != 0, 0)) {
        if (miss) {
            const uint32_t packed = careful_group<false>(r, tb, max_len, e0, e1, e2, e3, w,
                                                         __builtin_amdgcn_perm(e1, e0, 0x0c0c0501u) | __builtin_amdgcn_perm(e3, e2, 0x05010c0cu));
            // the same values by arithmetic: an integer of at most 256 in magnitude is a bf16 as it stands
            const uint32_t v0 = __float_as_uint(static_cast<float>(packed & 0xffu) - zf) >> 16;
            const uint32_t v1 = __float_as_uint(static_cast<float>((packed >> 8) & 0xffu) - zf) & 0xffff0000u;
            const uint32_t v2 = __float_as_uint(static_cast<float>((packed >> 16) & 0xffu) - zf) >> 16;
            const uint32_t v3 = __float_as_uint(static_cast<float>(packed >> 24) - zf) & 0xffff0000u;
            vals = u32x2{v0 | v1, v2 | v3};
            q_next = r.q;
        }
    }
    r.q = q_next;
    return vals;
}

template <int MODE, class TB>
__device__ __forceinline__ void gemv_segment(const DevTensor &t, const TB &tb, uint32_t k);

// Decode the kUnit segments from wave_first on, one per lane of this wavefront,
// SPB symbols per lane at a time into the wave's
// LDS tile (one row of symbol bytes per lane; all lanes move in step, four
// symbols per group), then consume the tile row-wise: write it out in the output
// type, so that every store instruction covers whole rows.
template <int MODE>
__device__ __forceinline__ void decode_rows(const DevTensor &t, const Tables &tb, WaveMem<Cfg<MODE>::row> *wms,
                                            uint32_t wave_first) {
    static_assert(!is_gemv(MODE), "the GEMV has a kernel of its own");
    constexpr bool PAIR = kPairMode<MODE>;
    constexpr int SPB = Cfg<MODE>::spb;                   // symbols of a lane per block
    constexpr int ROW = Cfg<MODE>::row;                   // bytes they make in the tile
    constexpr int OUT_ROW = Cfg<MODE>::out_row;
    constexpr uint32_t PIECE = Cfg<MODE>::piece;          // tile bytes one lane consumes per pass
    constexpr uint32_t LPR = ROW / PIECE;                 // lanes that consume one row
    constexpr uint32_t RPI = 64 / LPR;                    // rows per pass
    constexpr uint32_t EBITS = OutTraits<MODE>::ebits;
    constexpr int TRIPS = ROW / (kGroup * kTripGroups);
    static_assert(ROW % (kGroup * kTripGroups) == 0, "a row is a whole number of trips");
    static_assert(SPB == (PAIR ? 2 : 1) * ROW, "one tile byte per lookup");
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = threadIdx.x >> 6;
    WaveMem<ROW> &wm = wms[wave];
    if (wave_first >= t.n_chunks) return;
    const uint32_t C = t.chunk_symbols;
    const uint32_t blocks_total = C / SPB;
    const uint32_t k = wave_first + lane;
    uint32_t nsym = 0;
    if (k < t.n_chunks) {
        const uint64_t left = t.n - static_cast<uint64_t>(k) * C;
        nsym = left < C ? static_cast<uint32_t>(left) : C;
    }
    // A shorter last segment takes the row path for its whole blocks and the scalar path for the
    // rest.  The lane moves on with the others past its own end; what it decodes there is not stored.
    const bool fast = nsym != 0;
    const uint32_t my_blocks = nsym / SPB;
    uint64_t tail_pos = fast ? seg_start(t, k) : 0;       // where the symbols behind the lane's last whole block start
    Ring2 r;
    r.stale = Tables::stale;
    r.stream = t.stream;
    r.last_blk = t.stream_bytes - 16u;
    r.ring = (lds_v32)(wm.ring + lane);
    // a lane without a full segment decodes the start of the stream along with the others; nothing of it is stored
    ring2_fill<false>(r, tail_pos);
    const uint64_t bytes_per_chunk = (static_cast<uint64_t>(C) * EBITS) >> 3;
    const uint32_t n_full = static_cast<uint32_t>(t.n / C);          // segments of full length
    // whole blocks of the shorter last segment, if there is one
    const uint32_t tail_blocks = static_cast<uint32_t>((t.n - static_cast<uint64_t>(n_full) * C) / SPB);
    // a wave that holds only the shorter last segment stops after its blocks
    const uint32_t wave_blocks = wave_first < n_full ? blocks_total : tail_blocks;
    // where the first row this lane serves in a flush pass begins; the passes are RPI rows apart
    uint8_t *const row0 = static_cast<uint8_t *>(t.out) + (wave_first + lane / LPR) * bytes_per_chunk;
    const uint32_t max_len = t.max_len;
    const float zf = static_cast<float>(t.zero_point);    // exact: the host rejects |z| > 2^24
    const float scale = t.scale;
    lds_v32 tile = (lds_v32)wm.tile;

    // integer outputs whose blocks make 64 bytes per row: the even block's pieces, kept for the odd block's flush
    constexpr bool HOLD = OUT_ROW == 64;
    u32x4 held[HOLD ? 64 / RPI : 1];
    bool held_full[HOLD ? 64 / RPI : 1];
    for (uint32_t bs = 0; bs < wave_blocks; ++bs) {
#pragma unroll 1
        for (int trip = 0; trip < TRIPS; ++trip) {
            if (__builtin_expect(ring_short(r, kTripBits - 64), 0)) ring_reload(r);
#pragma unroll
            for (int g = 0; g < kTripGroups; ++g)
                tile[WaveMem<ROW>::tile_at(lane, trip * kTripGroups + g)] = ring_group<PAIR>(r, tb, max_len);
            // the short ring is topped up after every eight groups
            if (trip & 1) ring2_topup(r);
        }
        if (bs + 1 == my_blocks) tail_pos = (static_cast<uint64_t>(r.start64) << 3) + r.q + r.stale;
        wave_sync_lds();
#pragma unroll
        for (uint32_t it = 0; it < 64 / RPI; ++it) {
            const uint32_t rr = it * RPI + lane / LPR;
            const uint32_t piece = lane % LPR;
            const uint32_t kk = wave_first + rr;
            // the row has this block: always in a full segment, up to tail_blocks in the shorter last one
            const bool full = kk < n_full || (kk == n_full && bs < tail_blocks);
            uint8_t *dst = row0 + static_cast<uint64_t>(it) * (RPI * bytes_per_chunk) + static_cast<uint64_t>(bs) * OUT_ROW;
            // Store k of the pass writes the bytes [k * LPR * 16, (k + 1) * LPR * 16) of the row's
            // piece of this block, 16 per lane, so that every store instruction covers whole
            // stretches of memory; the lane fetches the tile bytes that become its 16 bytes.
            constexpr int OUT = base_mode(MODE);
            constexpr uint32_t SYMS = OUT == kModeF32 ? 4u : OUT == kModeBF16 ? 8u : OUT == kModeU8 ? 16u : 32u;   // per 16 bytes
            constexpr uint32_t TB = PAIR && OUT != kModeU4 ? SYMS / 2u : OUT == kModeU4 ? 16u : SYMS;   // tile bytes for them
            constexpr uint32_t NST = ROW / (LPR * TB);
            static_assert(NST * LPR * TB == ROW && NST * LPR * 16u == static_cast<uint32_t>(OUT_ROW), "the stores tile the row");
#pragma unroll
            for (uint32_t k = 0; k < NST; ++k) {
                const uint32_t tb0 = (k * LPR + piece) * TB;        // first tile byte of this lane's share
                uint32_t raw[TB >= 4 ? TB / 4 : 1];
#pragma unroll
                for (uint32_t j = 0; j < (TB >= 4 ? TB / 4 : 1); ++j) raw[j] = tile[WaveMem<ROW>::tile_at(rr, tb0 / 4 + j)];
                if (TB < 4) raw[0] = (raw[0] >> (8u * (tb0 & 3u))) & 0xffffu;    // two pair bytes out of a dword
                uint8_t *const at = dst + k * (LPR * 16u) + piece * 16u;
                if constexpr (OUT == kModeU8 || OUT == kModeU4) {
                    u32x4 v;
                    if constexpr (PAIR && OUT == kModeU8) {
                        // 8 pair bytes -> 16 symbol bytes
                        uint32_t u[4];
                        unpack_nibbles(raw[0], u[0], u[1]);
                        unpack_nibbles(raw[1], u[2], u[3]);
                        v = u32x4{u[0], u[1], u[2], u[3]};
                    } else {
                        // the tile bytes are the output bytes (4-bit pairs come packed out of the table)
                        v = u32x4{raw[0], raw[1], raw[2], raw[3]};
                    }
                    if constexpr (HOLD) {
                        // a block makes only 64 bytes per row: the even block's piece waits for the odd
                        // block's, and the two go out in neighbouring store instructions, which the L2
                        // merges into whole 128-byte lines (64 bytes at a time reach memory at 2.8 TB/s,
                        // the merged lines at 4.8)
                        if ((bs & 1u) == 0 && bs + 1 < wave_blocks) {
                            held[it] = v;
                            held_full[it] = full;
                        } else {
                            if ((bs & 1u) && held_full[it]) *(global_u4_wptr)(at - OUT_ROW) = held[it];
                            if (full) *(global_u4_wptr)at = v;
                        }
                    } else {
                        if (full) *(global_u4_wptr)at = v;
                    }
                } else {
                    // w = (q - z) * s: exact difference, one fp32 multiply
                    uint32_t sym4[SYMS / 4];                         // one symbol per byte
                    if constexpr (PAIR) {
                        if constexpr (SYMS == 8) {
                            unpack_nibbles(raw[0], sym4[0], sym4[1]);
                        } else {
                            uint32_t unused;
                            unpack_nibbles(raw[0], sym4[0], unused);
                        }
                    } else {
#pragma unroll
                        for (uint32_t j = 0; j < SYMS / 4; ++j) sym4[j] = raw[j];
                    }
                    float f[SYMS];
#pragma unroll
                    for (uint32_t j = 0; j < SYMS; ++j)
                        f[j] = (static_cast<float>((sym4[j / 4] >> (8 * (j % 4))) & 0xffu) - zf) * scale;
                    u32x4 v;
                    if constexpr (OUT == kModeF32) {
                        v = u32x4{__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3])};
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const f32x2 pr = {f[2 * j], f[2 * j + 1]};
                            const bf16x2 b = __builtin_convertvector(pr, bf16x2);   // round to nearest even
                            v[j] = __builtin_bit_cast(uint32_t, b);
                        }
                    }
                    if (full) {
                        if constexpr (OUT == kModeF32) *(global_u4_wptr)at = v;
                        else __builtin_nontemporal_store(v, (global_u4_wptr)at);
                    }
                }
            }
        }
        wave_sync_lds();
    }
    const uint32_t rest = nsym - my_blocks * SPB;
    if (rest) decode_scalar_from<MODE>(t, tb, tail_pos, static_cast<uint64_t>(k) * C + my_blocks * SPB, rest);
}

// decode_rows for the fp32 and bf16 outputs with a tile of half a block: sixteen wavefronts per
// workgroup instead of fourteen.  A block of 64 symbols per lane is decoded and flushed in two halves of 32.  A
// half makes 128 bytes of fp32 per row, which go out as they are; of bf16 it makes 64, so the first
// half's symbols wait in registers (in the lanes that will convert them) and the second half's flush
// writes whole 128-byte rows.
// ALLFULL: the unit's 64 segments all have full length (decided per wavefront): no store needs a
// condition, no lane a tail.
template <int MODE, bool ALLFULL>
__device__ __forceinline__ void decode_rows2_impl(const DevTensor &t, const Tables &tb, WaveMem2 &wm, uint32_t wave_first) {
    static_assert(MODE == kModeF32 || MODE == kModeBF16, "single codes, two or four bytes per symbol");
    constexpr int SPB = Cfg<MODE>::spb;                   // 64
    constexpr uint32_t EBITS = OutTraits<MODE>::ebits;
    constexpr int HALF_GROUPS = 8;                        // groups of four symbols per half block
    static_assert(SPB == 64 && HALF_GROUPS * kGroup * 2 == SPB && HALF_GROUPS % kTripGroups == 0, "two halves of two trips");
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t C = t.chunk_symbols;
    const uint32_t blocks_total = C / SPB;
    const uint32_t k = wave_first + lane;
    uint32_t nsym = C;
    if (!ALLFULL) {
        nsym = 0;
        if (k < t.n_chunks) {
            const uint64_t left = t.n - static_cast<uint64_t>(k) * C;
            nsym = left < C ? static_cast<uint32_t>(left) : C;
        }
    }
    const bool fast = nsym != 0;
    const uint32_t my_blocks = nsym / SPB;
    uint64_t tail_pos = fast ? seg_start(t, k) : 0;
    Ring2 r;
    r.stale = Tables::stale;
    r.stream = t.stream;
    r.last_blk = t.stream_bytes - 16u;
    r.ring = (lds_v32)(wm.ring + lane);
    ring2_fill<false>(r, tail_pos);
    const uint64_t bytes_per_chunk = (static_cast<uint64_t>(C) * EBITS) >> 3;
    const uint32_t n_full = static_cast<uint32_t>(t.n / C);
    const uint32_t tail_blocks = static_cast<uint32_t>((t.n - static_cast<uint64_t>(n_full) * C) / SPB);
    const uint32_t wave_blocks = ALLFULL || wave_first < n_full ? blocks_total : tail_blocks;
    // a flush pass serves eight rows, eight lanes each; the passes are eight rows apart
    const uint32_t piece = lane & 7u;
    uint8_t *const row0 = static_cast<uint8_t *>(t.out) + (wave_first + (lane >> 3)) * bytes_per_chunk + piece * 16u;
    const uint32_t max_len = t.max_len;
    const float zf = static_cast<float>(t.zero_point);    // exact: the host rejects |z| > 2^24
    const float scale = t.scale;
    lds_v32 tile = (lds_v32)wm.tile;
    typedef const u32x2 __attribute__((address_space(3))) *lds_p64;
    u32x2 held[8];                                        // bf16: the first half's eight symbols of each pass
    for (uint32_t bs = 0; bs < wave_blocks; ++bs) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll 1
            for (int trip = 0; trip < HALF_GROUPS / kTripGroups; ++trip) {
                if (__builtin_expect(ring_short(r, kTripBits - 64), 0)) ring_reload(r);
#pragma unroll
                for (int g = 0; g < kTripGroups; ++g)
                    tile[WaveMem2::tile_at(lane, trip * kTripGroups + g)] = ring_group<false>(r, tb, max_len);
            }
            if (!ALLFULL && half == 1 && bs + 1 == my_blocks) tail_pos = (static_cast<uint64_t>(r.start64) << 3) + r.q + r.stale;
            ring2_topup(r);
            wave_sync_lds();
#pragma unroll
            for (uint32_t it = 0; it < 8; ++it) {
                const uint32_t rr = it * 8u + (lane >> 3);
                const uint32_t kk = wave_first + rr;
                const bool full = ALLFULL || kk < n_full || (kk == n_full && bs < tail_blocks);
                uint8_t *const dst = row0 + static_cast<uint64_t>(it) * (8u * bytes_per_chunk);
                if constexpr (MODE == kModeF32) {
                    const uint32_t raw = tile[WaveMem2::tile_at(rr, piece)];
                    u32x4 v;
#pragma unroll
                    for (uint32_t j = 0; j < 4; ++j)
                        v[j] = __float_as_uint((static_cast<float>((raw >> (8 * j)) & 0xffu) - zf) * scale);
                    if (full) *(global_u4_wptr)(dst + (static_cast<uint64_t>(bs) * 2u + half) * 128u) = v;
                } else {
                    // lanes 0..3 of a row convert the first half's symbols, lanes 4..7 the second half's
                    const u32x2 raw = *(lds_p64)(wm.tile + WaveMem2::tile_at(rr, 2u * (piece & 3u)));
                    if (half == 0) {
                        held[it] = raw;
                    } else {
                        const u32x2 sym8 = piece < 4u ? held[it] : raw;
                        u32x4 v;
#pragma unroll
                        for (uint32_t j = 0; j < 4; ++j) {
                            const uint32_t d = sym8[j / 2];
                            const f32x2 pr = {(static_cast<float>((d >> (16 * (j & 1))) & 0xffu) - zf) * scale,
                                              (static_cast<float>((d >> (16 * (j & 1) + 8)) & 0xffu) - zf) * scale};
                            v[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));   // round to nearest even
                        }
                        if (full) __builtin_nontemporal_store(v, (global_u4_wptr)(dst + static_cast<uint64_t>(bs) * 128u));
                    }
                }
            }
            wave_sync_lds();
        }
    }
    if (!ALLFULL) {
        const uint32_t rest = nsym - my_blocks * SPB;
        if (rest) decode_scalar_from<MODE>(t, tb, tail_pos, static_cast<uint64_t>(k) * C + my_blocks * SPB, rest);
    }
}

template <int MODE>
__device__ __forceinline__ void decode_rows2(const DevTensor &t, const Tables &tb, WaveMem2 *wms, uint32_t wave_first) {
    if (wave_first >= t.n_chunks) return;
    WaveMem2 &wm = wms[threadIdx.x >> 6];
    const uint32_t n_full = static_cast<uint32_t>(t.n / t.chunk_symbols);
    if (wave_first + kUnit <= n_full) decode_rows2_impl<MODE, true>(t, tb, wm, wave_first);
    else decode_rows2_impl<MODE, false>(t, tb, wm, wave_first);
}

// Decode one segment straight into dot products with x.  A segment covers one
// or more row fragments; complete rows are stored, a leading / trailing
// incomplete fragment goes to the segment's head / tail partial.
template <int MODE, class TB>
__device__ __forceinline__ void gemv_segment(const DevTensor &t, const TB &tb, uint32_t k) {
    const uint32_t C = t.chunk_symbols;
    const uint64_t first_sym = static_cast<uint64_t>(k) * C;
    const uint64_t left = t.n - first_sym;
    const uint32_t nsym = left < C ? static_cast<uint32_t>(left) : C;
    ScalarReader r;
    r.stream = t.stream;
    r.last_off = t.stream_bytes - 8u;
    r.pos = seg_start(t, k);
    r.buf = 0;
    const uint32_t max_len = t.max_len;
    const int32_t z = t.zero_point;
    const uint32_t cols = t.cols;

    uint32_t row = static_cast<uint32_t>(first_sym / cols);
    uint32_t col = static_cast<uint32_t>(first_sym - static_cast<uint64_t>(row) * cols);
    const uint32_t start_col = col;
    bool first_fragment = true;
    float acc = 0.0f;
    float head = 0.0f, tail = 0.0f;
    for (uint32_t i = 0; i < nsym; ++i) {
        if (i % kScalarProbes == 0) r.buf = load_bits(r.stream, r.pos, r.last_off);
        const uint32_t sym = entry_sym(next_entry<kPairMode<MODE>>(r, tb, max_len));
        const float xv = __uint_as_float(static_cast<uint32_t>(t.x[col]) << 16);
        acc = fmaf(static_cast<float>(static_cast<int32_t>(sym) - z), xv, acc);
        if (++col == cols) {
            if (first_fragment && start_col != 0) {
                head = acc;                              // row began in an earlier segment
            } else {
                const float y = acc * t.scale;
                if (gemv_f32(MODE)) reinterpret_cast<float *>(t.out)[row] = y;
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

// Lanes that take pieces of a row, t.row_lanes (a power of two, 2..64) side by side in one wavefront: every
// lane's piece lies inside one row and `mine` is its sum; the row's lanes add theirs up in a fixed tree and
// the first of them stores the row.  Neither partial sums in memory nor a second kernel are needed then.
template <int MODE>
__device__ __forceinline__ void wave_row_sums(const DevTensor &t, uint32_t k, bool full, float mine) {
    const uint32_t rl = t.row_lanes;
    float v = full ? mine : 0.0f;                          // (lanes behind the tensor's end)
#pragma unroll
    for (uint32_t m = 1; m < 64u; m <<= 1)
        if (m < rl) v += __shfl_xor(v, static_cast<int>(m), 64);
    if (full && (k & (rl - 1u)) == 0) {
        const float y = v * t.scale;
        const uint32_t row = k / rl;
        if (gemv_f32(MODE)) reinterpret_cast<float *>(t.out)[row] = y;
        else reinterpret_cast<uint16_t *>(t.out)[row] = static_cast<uint16_t>(bf16_bits(y));
    }
}

// GEMV: the lane that decodes a segment also multiplies it into x, a group of symbols at a time as
// they come out of the table; there is no tile and no flush, which leaves LDS for 14 wavefronts.
// All lanes are at the same place of their segments, so where segments and rows coincide the lanes
// of a wave ask for the same piece of x (one request); elsewhere they ask for a handful of
// different ones.  The 64 activations of a half block are requested one half block ahead, before
// the stream lines that ring_topup asks for: loads return in order, and a wait for x must not
// become a wait for the stream.
// A segment may begin and end anywhere in a row and hold any number of row ends (cols >= 64, so a
// half block holds at most one): the sum up to the first row end is the head fragment (or a whole
// row, if the segment starts one), every further row end completes a whole row, which the lane
// stores itself, and what is left at the end is the tail fragment; the fragments go to the
// segment's two partial sums, which the second stage adds up per row.
template <int MODE>
__device__ __forceinline__ void gemv_direct(const DevTensor &t, const Tables &tb, uint32_t *ring_mem, uint32_t wave_first) {
    constexpr bool PAIR = kPairMode<MODE>;                 // two 4-bit symbols per table lookup
    constexpr int SPG = PAIR ? 8 : 4;                      // symbols per group
    constexpr int GPH = 64 / SPG;                          // groups per half block of 64 symbols
    const uint32_t lane = threadIdx.x & 63u;
    if (wave_first >= t.n_chunks) return;
    const uint32_t C = t.chunk_symbols;
    const uint32_t k = wave_first + lane;
    uint32_t nsym = 0;
    if (k < t.n_chunks) {
        const uint64_t left = t.n - static_cast<uint64_t>(k) * C;
        nsym = left < C ? static_cast<uint32_t>(left) : C;
    }
    const bool fast = nsym == C;                           // a shorter last segment takes the element-by-element path
    RingReader<4> r;
    r.stream = t.stream;
    r.last_blk = t.stream_bytes - 16u;
    r.ring = (lds_v32)(ring_mem + lane);
    // a lane without a full segment decodes the start of the stream along with the others; nothing of it is stored
    ring_load(r, fast ? seg_start(t, k) : 0);
    const uint32_t cols = t.cols;
    const uint16_t *xvec = t.x;
    const uint32_t max_len = t.max_len;
    const float zf = static_cast<float>(t.zero_point);    // exact: the host rejects |z| > 2^24
    const float scale = t.scale;
    const uint64_t flat0 = static_cast<uint64_t>(k) * C;
    uint32_t col = fast ? static_cast<uint32_t>(flat0 % cols) : 0u;    // column of the half block's first symbol
    uint32_t row = fast ? static_cast<uint32_t>(flat0 / cols) : 0u;    // the row the lane is in
    const bool starts_row = col == 0;
    float acc = 0.0f, first = 0.0f, end_sum = 0.0f;
    bool crossed = false;                                  // a row end has been passed
    bool ended = false;                                    // a row ended in this half block: end_sum holds its sum
    // eight activations per piece; a piece never straddles a row end (cols % 8 == 0, segments start at multiples of 64)
    u32x4 xb[8];
    auto ask_x = [&](uint32_t c0) {
#pragma unroll
        for (uint32_t p = 0; p < 8; ++p) {
            uint32_t c = c0 + 8u * p;
            c -= c >= cols ? cols : 0u;
            xb[p] = *(global_u4_ptr)(xvec + c);
        }
    };
    auto mul4 = [&](uint32_t s4, uint32_t xa, uint32_t xc) {
        acc = fmaf(static_cast<float>(s4 & 0xffu) - zf, __uint_as_float(xa << 16), acc);
        acc = fmaf(static_cast<float>((s4 >> 8) & 0xffu) - zf, __uint_as_float(xa & 0xffff0000u), acc);
        acc = fmaf(static_cast<float>((s4 >> 16) & 0xffu) - zf, __uint_as_float(xc << 16), acc);
        acc = fmaf(static_cast<float>(s4 >> 24) - zf, __uint_as_float(xc & 0xffff0000u), acc);
    };
    ask_x(col);
    const uint32_t halves = C / 64u;
    for (uint32_t h = 0; h < halves; ++h) {
#pragma unroll
        for (int g = 0; g < GPH; ++g) {
            if (g % kTripGroups == 0)
                if (__builtin_expect(ring_short(r, kTripBits - 64), 0)) ring_reload(r);
            const uint32_t s4 = ring_group<PAIR>(r, tb, max_len);
            if constexpr (PAIR) {
                uint32_t lo, hi;
                unpack_nibbles(s4, lo, hi);
                mul4(lo, xb[g].x, xb[g].y);
                mul4(hi, xb[g].z, xb[g].w);
            } else {
                const u32x4 xv = xb[g / 2];
                mul4(s4, (g & 1) ? xv.z : xv.x, (g & 1) ? xv.w : xv.y);
            }
            if (PAIR || (g & 1)) {
                // a row ends behind this piece (at most once per half block: cols >= 64): its sum is set
                // aside without a branch, so that the groups of the half block stay one stretch of code
                const uint32_t piece = PAIR ? g : g / 2;
                const bool row_end = col + 8u * piece + 8u == cols;
                end_sum = row_end ? acc : end_sum;
                acc = row_end ? 0.0f : acc;
                ended |= row_end;
            }
        }
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(ended) != 0, 0)) {
            if (ended) {
                if (!crossed && !starts_row) {
                    first = end_sum;                       // the head fragment
                } else if (fast) {                         // a whole row
                    const float y = end_sum * scale;
                    if (gemv_f32(MODE)) reinterpret_cast<float *>(t.out)[row] = y;
                    else reinterpret_cast<uint16_t *>(t.out)[row] = static_cast<uint16_t>(bf16_bits(y));
                }
                crossed = true;
                row += 1u;
                ended = false;
            }
        }
        col += 64u;
        col -= col >= cols ? cols : 0u;
        if (h + 1 < halves) ask_x(col);
        if (!PAIR || (h & 1u)) ring_topup(r);              // once per block of 16 groups
    }
    if (t.row_lanes) {
        wave_row_sums<MODE>(t, k, fast, crossed ? first : acc);
    } else if (fast) {
        if (!crossed) {
            t.partials[2 * static_cast<uint64_t>(k)] = acc;              // the segment lies inside one row
        } else {
            if (!starts_row) t.partials[2 * static_cast<uint64_t>(k)] = first;
            if (col != 0) t.partials[2 * static_cast<uint64_t>(k) + 1] = acc;   // the segment ends inside a row
        }
    } else if (nsym) {
        gemv_segment<MODE>(t, tb, k);
    }
}

// gemv_direct on wide tables and the short ring (8-bit symbols whose zero-point lies in [-1, 256], so that
// symbol - zero_point is a bf16 as it stands): the table entry carries that value, two v_perm gather a group's
// four values into two bf16 pairs and two v_dot2c_f32_bf16 multiply them into x; no conversion and no
// subtraction per symbol.  The 64 KB table and a ring of 64 bytes per lane leave LDS for sixteen wavefronts.
// The ring is topped up after every eight groups.  Row ends, fragments and the request for x one half block
// ahead are gemv_direct's; lanes that cut a row into a power of two of pieces add the row up themselves
// (wave_row_sums) instead of writing partial sums.
template <int MODE>
__device__ __forceinline__ void gemv_direct2(const DevTensor &t, const Tables32 &tb, uint32_t *ring_mem, uint32_t wave_first) {
    constexpr int GPH = 16;                                // groups of four symbols per half block of 64 symbols
    const uint32_t lane = threadIdx.x & 63u;
    if (wave_first >= t.n_chunks) return;
    const uint32_t C = t.chunk_symbols;
    const uint32_t k = wave_first + lane;
    uint32_t nsym = 0;
    if (k < t.n_chunks) {
        const uint64_t left = t.n - static_cast<uint64_t>(k) * C;
        nsym = left < C ? static_cast<uint32_t>(left) : C;
    }
    const bool fast = nsym == C;                           // a shorter last segment takes the element-by-element path
    Ring2 r;
    r.stale = Tables32::stale;
    r.stream = t.stream;
    r.last_blk = t.stream_bytes - 16u;
    r.ring = (lds_v32)(ring_mem + lane);
    // a lane without a full segment decodes the start of the stream along with the others; nothing of it is stored
    ring2_fill<false>(r, fast ? seg_start(t, k) : 0);
    const uint32_t cols = t.cols;
    const uint16_t *xvec = t.x;
    const uint32_t max_len = t.max_len;
    const float zf = static_cast<float>(t.zero_point);    // exact: the host rejects |z| > 2^24
    const float scale = t.scale;
    const uint64_t flat0 = static_cast<uint64_t>(k) * C;
    uint32_t col = fast ? static_cast<uint32_t>(flat0 % cols) : 0u;    // column of the half block's first symbol
    uint32_t row = fast ? static_cast<uint32_t>(flat0 / cols) : 0u;    // the row the lane is in
    const bool starts_row = col == 0;
    float acc = 0.0f, first = 0.0f, end_sum = 0.0f;
    bool crossed = false;                                  // a row end has been passed
    bool ended = false;                                    // a row ended in this half block: end_sum holds its sum
    // eight activations per piece; a piece never straddles a row end (cols % 8 == 0, segments start at multiples of 64)
    u32x4 xb[8];
    auto ask_x = [&](uint32_t c0) {
#pragma unroll
        for (uint32_t p = 0; p < 8; ++p) {
            uint32_t c = c0 + 8u * p;
            c -= c >= cols ? cols : 0u;
            xb[p] = *(global_u4_ptr)(xvec + c);
        }
    };
    // two products per instruction: the table entries hold symbol - zero_point as bf16, x is bf16 as it stands
    // (the halves of v go through scalars: a bit cast applied to a vector's element reads element 0 whichever is named)
    auto mul4 = [&](u32x2 v, uint32_t xa, uint32_t xc) {
        const uint32_t lo = v.x, hi = v.y;
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, lo), __builtin_bit_cast(bf16x2, xa), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, hi), __builtin_bit_cast(bf16x2, xc), acc, false);
    };
    ask_x(col);
    const uint32_t halves = C / 64u;
    // eight groups as one stretch of straight-line code; PART says which eight of the half block's sixteen
    auto eight = [&](auto part_tag) __attribute__((always_inline)) {
        constexpr int PART = decltype(part_tag)::value;
#pragma unroll
        for (int gg = 0; gg < GPH / 2; ++gg) {
            const int g = PART * (GPH / 2) + gg;
            if (g % kTripGroups == 0)
                if (__builtin_expect(ring_short(r, kTripBits - 64), 0)) ring_reload(r);
            const u32x2 v4 = ring_group_wide(r, tb, max_len, zf);
            const u32x4 xv = xb[g / 2];
            mul4(v4, (g & 1) ? xv.z : xv.x, (g & 1) ? xv.w : xv.y);
            if (g & 1) {
                // a row ends behind this piece (at most once per half block: cols >= 64): its sum is set
                // aside without a branch, so that the groups stay one stretch of code
                const uint32_t piece = g / 2;
                const bool row_end = col + 8u * piece + 8u == cols;
                end_sum = row_end ? acc : end_sum;
                acc = row_end ? 0.0f : acc;
                ended |= row_end;
            }
        }
    };
    for (uint32_t h = 0; h < halves; ++h) {
        eight(std::integral_constant<int, 0>{});
        ring2_topup(r);                                    // the short ring is topped up after every eight groups
        eight(std::integral_constant<int, 1>{});
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(ended) != 0, 0)) {
            if (ended) {
                if (!crossed && !starts_row) {
                    first = end_sum;                       // the head fragment
                } else if (fast) {                         // a whole row
                    const float y = end_sum * scale;
                    if (gemv_f32(MODE)) reinterpret_cast<float *>(t.out)[row] = y;
                    else reinterpret_cast<uint16_t *>(t.out)[row] = static_cast<uint16_t>(bf16_bits(y));
                }
                crossed = true;
                row += 1u;
                ended = false;
            }
        }
        col += 64u;
        col -= col >= cols ? cols : 0u;
        if (h + 1 < halves) ask_x(col);
        ring2_topup(r);
    }
    if (t.row_lanes) {
        wave_row_sums<MODE>(t, k, fast, crossed ? first : acc);
    } else if (fast) {
        if (!crossed) {
            t.partials[2 * static_cast<uint64_t>(k)] = acc;              // the segment lies inside one row
        } else {
            if (!starts_row) t.partials[2 * static_cast<uint64_t>(k)] = first;
            if (col != 0) t.partials[2 * static_cast<uint64_t>(k) + 1] = acc;   // the segment ends inside a row
        }
    } else if (nsym) {
        gemv_segment<MODE>(t, tb, k);
    }
}

// The GEMV kernels need the tables and the scratch table only.
struct alignas(256) RingMem { uint32_t ring[kRingDwords * 64]; };
// which modes decode on the short ring (decode_rows2)
constexpr bool short_ring(int mode) { return mode == kModeF32 || mode == kModeBF16; }
struct alignas(256) Ring2Mem { uint32_t ring[kRing2Dwords * 64]; };
template <int MODE, bool GEMV = is_gemv(MODE), bool SHORT = short_ring(MODE), bool WIDE = wide_gemv(MODE)>
struct SmemFor { Tables tb; WaveMem<Cfg<MODE>::row> wm[Cfg<MODE>::waves]; };
template <int MODE> struct SmemFor<MODE, true, false, false> { Tables tb; RingMem wm[Cfg<MODE>::waves]; };
template <int MODE> struct SmemFor<MODE, true, false, true> { Tables32 tb; Ring2Mem wm[Cfg<MODE>::waves]; };
template <int MODE> struct SmemFor<MODE, false, true, false> { Tables tb; WaveMem2 wm[Cfg<MODE>::waves]; };

// Does the tensor go through decode_rows?  Segments must tile into blocks; for the
// GEMV, pieces of eight must not straddle a matrix row and a segment must touch at
// most two rows.
template <int MODE>
__device__ __forceinline__ bool rows_fit(const DevTensor &t) {
    if (t.chunk_symbols % Cfg<MODE>::spb != 0) return false;
    if constexpr (is_gemv(MODE)) return t.cols % 8 == 0 && t.cols >= 64;
    return true;
}

// Segments [first, end) of a tensor that does not fit the row path: one lane per
// segment, element by element, the whole workgroup striding over them.
template <int MODE, class TB>
__device__ __forceinline__ void scalar_chunks(const DevTensor &t, const TB &tb, uint32_t first, uint32_t end) {
    constexpr uint32_t WG = 64 * Cfg<MODE>::waves;
    for (uint32_t k = first + threadIdx.x; k < end; k += WG) {
        if constexpr (is_gemv(MODE)) {
            gemv_segment<MODE>(t, tb, k);
        } else {
            const uint64_t left = t.n - static_cast<uint64_t>(k) * t.chunk_symbols;
            decode_scalar<MODE>(t, tb, k, left < t.chunk_symbols ? static_cast<uint32_t>(left) : t.chunk_symbols);
        }
    }
}

// One tensor per launch: workgroup b builds the tables and takes `wg_units` units
// (kUnit segments each, one unit per wavefront; at most as many as it has
// wavefronts) from unit b * wg_units on.
template <int MODE>
__device__ __forceinline__ void single_body(const DevTensor &t, uint32_t wg_units) {
    constexpr uint32_t WG = 64 * Cfg<MODE>::waves;
    __shared__ SmemFor<MODE> sm;
    // the per-wave symbol counts of the build live in the first wave's buffers, which are not in use yet
    build_tables<WG, kPairMode<MODE>>(t, sm.tb, reinterpret_cast<uint32_t *>(sm.wm));
    const uint32_t first = blockIdx.x * wg_units * kUnit;
    if (rows_fit<MODE>(t)) {
        const uint32_t wave = threadIdx.x >> 6;
        if (wave < wg_units) {
            if constexpr (wide_gemv(MODE)) gemv_direct2<MODE>(t, sm.tb, sm.wm[wave].ring, first + wave * kUnit);
            else if constexpr (is_gemv(MODE)) gemv_direct<MODE>(t, sm.tb, sm.wm[wave].ring, first + wave * kUnit);
            else if constexpr (short_ring(MODE)) decode_rows2<MODE>(t, sm.tb, sm.wm, first + wave * kUnit);
            else decode_rows<MODE>(t, sm.tb, sm.wm, first + wave * kUnit);
        }
    } else {
        const uint32_t end = first + wg_units * kUnit;
        scalar_chunks<MODE>(t, sm.tb, first, end < t.n_chunks ? end : t.n_chunks);
    }
}

// Many tensors per launch.  A unit is kUnit consecutive segments of one tensor:
// what a wavefront decodes at a time.  The work list has one item per
// `item_units` units of a tensor (fewer at the tensor's end), in tensor order;
// workgroup b of G takes the items [b * n / G, (b + 1) * n / G): a few stretches
// of one tensor each.  Per stretch it loads the tensor's tables (or builds them, if the
// launch was not prepared with them), then its wavefronts draw units from a counter in
// LDS until the stretch is used up.  The wavefronts of a workgroup do not run equally
// fast (fourteen of them share four SIMDs unevenly; lanes meet long codes at different
// times), so a fixed split would leave the faster ones waiting.
template <int MODE>
__device__ __forceinline__ void batch_body(const DevTensor *__restrict__ tensors, const WorkItem *__restrict__ items,
                                           uint32_t n_items, uint32_t item_units) {
    constexpr uint32_t WG = 64 * Cfg<MODE>::waves;
    __shared__ SmemFor<MODE> sm;
    __shared__ uint32_t next_unit;
    const uint32_t lo = static_cast<uint32_t>(static_cast<uint64_t>(blockIdx.x) * n_items / gridDim.x);
    const uint32_t hi = static_cast<uint32_t>(static_cast<uint64_t>(blockIdx.x + 1) * n_items / gridDim.x);
    uint32_t i = lo;
    while (i < hi) {
        const WorkItem it = items[i];
        const DevTensor &t = tensors[it.tensor];
        // the stretch ends with the tensor or with the workgroup's share
        const uint32_t left_in_tensor = (t.n_chunks - it.first + kUnit - 1) / kUnit;
        const uint64_t share = static_cast<uint64_t>(hi - i) * item_units;
        const uint32_t n_units = left_in_tensor < share ? left_in_tensor : static_cast<uint32_t>(share);
        // The units beyond the stretch's last whole round (a unit per wavefront), where the tensor is described
        // a second time with finer lanes (t.fine): they are drawn as 2^fine_shift times as many short ones, so
        // that the wavefronts run out of work at nearly the same time instead of most of them idling for the
        // length of a whole segment.
        const DevTensor *tf = &t;
        uint32_t n_coarse = n_units, n_all = n_units, fine_first = 0;
        if (!is_gemv(MODE) && t.fine) {                      // (the GEMV's descriptions have none)
            tf = &tensors[t.fine];
            const uint32_t refined = n_units % static_cast<uint32_t>(Cfg<MODE>::waves);   // what does not fill a round
            n_coarse = n_units - refined;
            fine_first = (it.first + n_coarse * kUnit) << t.fine_shift;
            uint64_t fine_end = static_cast<uint64_t>(it.first + n_units * kUnit) << t.fine_shift;
            if (fine_end > tf->n_chunks) fine_end = tf->n_chunks;
            n_all = n_coarse + static_cast<uint32_t>((fine_end - fine_first + kUnit - 1) / kUnit);
        }
        __syncthreads();                                     // nobody reads the previous tables or the counter any more
        if (t.tables) {
            // built once when the launch was prepared: 16 bytes per lane and step from memory into LDS
            const u32x4 *src = static_cast<const u32x4 *>(t.tables);
            u32x4 *dst = reinterpret_cast<u32x4 *>(&sm.tb);
            for (uint32_t j = threadIdx.x; j < sizeof(sm.tb) / 16u; j += WG) dst[j] = src[j];
            __syncthreads();
        } else {
            build_tables<WG, kPairMode<MODE>>(t, sm.tb, reinterpret_cast<uint32_t *>(sm.wm));
        }
        if (rows_fit<MODE>(t)) {
            if (threadIdx.x == 0) next_unit = 0;
            __syncthreads();
            for (;;) {
                uint32_t u = 0;
                if ((threadIdx.x & 63u) == 0) u = atomicAdd(&next_unit, 1u);
                u = __builtin_amdgcn_readfirstlane(u);
                if (u >= n_all) break;
                const bool fine = !is_gemv(MODE) && u >= n_coarse;
                const DevTensor &d = fine ? *tf : t;
                const uint32_t first = fine ? fine_first + (u - n_coarse) * kUnit : it.first + u * kUnit;
                if constexpr (wide_gemv(MODE)) gemv_direct2<MODE>(d, sm.tb, sm.wm[threadIdx.x >> 6].ring, first);
                else if constexpr (is_gemv(MODE)) gemv_direct<MODE>(d, sm.tb, sm.wm[threadIdx.x >> 6].ring, first);
                else if constexpr (short_ring(MODE)) decode_rows2<MODE>(d, sm.tb, sm.wm, first);
                else decode_rows<MODE>(d, sm.tb, sm.wm, first);
            }
        } else {
            const uint32_t end = it.first + n_units * kUnit;
            scalar_chunks<MODE>(t, sm.tb, it.first, end < t.n_chunks ? end : t.n_chunks);
        }
        i += (n_units + item_units - 1) / item_units;
    }
}

template <int MODE>
__global__ __launch_bounds__(64 * Cfg<MODE>::waves) void k_single(const DevTensor t, uint32_t wg_units) {
    single_body<MODE>(t, wg_units);
}
template <int MODE>
__global__ __launch_bounds__(64 * Cfg<MODE>::waves) void k_batch(const DevTensor *__restrict__ tensors,
                                                                 const WorkItem *__restrict__ items, uint32_t n_items,
                                                                 uint32_t item_units) {
    batch_body<MODE>(tensors, items, n_items, item_units);
}

// The lookup tables of the tensors of a prepared launch, built once (workgroup b: tensor b) and kept in
// memory for the launch's workgroups to load.
template <int MODE>
__global__ __launch_bounds__(64 * Cfg<MODE>::waves) void k_tables(const DevTensor *__restrict__ tensors) {
    constexpr uint32_t WG = 64 * Cfg<MODE>::waves;
    __shared__ SmemFor<MODE> sm;
    const DevTensor &t = tensors[blockIdx.x];
    build_tables<WG, kPairMode<MODE>>(t, sm.tb, reinterpret_cast<uint32_t *>(sm.wm));
    static_assert(sizeof(sm.tb) % 16 == 0, "copied in 16-byte steps");
    const u32x4 *src = reinterpret_cast<const u32x4 *>(&sm.tb);
    u32x4 *dst = static_cast<u32x4 *>(t.tables);
    for (uint32_t j = threadIdx.x; j < sizeof(sm.tb) / 16u; j += WG) dst[j] = src[j];
}

// Second stage of the GEMV: the partial sums of a row that straddles lanes are added up by sixteen lanes,
// lane j taking every sixteenth of them in segment order, then the sixteen in a fixed tree (the same sum
// in the same order on every run).
constexpr int kFixWG = 256;                                   // threads of a workgroup
constexpr int kFixRows = kFixWG / 16;                         // and the rows it sums

template <int MODE>
__device__ __forceinline__ void fix_row(const DevTensor &t, uint32_t row, uint32_t j) {
    const bool live = row < t.rows;
    uint32_t k_lo = 1, k_hi = 0;
    if (live) {
        const uint64_t lo = static_cast<uint64_t>(row) * t.cols;
        k_lo = static_cast<uint32_t>(lo / t.chunk_symbols);
        k_hi = static_cast<uint32_t>((lo + t.cols - 1) / t.chunk_symbols);
    }
    float acc = 0.0f;
    for (uint64_t k = static_cast<uint64_t>(k_lo) + j; k <= k_hi; k += 16u) {
        const uint32_t first_row = static_cast<uint32_t>((k * t.chunk_symbols) / t.cols);
        acc += t.partials[2 * k + (first_row == row ? 0 : 1)];
    }
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) acc += __shfl_xor(acc, m, 64);
    if (!live || k_lo == k_hi || j != 0) return;             // (a whole row inside one lane's segment is stored already)
    const float y = acc * t.scale;
    if (gemv_f32(MODE)) reinterpret_cast<float *>(t.out)[row] = y;
    else reinterpret_cast<uint16_t *>(t.out)[row] = static_cast<uint16_t>(bf16_bits(y));
}

template <int MODE>
__global__ __launch_bounds__(kFixWG) void k_fix_single(const DevTensor t) {
    fix_row<MODE>(t, blockIdx.x * kFixRows + threadIdx.x / 16u, threadIdx.x & 15u);
}

template <int MODE>
__global__ __launch_bounds__(kFixWG) void k_fix_batch(const DevTensor *__restrict__ tensors,
                                                   const WorkItem *__restrict__ items) {
    const WorkItem it = items[blockIdx.x];
    fix_row<MODE>(tensors[it.tensor], it.first + threadIdx.x / 16u, threadIdx.x & 15u);
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

// log2 of the entry points per segment of a tensor (0: none inside the segments)
uint32_t sub_levels(const entro_tensor &t) {
    if (!t.sub_symbols || !t.chunk_symbols || t.chunk_symbols % t.sub_symbols) return 0;
    uint32_t per = t.chunk_symbols / t.sub_symbols, lg = 0;
    while ((1u << lg) < per) ++lg;
    return lg;
}

// Symbols a lane takes of this tensor when pieces are merged `level` times pairwise (at most up to whole segments).
uint64_t lane_symbols_at(const entro_tensor &t, uint32_t level) {
    if (!t.sub_symbols) return t.chunk_symbols;
    return static_cast<uint64_t>(t.sub_symbols) << std::min(level, sub_levels(t));
}

// How coarse the lanes of a launch over these tensors are: as coarse as still gives every lane slot of the
// device (`lane_slots`) a lane -- a lane's work is serial, so small launches are cut as fine as the entry
// points allow, and large ones as coarse as their segments, which costs the least per symbol.
uint32_t choose_level(const entro_tensor *ts, uint32_t count, uint64_t lane_slots) {
    uint32_t top = 0;
    for (uint32_t i = 0; i < count; ++i) top = std::max(top, sub_levels(ts[i]));
    for (uint32_t level = top; level > 0; --level) {
        uint64_t lanes = 0;
        for (uint32_t i = 0; i < count; ++i)
            if (ts[i].chunk_symbols) lanes += (ts[i].n + lane_symbols_at(ts[i], level) - 1) / lane_symbols_at(ts[i], level);
        if (lanes * 8 >= lane_slots * 7) return level;        // (seven eighths of the slots: one unit per wavefront beats two for most)
    }
    return 0;
}

entro_status fill_dev_tensor(const entro_tensor *t, entro_op op, entro_dtype d, uint32_t level, DevTensor *dt) {
    if (!t || !t->stream || !t->offsets || !t->out || !t->cb) return ENTRO_ERR_NULL;
    entro_status st = check_codebook(t->cb);
    if (st != ENTRO_OK) return st;
    const int bits = t->cb->bits;
    if (!dtype_ok(op, d, bits)) return ENTRO_ERR_SCHEME;
    if (t->n == 0 || t->chunk_symbols == 0 || t->chunk_symbols > kMaxChunkSymbols) return ENTRO_ERR_SIZE;
    if (d == ENTRO_U4_PACKED && (t->chunk_symbols & 1u)) return ENTRO_ERR_SIZE;
    // offsets into the stream are 32-bit numbers in the kernels, with room for a line or two past the end
    if (t->stream_bytes < 32 || (t->stream_bytes & 15u) || t->stream_bytes >= (uint64_t{1} << 32) - 65536)
        return ENTRO_ERR_SIZE;
    // the symbols one lane decodes: 2^level pieces, where the tensor has entry points inside its segments
    uint32_t lane_symbols = t->chunk_symbols, sub_shift = 0, sub_merge = 0;
    if (t->sub_symbols) {
        if (!t->sub_bits) return ENTRO_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(t->sub_bits) & 3u) return ENTRO_ERR_ALIGN;
        if (t->chunk_symbols % t->sub_symbols != 0) return ENTRO_ERR_SIZE;
        const uint32_t per = t->chunk_symbols / t->sub_symbols;
        if (per > ENTRO_MAX_SUB_PER_CHUNK || (per & (per - 1u)) != 0) return ENTRO_ERR_SIZE;
        if (d == ENTRO_U4_PACKED && (t->sub_symbols & 1u)) return ENTRO_ERR_SIZE;
        sub_merge = std::min(level, sub_levels(*t));
        sub_shift = sub_levels(*t) - sub_merge;
        lane_symbols = t->sub_symbols << sub_merge;
    }
    const uint64_t n_chunks = entro_num_chunks(t->n, lane_symbols);
    if (n_chunks >= (uint64_t{1} << 32) - 1024) return ENTRO_ERR_SIZE;
    if (!aligned16(t->stream) || !aligned16(t->offsets) || !aligned16(t->out)) return ENTRO_ERR_ALIGN;
    if (op != ENTRO_OP_DECODE && t->qp.bits != bits) return ENTRO_ERR_BITS;
    // the kernels subtract the zero-point in fp32, which must represent it exactly
    if (op != ENTRO_OP_DECODE && (t->qp.zero_point > (1 << 24) || t->qp.zero_point < -(1 << 24))) return ENTRO_ERR_RANGE;
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
    dt->chunk_symbols = lane_symbols;
    dt->n_chunks = static_cast<uint32_t>(n_chunks);
    dt->sub = sub_shift ? t->sub_bits : nullptr;
    dt->sub_shift = sub_shift;
    dt->sub_merge = sub_merge;
    dt->rows = t->rows;
    dt->cols = t->cols;
    dt->bits = static_cast<uint32_t>(bits);
    dt->scale = t->qp.scale;
    dt->zero_point = t->qp.zero_point;
    dt->max_len = static_cast<uint32_t>(t->cb->max_len);
    dt->need_fix = (op == ENTRO_OP_GEMV && (lane_symbols % t->cols) != 0) ? 1u : 0u;
    // rows cut into a power of two of lanes (at most a wavefront's 64) that all go through the kernels' block
    // path: the wavefront adds the row up itself
    if (dt->need_fix && t->cols % lane_symbols == 0 && lane_symbols % 128u == 0) {
        const uint32_t per_row = t->cols / lane_symbols;
        if (per_row <= 64u && (per_row & (per_row - 1u)) == 0) {
            dt->row_lanes = per_row;
            dt->need_fix = 0;
        }
    }
    std::memcpy(dt->len, t->cb->len, 256);
    return ENTRO_OK;
}

template <class F>
void dispatch_mode(int mode, F f) {
    switch (mode) {
        case kModeU8: f(std::integral_constant<int, kModeU8>{}); break;
        case kModeU4: f(std::integral_constant<int, kModeU4>{}); break;
        case kModeF32: f(std::integral_constant<int, kModeF32>{}); break;
        case kModeBF16: f(std::integral_constant<int, kModeBF16>{}); break;
        case kModeGemvF32: f(std::integral_constant<int, kModeGemvF32>{}); break;
        case kModeU8P: f(std::integral_constant<int, kModeU8P>{}); break;
        case kModeF32P: f(std::integral_constant<int, kModeF32P>{}); break;
        case kModeBF16P: f(std::integral_constant<int, kModeBF16P>{}); break;
        case kModeGemvF32P: f(std::integral_constant<int, kModeGemvF32P>{}); break;
        case kModeGemvBF16P: f(std::integral_constant<int, kModeGemvBF16P>{}); break;
        case kModeGemvF32W: f(std::integral_constant<int, kModeGemvF32W>{}); break;
        case kModeGemvBF16W: f(std::integral_constant<int, kModeGemvBF16W>{}); break;
        default: f(std::integral_constant<int, kModeGemvBF16>{}); break;
    }
}

// Lanes (= segments) per workgroup of the main kernel of a mode.
unsigned wg_of(int mode) {
    unsigned wg = 64;
    dispatch_mode(mode, [&](auto m) { wg = 64u * Cfg<decltype(m)::value>::waves; });
    return wg;
}

// Symbols per block of a mode's kernel: lanes must be whole blocks to go through its fast path.
unsigned spb_of(int mode) {
    unsigned spb = 64;
    dispatch_mode(mode, [&](auto m) { spb = Cfg<decltype(m)::value>::spb; });
    return spb;
}

// `pairs`: every tensor of the launch holds 4-bit symbols, so the tables can hold two codes per entry.
// Does the GEMV of this tensor fit the wide tables?
bool wide_ok(const DevTensor &dt) { return dt.bits == 8 && dt.zero_point >= -1 && dt.zero_point <= 256; }

// `wide`: a GEMV all of whose tensors hold 8-bit symbols with a zero-point in [-1, 256] (symbol - zero_point is a
// bf16 then, which the wide tables hold ready for use).
int mode_of(entro_op op, entro_dtype d, bool pairs, bool wide = false) {
    if (op == ENTRO_OP_GEMV) {
        if (pairs) return d == ENTRO_F32 ? kModeGemvF32P : kModeGemvBF16P;
        if (wide) return d == ENTRO_F32 ? kModeGemvF32W : kModeGemvBF16W;
        return d == ENTRO_F32 ? kModeGemvF32 : kModeGemvBF16;
    }
    switch (d) {
        case ENTRO_U8: return pairs ? kModeU8P : kModeU8;
        case ENTRO_U4_PACKED: return kModeU4;
        case ENTRO_F32: return pairs ? kModeF32P : kModeF32;
        default: return pairs ? kModeBF16P : kModeBF16;
    }
}


// Workgroups of the batched kernel of `mode` that the current device holds at once
// (its LDS footprint decides); 0 if the device cannot be asked.
unsigned resident_workgroups(int mode) {
    thread_local int cached_dev = -1, cached_cus = 0;
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return 0;
    if (dev != cached_dev) {
        int n = 0;
        if (!hip_ok(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev), "hipDeviceGetAttribute")) return 0;
        cached_dev = dev;
        cached_cus = n;
    }
    const int cus = cached_cus;
    size_t smem = 1;
    dispatch_mode(mode, [&](auto m) { smem = sizeof(SmemFor<decltype(m)::value>); });
    const unsigned per_cu = static_cast<unsigned>((160u * 1024u) / smem);
    return static_cast<unsigned>(cus) * (per_cu ? per_cu : 1u);
}

entro_status launch_single(const entro_tensor *t, entro_op op, entro_dtype d, float *partials,
                           void *hip_stream) {
    // all argument checks first, on the host alone; then the device is asked how many lanes it holds, which
    // decides how fine the lanes are cut
    DevTensor dt;
    entro_status st = fill_dev_tensor(t, op, d, 0, &dt);
    if (st != ENTRO_OK) return st;
    const int mode = mode_of(op, d, dt.bits == 4, wide_ok(dt));
    const unsigned wg = wg_of(mode);
    const unsigned slots = resident_workgroups(mode);
    if (slots == 0) return ENTRO_ERR_DEVICE;
    st = fill_dev_tensor(t, op, d, choose_level(t, 1, static_cast<uint64_t>(slots) * wg), &dt);
    if (st != ENTRO_OK) return st;
    dt.partials = partials;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // a unit per wavefront when the tensor is large; fewer units per workgroup, down to one, when
    // that would leave compute units without a workgroup
    const unsigned units = (dt.n_chunks + kUnit - 1) / kUnit;
    const unsigned wg_units = std::min(wg / 64u, std::max(1u, units / slots));
    const unsigned grid = (units + wg_units - 1) / wg_units;
    dispatch_mode(mode, [&](auto m) {
        constexpr int M = decltype(m)::value;
        hipLaunchKernelGGL(k_single<M>, dim3(grid), dim3(wg), 0, s, dt, static_cast<uint32_t>(wg_units));
    });
    if (!hip_ok(hipGetLastError(), "launch decode kernel")) return ENTRO_ERR_DEVICE;
    if (dt.need_fix) {
        const unsigned g2 = (dt.rows + kFixRows - 1) / kFixRows;
        if (gemv_f32(mode)) hipLaunchKernelGGL(k_fix_single<kModeGemvF32>, dim3(g2), dim3(kFixWG), 0, s, dt);
        else hipLaunchKernelGGL(k_fix_single<kModeGemvBF16>, dim3(g2), dim3(kFixWG), 0, s, dt);
        if (!hip_ok(hipGetLastError(), "launch row-sum kernel")) return ENTRO_ERR_DEVICE;
    }
    return ENTRO_OK;
}

// Device address of `scratch` on the current device, looked up once per device; nullptr if the
// lookup fails (the error text is kept for entro_last_device_error).
float *static_scratch() {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static float *ptrs[kMaxDevices] = {};
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        g_last_error = "device index beyond the static scratch table";
        return nullptr;
    }
    std::lock_guard<std::mutex> guard(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)")) return nullptr;
        ptrs[dev] = static_cast<float *>(p);
    }
    return ptrs[dev];
}

uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

// Symbols one lane decodes of this tensor (what the work list and the partial sums are counted in).
uint32_t lane_symbols_of(const entro_tensor &t) { return t.sub_symbols ? t.sub_symbols : t.chunk_symbols; }

struct Layout {
    uint64_t off_tensors, off_items, off_fix, off_partials, off_tables, total;
    uint32_t n_items, n_fix;
};
// room for one tensor's lookup tables in the workspace (the larger kind, whichever the launch uses)
constexpr uint64_t kTablesStride = (sizeof(Tables32) + 255) / 256 * 256;

// Workspace layout shared by entro_workspace_bytes and entro_plan_init.
bool plan_layout(const entro_tensor *ts, uint32_t count, entro_op op, Layout *L) {
    uint64_t items = 0, fix = 0, partial_floats = 0;
    for (uint32_t i = 0; i < count; ++i) {
        if (ts[i].chunk_symbols == 0 || ts[i].n == 0) return false;
        const uint64_t nc = entro_num_chunks(ts[i].n, lane_symbols_of(ts[i]));
        items += (nc + kUnit - 1) / kUnit;
        if (op == ENTRO_OP_GEMV && ts[i].cols && (lane_symbols_of(ts[i]) % ts[i].cols) != 0) {
            fix += (static_cast<uint64_t>(ts[i].rows) + kFixRows - 1) / kFixRows;
            partial_floats += 2 * nc;
        }
    }
    if (items >= (uint64_t{1} << 31) || fix >= (uint64_t{1} << 31)) return false;
    L->n_items = static_cast<uint32_t>(items);
    L->n_fix = static_cast<uint32_t>(fix);
    L->off_tensors = 0;
    L->off_items = align_up(sizeof(DevTensor) * 2 * static_cast<uint64_t>(count), 256);   // a tensor may be described at two lane sizes
    L->off_fix = L->off_items + align_up(sizeof(WorkItem) * items, 256);
    L->off_partials = L->off_fix + align_up(sizeof(WorkItem) * fix, 256);
    L->off_tables = L->off_partials + align_up(sizeof(float) * partial_floats, 256);
    L->total = L->off_tables + kTablesStride * count;
    return true;
}

}  // namespace

// for the library's other device source: record a failed HIP call for entro_last_device_error
void entro_detail_note_hip_error(const char *what, int hip_error) {
    hip_ok(static_cast<hipError_t>(hip_error), what);
}

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
    if ((lane_symbols_of(*t) % t->cols) == 0) return 0;
    return align_up(2 * sizeof(float) * entro_num_chunks(t->n, lane_symbols_of(*t)), 256);
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

entro_status entro_decode_gemv_static(const entro_tensor *t, entro_dtype y_type, void *hip_stream) {
    if (!t) return ENTRO_ERR_NULL;
    float *partials = nullptr;
    if (entro_gemv_workspace_bytes(t)) {
        if (entro_num_chunks(t->n, lane_symbols_of(*t)) > ENTRO_STATIC_GEMV_MAX_SEGMENTS) return ENTRO_ERR_CAPACITY;
        partials = static_scratch();
        if (!partials) return ENTRO_ERR_DEVICE;
    }
    return launch_single(t, ENTRO_OP_GEMV, y_type, partials, hip_stream);
}

uint64_t entro_workspace_bytes(const entro_tensor *ts, uint32_t count, entro_op op) {
    Layout L;
    if (!ts || count == 0 || !plan_layout(ts, count, op, &L)) return 0;
    return L.total;
}

// Validate, lay the table out in `host` (L.off_partials bytes) and fill in the plan; nothing touches the device.
static entro_status build_plan(entro_plan *plan, const entro_tensor *ts, uint32_t count, entro_op op, entro_dtype out_type,
                               void *workspace, uint64_t workspace_bytes, const Layout &L, unsigned char *host) {
    std::memset(host, 0, L.off_partials);
    DevTensor *dts = reinterpret_cast<DevTensor *>(host + L.off_tensors);
    WorkItem *items = reinterpret_cast<WorkItem *>(host + L.off_items);
    WorkItem *fix = reinterpret_cast<WorkItem *>(host + L.off_fix);
    uint64_t n_items = 0, n_fix = 0, partial_floats = 0, total_units = 0;
    bool pairs = true;                                       // every tensor 4-bit: two codes per table entry
    bool multirow = false;                                   // GEMV: a tensor's segments are longer than its rows
    float *partials_base = reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + L.off_partials);
    // how fine the lanes are cut is decided for the launch as a whole (all its tensors are 4-bit, or the
    // tables take single codes: the kernel and with it the lane slots are known before the tensors are looked at)
    // (all argument checks come first, on the host alone)
    bool all4 = true, wide = true;
    for (uint32_t i = 0; i < count; ++i) {
        entro_status st = fill_dev_tensor(&ts[i], op, out_type, 0, &dts[i]);
        if (st != ENTRO_OK) return st;
        all4 = all4 && dts[i].bits == 4;
        wide = wide && wide_ok(dts[i]);
    }
    const int mode0 = mode_of(op, out_type, all4, wide);
    const unsigned slots0 = resident_workgroups(mode0);
    if (slots0 == 0) return ENTRO_ERR_DEVICE;
    const uint32_t level = choose_level(ts, count, static_cast<uint64_t>(slots0) * wg_of(mode0));
    for (uint32_t i = 0; i < count; ++i) {
        entro_status st = fill_dev_tensor(&ts[i], op, out_type, level, &dts[i]);
        if (st != ENTRO_OK) return st;
        dts[i].tables = static_cast<unsigned char *>(workspace) + L.off_tables + kTablesStride * i;
        total_units += (dts[i].n_chunks + kUnit - 1) / kUnit;
        pairs = pairs && dts[i].bits == 4;
        multirow = multirow || (op == ENTRO_OP_GEMV && dts[i].cols < dts[i].chunk_symbols);
        if (dts[i].need_fix) {
            dts[i].partials = partials_base + partial_floats;
            partial_floats += 2 * static_cast<uint64_t>(dts[i].n_chunks);
            for (uint32_t r = 0; r < dts[i].rows; r += kFixRows) fix[n_fix++] = WorkItem{i, r};
        }
    }
    // A work item is what a workgroup takes in one round when the launch is large (a unit per
    // wavefront: stretches of whole items end for all wavefronts together), and less when the launch
    // would not give every compute unit an item otherwise.
    const int mode = mode0;
    const unsigned slots = slots0;
    const uint64_t waves = wg_of(mode) / 64u;
    uint32_t item_units = static_cast<uint32_t>(std::min<uint64_t>(waves, std::max<uint64_t>(1, total_units / slots)));
    // Tensors with entry points inside their segments are described a second time, with lanes up to
    // 2^kTailShift times finer (as fine as still tiles into the kernel's blocks): the kernel draws what
    // is left over behind the last whole round of a stretch from that description.  (Not for the GEMV: its partial sums are laid out per lane.)
    uint32_t n_desc = count;
    const uint32_t block = spb_of(mode);
    for (uint32_t i = 0; i < count && op != ENTRO_OP_GEMV; ++i) {
        uint32_t finer = std::min<uint32_t>(dts[i].sub_merge, kTailShift);
        while (finer > 0 && ((dts[i].chunk_symbols >> finer) % block) != 0) --finer;
        if (finer == 0 || dts[i].chunk_symbols % block != 0) continue;
        entro_status st = fill_dev_tensor(&ts[i], op, out_type, dts[i].sub_merge - finer, &dts[n_desc]);
        if (st != ENTRO_OK) return st;
        dts[n_desc].tables = dts[i].tables;
        dts[i].fine = n_desc++;
        dts[i].fine_shift = finer;
    }
    // where every tensor has that second description a stretch may end anywhere at little cost: the
    // workgroups' shares are made equal to within one unit
    if (n_desc == 2 * count) item_units = 1;
    for (uint32_t i = 0; i < count; ++i)
        for (uint64_t c = 0; c < dts[i].n_chunks; c += static_cast<uint64_t>(item_units) * kUnit) {
            if (n_items >= L.n_items) return ENTRO_ERR_SIZE;     // (the layout counts the same units: cannot happen)
            items[n_items++] = WorkItem{i, static_cast<uint32_t>(c)};
        }
    plan->workspace = workspace;
    plan->workspace_bytes = workspace_bytes;
    plan->op = op;
    plan->out = out_type;
    plan->count = count;
    plan->n_items = static_cast<uint32_t>(n_items);
    plan->n_fix = static_cast<uint32_t>(n_fix);
    plan->item_units = item_units;
    plan->pair_tables = pairs ? 1u : 0u;
    plan->wide_tables = (op == ENTRO_OP_GEMV && !pairs && wide) ? 1u : 0u;
    plan->gemv_multirow = multirow ? 1u : 0u;
    plan->off_tensors = L.off_tensors;
    plan->off_items = L.off_items;
    plan->off_partials = L.off_partials;
    plan->off_fix = L.off_fix;
    return ENTRO_OK;
}

static entro_status plan_checks(entro_plan *plan, const entro_tensor *ts, uint32_t count, entro_op op, void *workspace,
                                uint64_t workspace_bytes, Layout *L) {
    if (!plan || !ts || !workspace) return ENTRO_ERR_NULL;
    if (count == 0) return ENTRO_ERR_SIZE;
    if (op != ENTRO_OP_DECODE && op != ENTRO_OP_DEQUANT && op != ENTRO_OP_GEMV) return ENTRO_ERR_SCHEME;
    if (!aligned16(workspace)) return ENTRO_ERR_ALIGN;
    if (!plan_layout(ts, count, op, L)) return ENTRO_ERR_SIZE;
    if (workspace_bytes < L->total) return ENTRO_ERR_CAPACITY;
    return ENTRO_OK;
}

// Enqueue the kernel that builds every tensor's lookup tables into the workspace (behind the copy of the
// descriptor table on the same stream).
static entro_status enqueue_tables(const entro_plan *plan, hipStream_t s) {
    const DevTensor *dts = reinterpret_cast<const DevTensor *>(static_cast<const unsigned char *>(plan->workspace) + plan->off_tensors);
    const int mode = mode_of(static_cast<entro_op>(plan->op), static_cast<entro_dtype>(plan->out), plan->pair_tables != 0,
                             plan->wide_tables != 0);
    dispatch_mode(mode, [&](auto m) {
        constexpr int M = decltype(m)::value;
        hipLaunchKernelGGL(k_tables<M>, dim3(plan->count), dim3(wg_of(mode)), 0, s, dts);
    });
    return hip_ok(hipGetLastError(), "launch table kernel") ? ENTRO_OK : ENTRO_ERR_DEVICE;
}

uint64_t entro_plan_staging_bytes(const entro_tensor *ts, uint32_t count, entro_op op) {
    Layout L;
    if (!ts || count == 0 || !plan_layout(ts, count, op, &L)) return 0;
    return L.off_partials;
}

entro_status entro_plan_init_staged(entro_plan *plan, const entro_tensor *ts, uint32_t count, entro_op op,
                                    entro_dtype out_type, void *workspace, uint64_t workspace_bytes, void *staging,
                                    uint64_t staging_bytes, void *hip_stream) {
    Layout L;
    entro_status st = plan_checks(plan, ts, count, op, workspace, workspace_bytes, &L);
    if (st != ENTRO_OK) return st;
    if (!staging) return ENTRO_ERR_NULL;
    if (staging_bytes < L.off_partials) return ENTRO_ERR_CAPACITY;
    st = build_plan(plan, ts, count, op, out_type, workspace, workspace_bytes, L, static_cast<unsigned char *>(staging));
    if (st != ENTRO_OK) return st;
    if (!hip_ok(hipMemcpyAsync(workspace, staging, L.off_partials, hipMemcpyHostToDevice, static_cast<hipStream_t>(hip_stream)),
                "copy plan table"))
        return ENTRO_ERR_DEVICE;
    return enqueue_tables(plan, static_cast<hipStream_t>(hip_stream));
}

entro_status entro_plan_init(entro_plan *plan, const entro_tensor *ts, uint32_t count, entro_op op,
                             entro_dtype out_type, void *workspace, uint64_t workspace_bytes,
                             void *hip_stream) {
    Layout L;
    entro_status st = plan_checks(plan, ts, count, op, workspace, workspace_bytes, &L);
    if (st != ENTRO_OK) return st;
    std::vector<unsigned char> host(L.off_partials);
    st = build_plan(plan, ts, count, op, out_type, workspace, workspace_bytes, L, host.data());
    if (st != ENTRO_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (!hip_ok(hipMemcpyAsync(workspace, host.data(), host.size(), hipMemcpyHostToDevice, s), "copy plan table"))
        return ENTRO_ERR_DEVICE;
    // the staging vector dies with this call, so wait for the copy
    if (!hip_ok(hipStreamSynchronize(s), "wait for plan table")) return ENTRO_ERR_DEVICE;
    return enqueue_tables(plan, s);
}

entro_status entro_plan_run(const entro_plan *plan, void *hip_stream) {
    if (!plan || !plan->workspace) return ENTRO_ERR_NULL;
    if (plan->n_items == 0 || plan->item_units == 0) return ENTRO_ERR_SIZE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const unsigned char *ws = static_cast<const unsigned char *>(plan->workspace);
    const DevTensor *dts = reinterpret_cast<const DevTensor *>(ws + plan->off_tensors);
    const WorkItem *items = reinterpret_cast<const WorkItem *>(ws + plan->off_items);
    const WorkItem *fix = reinterpret_cast<const WorkItem *>(ws + plan->off_fix);
    const int mode = mode_of(static_cast<entro_op>(plan->op), static_cast<entro_dtype>(plan->out), plan->pair_tables != 0,
                             plan->wide_tables != 0);
    const unsigned slots = resident_workgroups(mode);
    if (slots == 0) return ENTRO_ERR_DEVICE;
    const unsigned grid = plan->n_items < slots ? plan->n_items : slots;
    dispatch_mode(mode, [&](auto m) {
        constexpr int M = decltype(m)::value;
        hipLaunchKernelGGL(k_batch<M>, dim3(grid), dim3(wg_of(mode)), 0, s, dts, items, plan->n_items, plan->item_units);
    });
    if (!hip_ok(hipGetLastError(), "launch batched decode kernel")) return ENTRO_ERR_DEVICE;
    if (plan->n_fix) {
        if (gemv_f32(mode)) hipLaunchKernelGGL(k_fix_batch<kModeGemvF32>, dim3(plan->n_fix), dim3(kFixWG), 0, s, dts, fix);
        else hipLaunchKernelGGL(k_fix_batch<kModeGemvBF16>, dim3(plan->n_fix), dim3(kFixWG), 0, s, dts, fix);
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
