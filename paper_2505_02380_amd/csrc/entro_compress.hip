// Compression side of libentro on the GPU: the steps that come before the
// decode path, for weights that already sit in device memory.
//
// EntroLLM's offline pipeline (Proposed Method: "Mixed Quantization Scheme",
// Eq. 1 / Fig. 2; "Huffman weight encoding"; "Segmentation for parallel
// Huffman decoding", Fig. 3) is range -> (s, z) -> integer grid -> symbol
// counts -> prefix code -> segmented bit stream.  Three of those steps touch
// every weight and run here as kernels (range, quantise + count, encode); the
// two that touch only 256 numbers ((s, z) from the range, the code from the
// counts) stay on the host between them.
//
// Encoding is segment-parallel like decoding: a first kernel adds up the code
// lengths of every segment, a scan turns them into the bit-offset table, and a
// third kernel has one wavefront write one segment.  Within a segment the
// wavefront takes 256 symbols at a time (one aligned dword of four symbols per
// lane), a prefix sum over the lanes' code lengths gives every code its bit
// position, and the lanes OR their codes into a staging buffer in LDS, whose
// whole dwords then go to memory in one coalesced store per 64 dwords.
// Segments are bit-packed back to back, so the first and the last dword of a
// segment may be shared with its neighbours: those two are zeroed beforehand
// and OR-ed into atomically, everything between is stored plainly.
#include "entro.h"

#include <hip/hip_runtime.h>

#include <cstring>

// defined beside entro_last_device_error
void entro_detail_note_hip_error(const char *what, int hip_error);

namespace {

constexpr int kWG = 256;                       // four wavefronts
constexpr int kWaves = kWG / 64;
// The two streaming kernels run one large workgroup per compute unit with many loads in flight per lane:
// what a workgroup finds goes into a few words of memory by atomics, and those queue up, so the fewer
// workgroups the better.
constexpr int kBigWG = 1024;
constexpr int kBigWaves = kBigWG / 64;
constexpr int kHistCopies = 8;                 // counters per bin and set of waves, picked by lane: spreads the hits on the few frequent symbols
constexpr int kPrefetch = 8;                   // dwords of symbols a lane requests together
constexpr uint64_t kMissBit = 1ull << 63;       // in a segment's bit count: it holds a symbol without a code
constexpr uint32_t kFlagSymbol = 1u;           // a symbol without a code (or >= 2^bits)
constexpr uint32_t kFlagCapacity = 2u;         // the stream does not fit stream_cap
constexpr uint32_t kFlagSize = 4u;             // the stream would reach 4 GiB

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

bool hip_ok(hipError_t e, const char *what) {
    if (e == hipSuccess) return true;
    entro_detail_note_hip_error(what, static_cast<int>(e));
    return false;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Number of workgroups for a grid-stride kernel over `items` work items of one thread each.
unsigned grid_for(uint64_t items, unsigned per_cu, unsigned wg = kWG) {
    thread_local int cached_dev = -1, cached_cus = 0;
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return 0;
    if (dev != cached_dev) {
        int n = 0;
        if (!hip_ok(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev), "hipDeviceGetAttribute")) return 0;
        cached_dev = dev;
        cached_cus = n;
    }
    const uint64_t want = (items + wg - 1) / wg;
    const uint64_t cap = static_cast<uint64_t>(cached_cus) * per_cu;
    const uint64_t g = want < cap ? want : cap;
    return static_cast<unsigned>(g ? g : 1);
}

__device__ __forceinline__ void wave_sync_lds() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// floats as unsigned keys of the same order (negative values below positive ones)
__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// ------------------------------------------------------------------ range
__global__ void k_range_init(uint32_t *r) {
    r[0] = 0xffffffffu;   // smallest key seen
    r[1] = 0u;            // largest key seen
    r[2] = 0u;            // NaN / Inf seen
    r[3] = 0u;
}

__global__ __launch_bounds__(kBigWG) void k_range(const float *__restrict__ w, uint64_t n, uint32_t *__restrict__ r) {
    constexpr int kLoads = 8;                            // loads in flight per lane
    const uint64_t n4 = n >> 2;
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kBigWG;
    const uint64_t gid = static_cast<uint64_t>(blockIdx.x) * kBigWG + threadIdx.x;
    float lo = __uint_as_float(0x7f800000u), hi = __uint_as_float(0xff800000u);
    uint32_t bad = 0;
    auto take = [&](float v) {
        bad |= ((__float_as_uint(v) & 0x7f800000u) == 0x7f800000u) ? 1u : 0u;
        lo = v < lo ? v : lo;
        hi = v > hi ? v : hi;
    };
    const f32x4 *w4 = reinterpret_cast<const f32x4 *>(w);
    uint64_t i = gid;
    for (; i + (kLoads - 1) * stride < n4; i += kLoads * stride) {
        f32x4 v[kLoads];
#pragma unroll
        for (int j = 0; j < kLoads; ++j) v[j] = w4[i + j * stride];
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            take(v[j].x); take(v[j].y); take(v[j].z); take(v[j].w);
        }
    }
    for (; i < n4; i += stride) {
        const f32x4 a = w4[i];
        take(a.x); take(a.y); take(a.z); take(a.w);
    }
    if (gid < (n & 3u)) take(w[(n4 << 2) + gid]);
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const float l2 = __shfl_xor(lo, m, 64), h2 = __shfl_xor(hi, m, 64);
        lo = l2 < lo ? l2 : lo;
        hi = h2 > hi ? h2 : hi;
        bad |= __shfl_xor(bad, m, 64);
    }
    __shared__ float wlo[kBigWaves], whi[kBigWaves];
    __shared__ uint32_t wbad[kBigWaves];
    if ((threadIdx.x & 63u) == 0) {
        wlo[threadIdx.x >> 6] = lo;
        whi[threadIdx.x >> 6] = hi;
        wbad[threadIdx.x >> 6] = bad;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int wv = 1; wv < kBigWaves; ++wv) {
            lo = wlo[wv] < lo ? wlo[wv] : lo;
            hi = whi[wv] > hi ? whi[wv] : hi;
            bad |= wbad[wv];
        }
        // a workgroup that saw nothing still holds +Inf / -Inf, which lose against every finite value;
        // only a workgroup that improves on what is there already (the values only ever move one way)
        // sends an atomic
        const uint32_t klo = order_key(lo), khi = order_key(hi);
        if (klo < __hip_atomic_load(&r[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMin(&r[0], klo);
        if (khi > __hip_atomic_load(&r[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(&r[1], khi);
        if (bad) atomicOr(&r[2], 1u);
    }
}

__global__ void k_range_finish(uint32_t *r) {
    r[0] = __float_as_uint(key_value(r[0]));
    r[1] = __float_as_uint(key_value(r[1]));
}

// ------------------------------------------------------- quantise and count
__global__ void k_zero_counts(unsigned long long *counts) { counts[threadIdx.x] = 0ull; }

// Eq. 1 on one weight: true division, round half to even, zero-point added in
// integers, clamped to the grid.  |z| <= 2^24 (checked on the host), so
// limiting the rounded quotient to +-2^30 first changes no result.
__device__ __forceinline__ uint32_t quantize_one(float v, float s, int32_t z, int32_t Q) {
    float r = __builtin_rintf(v / s);
    r = r < -1073741824.0f ? -1073741824.0f : (r > 1073741824.0f ? 1073741824.0f : r);
    int32_t q = static_cast<int32_t>(r) + z;
    q = q < 0 ? 0 : (q > Q ? Q : q);
    return static_cast<uint32_t>(q);
}

constexpr int kHistSets = 4;                     // histograms per workgroup, picked by wave
__global__ __launch_bounds__(kBigWG) void k_quantize(const float *__restrict__ w, uint64_t n, float s, int32_t z, int32_t Q,
                                                     uint8_t *__restrict__ q, unsigned long long *__restrict__ counts) {
    constexpr int kLoads = 4;                            // loads in flight per lane
    // hist[set][bin][copy]: the copies of a bin lie in neighbouring banks
    __shared__ uint32_t hist[kHistSets * 256 * kHistCopies];
    for (int i = threadIdx.x; i < kHistSets * 256 * kHistCopies; i += kBigWG) hist[i] = 0;
    __syncthreads();
    uint32_t *mine = hist + ((threadIdx.x >> 6) & (kHistSets - 1)) * (256 * kHistCopies) + (threadIdx.x & (kHistCopies - 1));
    const uint64_t n4 = n >> 2;
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * kBigWG;
    const uint64_t gid = static_cast<uint64_t>(blockIdx.x) * kBigWG + threadIdx.x;
    const f32x4 *w4 = reinterpret_cast<const f32x4 *>(w);
    uint32_t *q4 = reinterpret_cast<uint32_t *>(q);
    auto four = [&](const f32x4 v) {
        const uint32_t a = quantize_one(v.x, s, z, Q), b = quantize_one(v.y, s, z, Q), c = quantize_one(v.z, s, z, Q),
                       d = quantize_one(v.w, s, z, Q);
        atomicAdd(&mine[a * kHistCopies], 1u);
        atomicAdd(&mine[b * kHistCopies], 1u);
        atomicAdd(&mine[c * kHistCopies], 1u);
        atomicAdd(&mine[d * kHistCopies], 1u);
        return a | (b << 8) | (c << 16) | (d << 24);
    };
    uint64_t i = gid;
    for (; i + (kLoads - 1) * stride < n4; i += kLoads * stride) {
        f32x4 v[kLoads];
#pragma unroll
        for (int j = 0; j < kLoads; ++j) v[j] = w4[i + j * stride];
#pragma unroll
        for (int j = 0; j < kLoads; ++j) q4[i + j * stride] = four(v[j]);
    }
    for (; i < n4; i += stride) q4[i] = four(w4[i]);
    if (gid < (n & 3u)) {
        const uint32_t a = quantize_one(w[(n4 << 2) + gid], s, z, Q);
        q[(n4 << 2) + gid] = static_cast<uint8_t>(a);
        atomicAdd(&mine[a * kHistCopies], 1u);
    }
    __syncthreads();
    if (threadIdx.x < 256) {                             // thread t owns bin t
        unsigned long long sum = 0;                      // a counter stays below 2^32 for tensors of up to 2^44 symbols
        for (int st = 0; st < kHistSets; ++st)
            for (int c = 0; c < kHistCopies; ++c) sum += hist[st * (256 * kHistCopies) + threadIdx.x * kHistCopies + c];
        if (sum) atomicAdd(&counts[threadIdx.x], sum);
    }
}

// ------------------------------------------------------------------ encode
struct EncTable {
    uint32_t rev[256];    // the code's bits in stream order: first code bit in bit 0
    uint8_t len[256];     // 0: no code
};

// Bits of every segment, into offsets[k + 1]; one wavefront per segment.
__global__ __launch_bounds__(kWG) void k_segment_bits(const uint8_t *__restrict__ q, uint64_t n, uint32_t chunk_symbols,
                                                      uint32_t n_chunks, const EncTable tab, uint64_t *__restrict__ offsets) {
    __shared__ uint8_t len[256];
    len[threadIdx.x] = tab.len[threadIdx.x];
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t *q32 = reinterpret_cast<const uint32_t *>(q);
    for (uint64_t k = static_cast<uint64_t>(blockIdx.x) * kWaves + (threadIdx.x >> 6); k < n_chunks;
         k += static_cast<uint64_t>(gridDim.x) * kWaves) {
        const uint64_t b0 = k * chunk_symbols;
        const uint64_t b1 = b0 + chunk_symbols < n ? b0 + chunk_symbols : n;
        // the aligned dwords that hold the segment's bytes; bytes of a dword outside [b0, b1) are skipped
        // (a dword with one byte inside the buffer lies inside the buffer's pages as a whole)
        const uint32_t skew = static_cast<uint32_t>(b0 & 3u);       // bytes of the first dword that are not the segment's
        const uint32_t nsym = static_cast<uint32_t>(b1 - b0);
        const uint32_t nd = (skew + nsym + 3u) >> 2;
        const uint32_t *src = q32 + (b0 >> 2);
        uint32_t sum = 0, miss = 0;
        for (uint32_t dd = 0; dd < nd; dd += 64 * kPrefetch) {
            uint32_t words[kPrefetch];
#pragma unroll
            for (int r = 0; r < kPrefetch; ++r) {
                const uint32_t ld = dd + 64u * r + lane;
                words[r] = ld < nd ? src[ld] : 0u;
            }
#pragma unroll
            for (int r = 0; r < kPrefetch; ++r) {
                const uint32_t rel = 4u * (dd + 64u * r + lane) - skew;   // wraps for the skipped bytes: not < nsym
#pragma unroll
                for (uint32_t j = 0; j < 4; ++j) {
                    const uint32_t l = len[(words[r] >> (8 * j)) & 0xffu];
                    const bool in = rel + j < nsym;
                    sum += in ? l : 0u;
                    miss |= (in && l == 0) ? 1u : 0u;
                }
            }
        }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            sum += __shfl_xor(sum, m, 64);
            miss |= __shfl_xor(miss, m, 64);
        }
        if (lane == 0) offsets[k + 1] = sum | (miss ? kMissBit : 0ull);
    }
}

__device__ __forceinline__ uint64_t padded_bytes(uint64_t total_bits) {
    uint64_t b = (total_bits + 7) / 8;
    b = (b + 15) / 16 * 16;
    return b + 16;
}

// offsets[k + 1] holds segment k's bits on entry (bit 63 set: it has a symbol without a code) and the
// stream bit behind segment k on exit.  One workgroup walks the table in tiles of eight entries per
// thread, sets the status word, and, if all is well, clears the stream dwords that are OR-ed into
// rather than stored: the one every segment starts in (which is also the one the segment before ends
// in, and for k = n_chunks the stream's last, partial one) and the padding behind the last code.
// Everything else is overwritten as whole dwords.  (zero_here false: the table is long, and a kernel
// of many workgroups clears them instead; one workgroup's scattered stores take too long then.)
constexpr int kScanWG = 1024;
constexpr int kScanPer = 8;                  // table entries per thread and tile
__global__ __launch_bounds__(kScanWG) void k_scan_offsets(uint64_t *__restrict__ offsets, uint32_t n_chunks,
                                                          uint32_t *__restrict__ stream, uint64_t stream_cap,
                                                          uint32_t *__restrict__ status, bool zero_here) {
    __shared__ uint64_t wave_sum[kScanWG / 64];
    __shared__ uint64_t carry_s;
    __shared__ uint32_t flags_s;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) {
        offsets[0] = 0;
        carry_s = 0;
        flags_s = 0;
    }
    __syncthreads();
    bool miss = false;
    for (uint64_t base = 0; base < n_chunks; base += kScanPer * kScanWG) {
        const uint64_t at = base + static_cast<uint64_t>(kScanPer) * threadIdx.x;
        uint64_t v[kScanPer];
#pragma unroll
        for (int j = 0; j < kScanPer; ++j) {
            v[j] = at + j < n_chunks ? offsets[at + j + 1] : 0;
            miss |= (v[j] & kMissBit) != 0;
            v[j] &= ~kMissBit;
        }
#pragma unroll
        for (int j = 1; j < kScanPer; ++j) v[j] += v[j - 1];
        uint64_t x = v[kScanPer - 1];
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            const uint64_t y = __shfl_up(x, m, 64);
            if (lane >= static_cast<uint32_t>(m)) x += y;
        }
        if (lane == 63) wave_sum[wave] = x;
        __syncthreads();
        uint64_t before = carry_s;
        for (uint32_t wv = 0; wv < wave; ++wv) before += wave_sum[wv];
        before += x - v[kScanPer - 1];
#pragma unroll
        for (int j = 0; j < kScanPer; ++j)
            if (at + j < n_chunks) offsets[at + j + 1] = before + v[j];
        __syncthreads();
        if (threadIdx.x == kScanWG - 1) carry_s = before + v[kScanPer - 1];
        __syncthreads();
    }
    if (miss) atomicOr(&flags_s, kFlagSymbol);
    __syncthreads();                                     // also: the offsets written above are visible to the whole workgroup
    const uint64_t total = carry_s;
    const uint64_t need = padded_bytes(total);
    uint32_t flags = flags_s;
    if (need > stream_cap) flags |= kFlagCapacity;
    if (need >= (1ull << 32)) flags |= kFlagSize;
    if (threadIdx.x == 0) *status = flags;
    if (flags || !zero_here) return;
    const uint64_t pad0 = total >> 5, pad1 = need >> 2;  // the last partial dword and the padding
    const uint64_t items = static_cast<uint64_t>(n_chunks) + (pad1 - pad0);
    for (uint64_t base = 0; base < items; base += 8 * kScanWG) {      // eight independent loads per thread and trip
        uint64_t g[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint64_t i = base + static_cast<uint64_t>(j) * kScanWG + threadIdx.x;
            g[j] = i < n_chunks ? offsets[i] >> 5 : pad0 + (i - n_chunks);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (base + static_cast<uint64_t>(j) * kScanWG + threadIdx.x < items) stream[g[j]] = 0u;   // g < need / 4 <= stream_cap / 4
    }
}

__global__ __launch_bounds__(kWG) void k_zero_shared_dwords(uint32_t *__restrict__ stream, const uint64_t *__restrict__ offsets,
                                                            uint32_t n_chunks, const uint32_t *__restrict__ status) {
    if (*status != 0u) return;
    const uint64_t total = offsets[n_chunks];
    const uint64_t pad0 = total >> 5, pad1 = padded_bytes(total) >> 2;
    const uint64_t items = static_cast<uint64_t>(n_chunks) + (pad1 - pad0);
    for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * kWG + threadIdx.x; i < items;
         i += static_cast<uint64_t>(gridDim.x) * kWG)
        stream[i < n_chunks ? offsets[i] >> 5 : pad0 + (i - n_chunks)] = 0u;     // inside the stream: status 0 says it fits
}

// One wavefront writes one segment.  The stage is a ring of dwords addressed by the bit position
// counted from the start of the stream dword the segment begins in; a round adds at most 256 codes
// of 32 bits and every round's whole dwords leave at once, so 512 dwords never wrap onto live ones.
constexpr int kStageRing = 512;
__global__ __launch_bounds__(kWG) void k_write_segments(const uint8_t *__restrict__ q, uint64_t n, uint32_t chunk_symbols,
                                                        uint32_t n_chunks, const EncTable tab,
                                                        const uint64_t *__restrict__ offsets, uint32_t *__restrict__ stream,
                                                        uint64_t stream_dwords, const uint32_t *__restrict__ status) {
    __shared__ uint64_t entry[256];                      // rev | len << 32
    __shared__ uint32_t stage_all[kWaves][kStageRing];
    entry[threadIdx.x] = tab.rev[threadIdx.x] | (static_cast<uint64_t>(tab.len[threadIdx.x]) << 32);
    for (int i = threadIdx.x; i < kWaves * kStageRing; i += kWG) (&stage_all[0][0])[i] = 0;
    __syncthreads();
    if (*status != 0u) return;                           // a symbol without a code, or no room: nothing is written
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t *stage = stage_all[threadIdx.x >> 6];
    const uint32_t *q32 = reinterpret_cast<const uint32_t *>(q);
    for (uint64_t k = static_cast<uint64_t>(blockIdx.x) * kWaves + (threadIdx.x >> 6); k < n_chunks;
         k += static_cast<uint64_t>(gridDim.x) * kWaves) {
        const uint64_t b0 = k * chunk_symbols;
        const uint64_t b1 = b0 + chunk_symbols < n ? b0 + chunk_symbols : n;
        const uint32_t skew = static_cast<uint32_t>(b0 & 3u);       // bytes of the first dword that are not the segment's
        const uint32_t nsym = static_cast<uint32_t>(b1 - b0);
        const uint32_t nd = (skew + nsym + 3u) >> 2;
        const uint32_t *src = q32 + (b0 >> 2);
        const uint64_t start = offsets[k];
        uint32_t *const out = stream + (start >> 5);     // the stream dword the segment starts in
        const uint64_t room = stream_dwords > (start >> 5) ? stream_dwords - (start >> 5) : 0;   // dwords up to the end of the buffer
        uint32_t fill = static_cast<uint32_t>(start & 31u);   // bits written, counted from bit 0 of that dword
        uint32_t done = 0;                               // dwords that have left the stage
        // dword i of the segment leaves the stage; the first one may hold the end of the segment before
        auto emit = [&](uint32_t i) {
            const uint32_t v = stage[i & (kStageRing - 1)];
            stage[i & (kStageRing - 1)] = 0;
            if (i < room) {
                if (i == 0) atomicOr(out, v);
                else out[i] = v;
            }
        };
        for (uint32_t dd = 0; dd < nd; dd += 64 * kPrefetch) {
            uint32_t words[kPrefetch];
#pragma unroll
            for (int r = 0; r < kPrefetch; ++r) {
                const uint32_t ld = dd + 64u * r + lane;
                words[r] = ld < nd ? src[ld] : 0u;
            }
#pragma unroll
            for (int r = 0; r < kPrefetch; ++r) {
                if (dd + 64u * r >= nd) break;           // the same for all lanes
                const uint32_t word = words[r];
                const uint32_t rel = 4u * (dd + 64u * r + lane) - skew;   // wraps for the skipped bytes: not < nsym
                // the lane's four codes, strung together in stream order: up to 128 bits in c[0..3];
                // a symbol that is not this segment's counts as no bits
                uint64_t pair[2];
                uint32_t plen[2];
#pragma unroll
                for (uint32_t h = 0; h < 2; ++h) {
                    const uint64_t e0 = entry[(word >> (16 * h)) & 0xffu], e1 = entry[(word >> (16 * h + 8)) & 0xffu];
                    const bool in0 = rel + 2 * h < nsym, in1 = rel + 2 * h + 1 < nsym;
                    const uint32_t l0 = in0 ? static_cast<uint32_t>(e0 >> 32) : 0u, l1 = in1 ? static_cast<uint32_t>(e1 >> 32) : 0u;
                    const uint32_t r0 = in0 ? static_cast<uint32_t>(e0) : 0u, r1 = in1 ? static_cast<uint32_t>(e1) : 0u;
                    pair[h] = r0 | (static_cast<uint64_t>(r1) << l0);          // l0 <= 32
                    plen[h] = l0 + l1;
                }
                const uint32_t tot = plen[0] + plen[1];
                const uint64_t lo = pair[0] | (plen[0] == 64u ? 0ull : pair[1] << (plen[0] & 63u));
                const uint64_t hi = plen[0] ? pair[1] >> ((64u - plen[0]) & 63u) : 0ull;
                const uint32_t c[4] = {static_cast<uint32_t>(lo), static_cast<uint32_t>(lo >> 32), static_cast<uint32_t>(hi),
                                       static_cast<uint32_t>(hi >> 32)};
                // inclusive prefix sum of the lanes' bit counts: within rows of 16 lanes by DPP shifts (a lane
                // without a source adds 0), then the three row totals in front of a row are added
                uint32_t x = tot;
                x += __builtin_amdgcn_update_dpp(0u, x, 0x111, 0xf, 0xf, true);    // row_shr:1
                x += __builtin_amdgcn_update_dpp(0u, x, 0x112, 0xf, 0xf, true);    // row_shr:2
                x += __builtin_amdgcn_update_dpp(0u, x, 0x114, 0xf, 0xf, true);    // row_shr:4
                x += __builtin_amdgcn_update_dpp(0u, x, 0x118, 0xf, 0xf, true);    // row_shr:8
                const uint32_t t0 = __builtin_amdgcn_readlane(x, 15), t1 = __builtin_amdgcn_readlane(x, 31),
                               t2 = __builtin_amdgcn_readlane(x, 47), t3 = __builtin_amdgcn_readlane(x, 63);
                x += (lane >= 16 ? t0 : 0u) + (lane >= 32 ? t1 : 0u) + (lane >= 48 ? t2 : 0u);
                const uint32_t round_bits = t0 + t1 + t2 + t3;
                // shifted to its place in the stage the string covers up to five dwords; the first two are
                // OR-ed in by every lane (zeros do no harm), the others only where a lane reaches them
                const uint32_t p = fill + x - tot;
                const uint32_t sh = p & 31u, at = p >> 5;
#pragma unroll
                for (uint32_t i = 0; i < 5; ++i) {
                    const uint32_t up = i < 4 ? c[i < 4 ? i : 0] : 0u, down = i ? c[i ? i - 1 : 0] : 0u;
                    // ({up, down} << sh) >> 32
                    const uint32_t v = sh ? __builtin_amdgcn_alignbit(up, down, 32u - sh) : up;
                    if (i < 2 || sh + tot > 32u * i) atomicOr(&stage[(at + i) & (kStageRing - 1)], v);
                }
                fill += round_bits;
                wave_sync_lds();
                // whole dwords leave 64 at a time
                while ((fill >> 5) - done >= 64u) {
                    emit(done + lane);
                    done += 64u;
                }
                wave_sync_lds();
            }
        }
        {
            const uint32_t full = fill >> 5;
            if (done + lane < full) emit(done + lane);
            done = full;
        }
        // what is left is shared with the next segment
        if (lane == 0 && (fill & 31u)) {
            const uint32_t c = stage[done & (kStageRing - 1)];
            stage[done & (kStageRing - 1)] = 0;
            if (done < room) atomicOr(out + done, c);
        }
        wave_sync_lds();
    }
}

EncTable make_table(const entro_codebook *cb) {
    EncTable t;
    std::memset(&t, 0, sizeof(t));
    for (int s = 0; s < (1 << cb->bits); ++s) {
        const uint32_t l = cb->len[s];
        if (!l) continue;
        uint32_t r = 0;
        for (uint32_t b = 0; b < l; ++b) r |= ((cb->code[s] >> (l - 1 - b)) & 1u) << b;
        t.rev[s] = r;
        t.len[s] = static_cast<uint8_t>(l);
    }
    return t;
}

}  // namespace

extern "C" {

entro_status entro_range_device(const float *w, uint64_t n, void *range16, void *hip_stream) {
    if (!w || !range16) return ENTRO_ERR_NULL;
    if (n == 0) return ENTRO_ERR_SIZE;
    if (!aligned16(w) || !aligned16(range16)) return ENTRO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const unsigned grid = grid_for((n + 3) / 4, 1, kBigWG);
    if (!grid) return ENTRO_ERR_DEVICE;
    uint32_t *r = static_cast<uint32_t *>(range16);
    hipLaunchKernelGGL(k_range_init, dim3(1), dim3(1), 0, st, r);
    hipLaunchKernelGGL(k_range, dim3(grid), dim3(kBigWG), 0, st, w, n, r);
    hipLaunchKernelGGL(k_range_finish, dim3(1), dim3(1), 0, st, r);
    return hip_ok(hipGetLastError(), "entro_range_device") ? ENTRO_OK : ENTRO_ERR_DEVICE;
}

entro_status entro_quantize_device(const float *w, uint64_t n, const entro_qparams *qp, uint8_t *q, uint64_t *counts,
                                   void *hip_stream) {
    if (!w || !qp || !q || !counts) return ENTRO_ERR_NULL;
    if (qp->bits != 4 && qp->bits != 8) return ENTRO_ERR_BITS;
    if (qp->scheme != ENTRO_UNSIGNED && qp->scheme != ENTRO_ASYMMETRIC) return ENTRO_ERR_SCHEME;
    if (n == 0) return ENTRO_ERR_SIZE;
    if (!(qp->scale > 0.0f) || qp->scale > 3.0e38f) return ENTRO_ERR_RANGE;
    if (qp->zero_point > (1 << 24) || qp->zero_point < -(1 << 24)) return ENTRO_ERR_RANGE;
    if (!aligned16(w) || !aligned16(q) || !aligned16(counts)) return ENTRO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const unsigned grid = grid_for((n + 3) / 4, 1, kBigWG);
    if (!grid) return ENTRO_ERR_DEVICE;
    unsigned long long *c = reinterpret_cast<unsigned long long *>(counts);
    hipLaunchKernelGGL(k_zero_counts, dim3(1), dim3(256), 0, st, c);
    hipLaunchKernelGGL(k_quantize, dim3(grid), dim3(kBigWG), 0, st, w, n, qp->scale, qp->zero_point, (1 << qp->bits) - 1, q, c);
    return hip_ok(hipGetLastError(), "entro_quantize_device") ? ENTRO_OK : ENTRO_ERR_DEVICE;
}

entro_status entro_encode_device(const uint8_t *q, uint64_t n, const entro_codebook *cb, uint32_t chunk_symbols, void *stream,
                                 uint64_t stream_cap, uint64_t *offsets, uint32_t *status, void *hip_stream) {
    if (!q || !cb || !stream || !offsets || !status) return ENTRO_ERR_NULL;
    if (cb->bits != 4 && cb->bits != 8) return ENTRO_ERR_BITS;
    if (n == 0 || chunk_symbols == 0 || chunk_symbols > (1u << 20)) return ENTRO_ERR_SIZE;
    if (cb->max_len < 1 || cb->max_len > ENTRO_MAX_CODE_LEN) return ENTRO_ERR_CORRUPT;
    for (int s = 0; s < ENTRO_MAX_SYMBOLS; ++s)
        if (cb->len[s] > cb->max_len || (s >= (1 << cb->bits) && cb->len[s])) return ENTRO_ERR_CORRUPT;
    {
        // the codes must be the canonical ones of the lengths: that is what every decoder rebuilds
        entro_codebook ref;
        if (entro_codebook_from_lengths(cb->len, cb->bits, &ref) != ENTRO_OK) return ENTRO_ERR_CORRUPT;
        for (int s = 0; s < (1 << cb->bits); ++s)
            if (ref.code[s] != cb->code[s]) return ENTRO_ERR_CORRUPT;
    }
    const uint64_t n_chunks = entro_num_chunks(n, chunk_symbols);
    if (n_chunks >= (uint64_t{1} << 32) - 1024) return ENTRO_ERR_SIZE;
    if (stream_cap < 32 || (stream_cap & 15u)) return ENTRO_ERR_CAPACITY;
    if (!aligned16(q) || !aligned16(stream) || !aligned16(offsets) || (reinterpret_cast<uintptr_t>(status) & 3u)) return ENTRO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const EncTable tab = make_table(cb);
    const unsigned grid = grid_for(n_chunks * 64, 8);
    if (!grid) return ENTRO_ERR_DEVICE;
    const uint32_t nc = static_cast<uint32_t>(n_chunks);
    hipLaunchKernelGGL(k_segment_bits, dim3(grid), dim3(kWG), 0, st, q, n, chunk_symbols, nc, tab, offsets);
    const bool zero_here = n_chunks <= 2048;
    hipLaunchKernelGGL(k_scan_offsets, dim3(1), dim3(kScanWG), 0, st, offsets, nc, static_cast<uint32_t *>(stream), stream_cap, status,
                       zero_here);
    if (!zero_here)
        hipLaunchKernelGGL(k_zero_shared_dwords, dim3(grid_for(n_chunks + 16, 8)), dim3(kWG), 0, st, static_cast<uint32_t *>(stream),
                           offsets, nc, status);
    hipLaunchKernelGGL(k_write_segments, dim3(grid), dim3(kWG), 0, st, q, n, chunk_symbols, nc, tab, offsets,
                       static_cast<uint32_t *>(stream), stream_cap / 4, status);
    return hip_ok(hipGetLastError(), "entro_encode_device") ? ENTRO_OK : ENTRO_ERR_DEVICE;
}

entro_status entro_encode_device_status(uint32_t status_word) {
    if (status_word & kFlagSymbol) return ENTRO_ERR_SYMBOL;
    if (status_word & kFlagCapacity) return ENTRO_ERR_CAPACITY;
    if (status_word & kFlagSize) return ENTRO_ERR_SIZE;
    return status_word ? ENTRO_ERR_CORRUPT : ENTRO_OK;
}

}  // extern "C"
