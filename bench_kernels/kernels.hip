// Comparison and calibration kernels for bench.py (gfx950); not part of the library.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cstdint>
#include "entro_bench.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const u32x4 __attribute__((address_space(1))) *global_u4_ptr;

// Read `rd` and write `wr` 16-byte blocks, perfectly coalesced (grid-stride), `ra` reads then `wa`
// writes per round, so that the two streams advance in the ratio of their sizes.
__global__ __launch_bounds__(1024) void k_stream_probe(const u32x4 *__restrict__ src, uint64_t rd, u32x4 *__restrict__ dst,
                                                       uint64_t wr, uint32_t ra, uint32_t wa, uint32_t *sink) {
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
    uint64_t r = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x, w = r;
    u32x4 acc = {1, 2, 3, 4};
    while (r < rd || w < wr) {
        for (uint32_t j = 0; j < ra && r < rd; ++j, r += stride) {
            const u32x4 v = src[r];
            acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
        }
        for (uint32_t j = 0; j < wa && w < wr; ++j, w += stride) __builtin_nontemporal_store(acc, dst + w);
    }
    if (acc.x == 0x9e3779b9u && acc.y == 0x7f4a7c15u) *sink = acc.z;     // keeps the reads alive
}

// Sixteen weights of one row (as they are stored, zero-point not yet taken off) times sixteen activations.
__device__ __forceinline__ float dot16(const u32x4 w, const float (&xf)[16], float acc) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        acc = fmaf(static_cast<float>(w[j] & 0xffu), xf[4 * j], acc);
        acc = fmaf(static_cast<float>((w[j] >> 8) & 0xffu), xf[4 * j + 1], acc);
        acc = fmaf(static_cast<float>((w[j] >> 16) & 0xffu), xf[4 * j + 2], acc);
        acc = fmaf(static_cast<float>(w[j] >> 24), xf[4 * j + 3], acc);
    }
    return acc;
}

constexpr uint32_t kRowsPerTask = 4;

// One wavefront per task (four matrix rows), 16 weights per lane, row and load; sum(Q x) and sum(x) are
// kept apart, y = s * (sum(Q x) - z * sum(x)), and the lanes' sums are added by shuffles.  Wavefronts
// stride over the tasks of all matrices, so one launch keeps the whole chip reading.
__global__ __launch_bounds__(256) void k_gemv_u8_plain(const bench_gemv_item *__restrict__ items, uint32_t count, uint32_t total_tasks) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t waves = gridDim.x * 4u;
    for (uint32_t task = blockIdx.x * 4u + (threadIdx.x >> 6); task < total_tasks; task += waves) {
        // the matrix this task belongs to: the last one whose first task is not behind it
        uint32_t lo = 0, hi = count;
        while (hi - lo > 1u) {
            const uint32_t mid = (lo + hi) >> 1;
            if (items[mid].first_task <= task) lo = mid; else hi = mid;
        }
        const bench_gemv_item it = items[lo];
        const uint32_t r0 = kRowsPerTask * (task - it.first_task);
        const uint8_t *row[kRowsPerTask];
#pragma unroll
        for (uint32_t r = 0; r < kRowsPerTask; ++r)         // rows behind the last one read it again; nothing of them is stored
            row[r] = it.q + static_cast<uint64_t>(r0 + r < it.rows ? r0 + r : it.rows - 1u) * it.cols;
        const uint16_t *x = static_cast<const uint16_t *>(it.x);
        float acc[kRowsPerTask] = {0.0f, 0.0f, 0.0f, 0.0f}, xsum = 0.0f;
#pragma unroll 2
        for (uint32_t c = lane * 16u; c < it.cols; c += 1024u) {
            u32x4 w[kRowsPerTask];
#pragma unroll
            for (uint32_t r = 0; r < kRowsPerTask; ++r) w[r] = __builtin_nontemporal_load((global_u4_ptr)(row[r] + c));
            const u32x4 xa = *(global_u4_ptr)(x + c), xb = *(global_u4_ptr)(x + c + 8u);
            float xf[16];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                xf[2 * j] = __uint_as_float(xa[j] << 16);
                xf[2 * j + 1] = __uint_as_float(xa[j] & 0xffff0000u);
                xf[8 + 2 * j] = __uint_as_float(xb[j] << 16);
                xf[8 + 2 * j + 1] = __uint_as_float(xb[j] & 0xffff0000u);
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) xsum += xf[j];
#pragma unroll
            for (uint32_t r = 0; r < kRowsPerTask; ++r) acc[r] = dot16(w[r], xf, acc[r]);
        }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            xsum += __shfl_xor(xsum, m, 64);
#pragma unroll
            for (uint32_t r = 0; r < kRowsPerTask; ++r) acc[r] += __shfl_xor(acc[r], m, 64);
        }
        if (lane == 0) {
#pragma unroll
            for (uint32_t r = 0; r < kRowsPerTask; ++r)
                if (r0 + r < it.rows) it.y[r0 + r] = (acc[r] - it.zero_point * xsum) * it.scale;
        }
    }
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

uint32_t bench_gemv_tasks(uint32_t rows) { return (rows + kRowsPerTask - 1u) / kRowsPerTask; }

int bench_gemv_u8_plain(const bench_gemv_item *items, uint32_t count, uint32_t total_tasks, void *hip_stream) {
    if (!items || count == 0 || total_tasks == 0) return 1;
    // the shapes and pointers inside `items` are the caller's to get right: they live on the device
    const unsigned grid = std::min<unsigned>((total_tasks + 3u) / 4u, 256u * 8u);
    hipLaunchKernelGGL(k_gemv_u8_plain, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(hip_stream), items, count, total_tasks);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

int bench_stream_probe(const void *src, uint64_t read_bytes, void *dst, uint64_t write_bytes, void *scratch4, void *hip_stream) {
    if (!src || !dst || !scratch4) return 1;
    if (!aligned16(src) || !aligned16(dst) || (read_bytes & 15u) || (write_bytes & 15u) || !read_bytes || !write_bytes) return 1;
    const uint64_t rd = read_bytes / 16, wr = write_bytes / 16, mx = std::max(rd, wr);
    const uint32_t ra = static_cast<uint32_t>(std::max<uint64_t>(1, (8 * rd + mx / 2) / mx));
    const uint32_t wa = static_cast<uint32_t>(std::max<uint64_t>(1, (8 * wr + mx / 2) / mx));
    // many small workgroups: the launch shape that streams fastest on this chip among those tried
    hipLaunchKernelGGL(k_stream_probe, dim3(65536), dim3(1024), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const u32x4 *>(src), rd, static_cast<u32x4 *>(dst), wr, ra, wa, static_cast<uint32_t *>(scratch4));
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

}  // extern "C"
