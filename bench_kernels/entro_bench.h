/* Kernels that bench.py times beside the library's own: a memory probe and the plain
 * uint8 GEMV that the entropy-coded one is compared with.  Neither is part of the
 * hot path or of libentro.so; both live in bench_kernels/libentro_bench.so.
 *
 * All pointers are device pointers unless said otherwise; calls enqueue on
 * hip_stream (NULL: the default stream) and return without waiting.  Return value:
 * 0 on success, 1 for a bad argument, 2 if the launch failed. */
#ifndef ENTRO_BENCH_H
#define ENTRO_BENCH_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* One kernel that reads read_bytes from src and writes write_bytes to dst (16-byte
 * aligned, sizes multiples of 16), perfectly coalesced, reads and writes interleaved
 * in the ratio of the two sizes: the rate at which this GPU's memory takes a plain
 * stream with a decode launch's read/write mix.  scratch4: four bytes the kernel may write. */
int bench_stream_probe(const void *src, uint64_t read_bytes, void *dst, uint64_t write_bytes, void *scratch4, void *hip_stream);

/* One matrix of the plain uint8 model (Table 3's "uint8" column): y = s * (Q - z) x with
 * Q stored one byte per weight, row-major. */
typedef struct bench_gemv_item {
    const uint8_t *q;    /* rows * cols bytes, 16-byte aligned */
    const void *x;       /* bf16[cols], 16-byte aligned */
    float *y;            /* float[rows] */
    uint32_t rows, cols; /* cols a multiple of 16 */
    float scale, zero_point;
    uint32_t first_task; /* tasks (four rows each) of the items before this one */
    uint32_t reserved;
} bench_gemv_item;

/* Number of tasks of a matrix with `rows` rows (host). */
uint32_t bench_gemv_tasks(uint32_t rows);

/* All `count` products in one launch.  items: device array, first_task filled in as the
 * running sum of bench_gemv_tasks(rows); total_tasks: that sum over all items. */
int bench_gemv_u8_plain(const bench_gemv_item *items, uint32_t count, uint32_t total_tasks, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
