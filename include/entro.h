/*
 * libentro -- entropy-coded LLM weights decoded on MI355X (gfx950).
 *
 * C ABI of the data-parallel hot path of EntroLLM (arxiv 2505.02380):
 *   offline, host:  quantize a tensor to 8 or 4 bits with one (s, z) pair
 *                   (Proposed Method, "Mixed Quantization Scheme", Eq. 1,
 *                   Fig. 2), build a Huffman code over the 256 / 16 symbols
 *                   ("Huffman weight encoding"), encode the symbols into
 *                   independently decodable segments ("Segmentation for
 *                   parallel Huffman decoding", Fig. 3);
 *   on the GPU:     decode all segments in parallel back to integers, or
 *                   straight to dequantised fp32 / bf16 weights, or straight
 *                   into a batch-1 matrix-vector product of the
 *                   bandwidth-bound token-generation phase ("Latency Reduction
 *                   from Huffman Coding").
 *
 * Conventions
 *   - Plain pointers and sizes only.  "host" pointers are ordinary memory,
 *     "device" pointers are HIP device memory of the current device.
 *   - The caller owns every buffer.  The library allocates no device memory
 *     and keeps no state between calls.
 *   - Device entry points enqueue their work on `hip_stream` (a hipStream_t
 *     passed as void*, NULL = the default stream) and return without waiting
 *     for it.  Two exceptions wait for the stream ONCE, before their kernel is
 *     enqueued, because they upload a table from memory that dies with the
 *     call: entro_plan_init, and the three *_batch forms, which call it.  The
 *     form for callers that must not block is entro_plan_init_staged (the
 *     table goes through pinned memory of the caller's) followed by
 *     entro_plan_run.
 *   - Every failure is a return code; nothing is thrown, nothing aborts.  All
 *     argument checks happen on the host before any launch.  A corrupt stream
 *     can decode to wrong symbols but is never read outside
 *     [stream, stream + stream_bytes) nor written outside the output tensor.
 *   - Device pointers (stream, offsets, x, out, workspace) must be 16-byte
 *     aligned.
 *
 * Stream format (the paper fixes none; this is the library's own)
 *   - One stream, one codebook, one offset table per tensor.
 *   - A segment ("chunk") is `chunk_symbols` consecutive symbols of the
 *     flattened row-major tensor; the last one may be shorter.  Segments are
 *     bit-packed back to back without alignment.
 *   - Bit k of a stream is (stream[k >> 3] >> (k & 7)) & 1.  A code of length
 *     L is written first code bit first, i.e. its most significant bit goes
 *     to the lowest stream position.
 *   - offsets[k], k = 0..n_chunks, is the stream bit at which segment k
 *     starts; offsets[n_chunks] is the total bit count.
 *   - After the last code the stream is zero-padded to a whole byte, then to a
 *     multiple of 16 bytes, then by 16 more bytes; stream_bytes includes all
 *     padding.
 *   - Codes are canonical: present symbols ordered by (length, symbol value)
 *     receive increasing code values, first code 0, next = (prev + 1) shifted
 *     left by the increase in length.
 */
#ifndef ENTRO_H
#define ENTRO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ENTRO_MAX_CODE_LEN 32
#define ENTRO_MAX_SYMBOLS 256
#define ENTRO_MAX_SUB_PER_CHUNK 16   /* entry points per segment (entro_sub_index) */

typedef enum {
    ENTRO_OK = 0,
    ENTRO_ERR_NULL = 1,          /* a required pointer is NULL */
    ENTRO_ERR_BITS = 2,          /* bits is neither 4 nor 8 */
    ENTRO_ERR_SCHEME = 3,        /* unknown quantisation scheme / output type not valid for the call */
    ENTRO_ERR_SIZE = 4,          /* n == 0, chunk_symbols == 0, rows*cols != n, odd chunk for packed 4-bit, ... */
    ENTRO_ERR_NONFINITE = 5,     /* NaN or Inf in the weights */
    ENTRO_ERR_RANGE = 6,         /* negative weight under the unsigned scheme; constant tensor */
    ENTRO_ERR_SYMBOL = 7,        /* symbol >= 2^bits, or symbol without a code */
    ENTRO_ERR_CODE_TOO_LONG = 8, /* a code would exceed ENTRO_MAX_CODE_LEN bits */
    ENTRO_ERR_CAPACITY = 9,      /* an output buffer or workspace is too small */
    ENTRO_ERR_CORRUPT = 10,      /* inconsistent codebook or offset table */
    ENTRO_ERR_ALIGN = 11,        /* a device pointer is not 16-byte aligned */
    ENTRO_ERR_DEVICE = 12        /* a HIP call failed; see entro_last_device_error() */
} entro_status;

typedef enum { ENTRO_UNSIGNED = 0, ENTRO_ASYMMETRIC = 1 } entro_scheme;
typedef enum { ENTRO_U8 = 0, ENTRO_U4_PACKED = 1, ENTRO_F32 = 2, ENTRO_BF16 = 3 } entro_dtype;
typedef enum { ENTRO_OP_DECODE = 0, ENTRO_OP_DEQUANT = 1, ENTRO_OP_GEMV = 2 } entro_op;

/* One scale and zero-point per tensor (Eq. 1, Fig. 2).  w ~ (q - zero_point) * scale. */
typedef struct {
    float scale;
    int32_t zero_point;   /* 0 for the unsigned scheme; may lie outside [0, 2^bits) */
    int32_t bits;         /* 4 or 8 */
    int32_t scheme;       /* entro_scheme */
} entro_qparams;

/* Canonical Huffman code over 2^bits symbols.  len[s] == 0: symbol s has no code. */
typedef struct {
    int32_t bits;                        /* 4 or 8 */
    int32_t n_used;                      /* symbols with a code */
    int32_t max_len;                     /* longest code, <= ENTRO_MAX_CODE_LEN */
    int32_t reserved;
    uint8_t len[ENTRO_MAX_SYMBOLS];
    uint32_t code[ENTRO_MAX_SYMBOLS];    /* code value, read as a len-bit integer, MSB = first bit */
} entro_codebook;

/* One encoded tensor as the device entry points see it. */
typedef struct {
    const void *stream;          /* device: encoded bytes, padded as described above */
    uint64_t stream_bytes;       /* < 2^32 */
    const uint64_t *offsets;     /* device: n_chunks + 1 bit offsets */
    uint64_t n;                  /* symbols (= rows * cols for the GEMV) */
    uint32_t chunk_symbols;      /* symbols per segment; even when the output is ENTRO_U4_PACKED */
    uint32_t rows, cols;         /* GEMV only: W is [rows][cols] row-major */
    uint32_t sub_symbols;        /* 0, or the spacing of the entry points in sub_bits (see entro_sub_index) */
    const entro_codebook *cb;    /* host */
    entro_qparams qp;            /* dequant and GEMV: scale and zero_point; bits must equal cb->bits */
    const void *x;               /* GEMV only, device: bf16[cols] */
    void *out;                   /* device: u8[n] | u8[(n+1)/2] | f32[n] | bf16[n]; GEMV: f32[rows] | bf16[rows] */
    const uint16_t *sub_bits;    /* device, 4-byte aligned: ceil(n / sub_symbols) piece lengths; NULL if sub_symbols == 0 */
} entro_tensor;

/* A prepared launch over `count` tensors.  Filled by entro_plan_init; plain data, caller-owned.
 * The workspace it points to (device memory) must stay untouched while the plan is in use. */
typedef struct {
    void *workspace;
    uint64_t workspace_bytes;
    uint32_t op;          /* entro_op */
    uint32_t out;         /* entro_dtype */
    uint32_t count;       /* tensors */
    uint32_t n_items;     /* work items in the launch */
    uint32_t n_fix;       /* GEMV: rows that need the second-stage sum */
    uint32_t item_units;  /* units (the segments or pieces of one tensor that the 64 lanes of a wavefront take) per work item */
    uint32_t pair_tables; /* 1: every tensor holds 4-bit symbols, the kernels decode two per table lookup */
    uint32_t gemv_multirow; /* 1: a tensor's segments are longer than its matrix rows (information only) */
    uint32_t wide_tables; /* 1: GEMV over 8-bit tensors with zero-points in [-1, 256]: table entries hold the centred value */
    uint32_t reserved;
    uint64_t off_tensors, off_items, off_partials, off_fix;   /* byte offsets inside the workspace */
} entro_plan;

/* ------------------------------------------------------------------ host side
 * Synchronous, no allocation visible to the caller, safe to call from several
 * threads on different buffers. */

/* Eq. 1 with Q = 2^bits - 1, binary32 arithmetic, round-half-even:
 *   unsigned:   s = max/Q, z = 0;   asymmetric: s = (max - min)/Q, z = rint(-min/s);
 *   q = clamp(rint(w/s) + z, 0, Q), one symbol per output byte.
 * w: host, n floats.  q: host, n bytes.  qp: receives scale, zero_point, bits, scheme. */
entro_status entro_quantize(const float *w, uint64_t n, int bits, entro_scheme scheme,
                            uint8_t *q, entro_qparams *qp);

/* "Huffman weight encoding": count the symbols, build an optimal prefix code
 * (length = depth in the merge tree), assign canonical code values.
 * q: host, n symbols one per byte, each < 2^bits.  A lone symbol gets a 1-bit code. */
entro_status entro_build_codebook(const uint8_t *q, uint64_t n, int bits, entro_codebook *cb);

/* The same ("Huffman weight encoding"), from a ready histogram of 2^bits counts. */
entro_status entro_codebook_from_counts(const uint64_t *counts, int bits, entro_codebook *cb);

/* Length-limited variants of "Huffman weight encoding" (an extension towards the
 * hardware-aware coding the paper's conclusions name as future work): the cheapest prefix code none of
 * whose codes is longer than max_len bits (package-merge), so that a decoder's
 * single-level table of max_len index bits holds every code and the slow path for
 * long codes never runs.  1 <= max_len <= ENTRO_MAX_CODE_LEN; the alphabet must
 * fit (ENTRO_ERR_CODE_TOO_LONG if more than 2^max_len symbols occur).  With
 * max_len at or above the longest unrestricted Huffman code the cost equals the
 * unrestricted optimum.  The device side needs no change: a codebook is a
 * codebook. */
entro_status entro_codebook_from_counts_limited(const uint64_t *counts, int bits, int max_len, entro_codebook *cb);
entro_status entro_build_codebook_limited(const uint8_t *q, uint64_t n, int bits, int max_len, entro_codebook *cb);

/* Canonical code values for given lengths (0 = absent): the codebook of "Huffman
 * weight encoding" as it is stored with a model, the lengths alone.  Rejects lengths
 * above ENTRO_MAX_CODE_LEN and length sets whose Kraft sum exceeds 1. */
entro_status entro_codebook_from_lengths(const uint8_t *len, int bits, entro_codebook *cb);

/* Number of segments of "Segmentation for parallel Huffman decoding" (Fig. 3):
 * ceil(n / chunk_symbols); 0 if chunk_symbols == 0. */
uint64_t entro_num_chunks(uint64_t n, uint32_t chunk_symbols);

/* Upper bound in bytes (padding included) of the stream entro_encode writes ("Huffman
 * weight encoding": no symbol takes more than the longest code); 0 on bad arguments. */
uint64_t entro_encode_bound(uint64_t n, const entro_codebook *cb);

/* "Huffman weight encoding" into the independently decodable segments of
 * "Segmentation for parallel Huffman decoding" (Fig. 3): encode q (host, n symbols)
 * into stream (host, stream_cap bytes) and fill
 * offsets (host, entro_num_chunks + 1 entries).  *stream_bytes receives the
 * padded size.  ENTRO_ERR_SYMBOL if a symbol has no code, ENTRO_ERR_CAPACITY
 * if stream_cap is too small (nothing useful is written then). */
entro_status entro_encode(const uint8_t *q, uint64_t n, const entro_codebook *cb,
                          uint32_t chunk_symbols, uint8_t *stream, uint64_t stream_cap,
                          uint64_t *stream_bytes, uint64_t *offsets);

/* Entry points inside the segments (an extension of "Segmentation for parallel Huffman
 * decoding", Fig. 3: the more places of the stream have known positions, the more lanes
 * can decode it at once; a segment of 4096 symbols is one lane's serial work otherwise,
 * which bounds the latency of a small launch from below).  chunk_symbols must be
 * sub_symbols times a power of two of at most ENTRO_MAX_SUB_PER_CHUNK.
 * sub_bits[j], j = 0 .. ceil(n / sub_symbols) - 1 (host), receives the number of stream
 * bits that piece j (symbols j * sub_symbols ...) occupies: piece j starts at its
 * segment's offset plus the entries of the pieces before it in the same segment.  The
 * stream and the offset table are those of entro_encode, unchanged.  With sub_bits and
 * sub_symbols in an entro_tensor the device calls give a lane a piece instead of a
 * segment; results are identical.  ENTRO_ERR_CODE_TOO_LONG if a piece exceeds 65535 bits
 * (cannot happen for sub_symbols <= 2047), ENTRO_ERR_SYMBOL for a symbol without a code. */
entro_status entro_sub_index(const uint8_t *q, uint64_t n, const entro_codebook *cb, uint32_t chunk_symbols,
                             uint32_t sub_symbols, uint16_t *sub_bits);

/* Consistency check of a host copy of the offset table of Fig. 3's segments against a stream size:
 * offsets[0] == 0, non-decreasing, each segment no longer than
 * chunk_symbols * max_len bits and no shorter than its symbol count times the
 * shortest code, last offset within stream_bytes minus the 16 trailing pad
 * bytes.  ENTRO_ERR_CORRUPT otherwise. */
entro_status entro_check_offsets(const uint64_t *offsets, uint64_t n, uint32_t chunk_symbols,
                                 uint64_t stream_bytes, const entro_codebook *cb);

/* Reporting helpers for the quantities the paper tabulates (Table 2 "bits
 * saved" = bits - mean code length; theoretical token-generation speed-up =
 * bits / mean code length, as in "Latency Reduction from Huffman Coding"). */
double entro_bits_saved(int bits, double mean_code_len);
double entro_theoretical_speedup(int bits, double mean_code_len);

/* Text for a status code (error reporting; no passage of the paper defines it). */
const char *entro_status_string(entro_status s);

/* ---------------------------------------------------------------- device side
 * One tensor per call, descriptor passed in kernel arguments (no workspace
 * needed except for the GEMV's second-stage sum). */

/* Segment-parallel decode back to integers ("Segmentation for parallel Huffman
 * decoding", Fig. 3, lower half: every segment by a worker of its own).  out_type: ENTRO_U8 (one symbol
 * per byte) or ENTRO_U4_PACKED (4-bit codebooks only; symbol 2i in the low
 * nibble of byte i, 2i+1 in the high nibble, last high nibble zero if n is odd). */
entro_status entro_decode(const entro_tensor *t, entro_dtype out_type, void *hip_stream);

/* Decode (Fig. 3) fused with the inverse of Eq. 1's grid map, w = (q - z) * s (integer difference,
 * exact conversion, one binary32 multiply).  out_type: ENTRO_F32 (bit-exact)
 * or ENTRO_BF16 (the binary32 value rounded to nearest even). */
entro_status entro_decode_dequant(const entro_tensor *t, entro_dtype out_type, void *hip_stream);

/* Bytes of device workspace entro_decode_gemv ("Latency Reduction from Huffman Coding")
 * needs for this tensor (may be 0). */
uint64_t entro_gemv_workspace_bytes(const entro_tensor *t);

/* y = W x for batch-1 token generation without materialising W ("Latency Reduction from
 * Huffman Coding", Table 3: the phase is bound by the weight bytes read, and the coded
 * stream is fewer bytes):
 * y[r] = s * sum_j (q[r][j] - z) * x[j], fp32 accumulation, x bf16, W row-major.
 * y_type: ENTRO_F32 or ENTRO_BF16.  Rows that straddle segments are summed in
 * segment order by a second small kernel (deterministic). */
entro_status entro_decode_gemv(const entro_tensor *t, entro_dtype y_type, void *workspace,
                               uint64_t workspace_bytes, void *hip_stream);

/* entro_decode_gemv for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and
 * results as entro_decode_gemv; the partial sums of rows that straddle segments live in an array
 * inside the library's device image (8 * ENTRO_STATIC_GEMV_MAX_SEGMENTS bytes per GPU, held until the
 * process ends) instead of a workspace.  The call allocates nothing and only enqueues kernels.
 * ENTRO_ERR_CAPACITY if the tensor needs partial sums and has more than
 * ENTRO_STATIC_GEMV_MAX_SEGMENTS segments.  All calls on one GPU share the array: calls that may
 * overlap there (different streams, or graphs replayed concurrently) race; order them. */
#define ENTRO_STATIC_GEMV_MAX_SEGMENTS 65536
entro_status entro_decode_gemv_static(const entro_tensor *t, entro_dtype y_type, void *hip_stream);

/* Batched forms: ONE launch over `count` tensors (a single tensor has too few of
 * Fig. 3's segments to fill 256 compute units).  The descriptor table, the work list,
 * the tensors' lookup tables (about 68 KB per tensor) and the GEMV partial sums live
 * in `workspace` (device). */
uint64_t entro_workspace_bytes(const entro_tensor *ts, uint32_t count, entro_op op);

/* Prepare a batched launch of Fig. 3's segment-parallel decode (or of the fused forms above):
 * validate, build the table on the host, copy it into the workspace and enqueue a small kernel
 * that builds every tensor's lookup tables there (so that the launches need not).  BLOCKS until
 * the copy, and with it everything enqueued on hip_stream before, has completed (the
 * table is staged in memory that dies with the call); entro_plan_init_staged does not.
 * The tensors' device buffers are referenced, not copied.
 * The work list is cut for the current device (its number of compute units
 * decides how many units a work item holds and, for tensors with entry points
 * inside their segments, how many pieces a lane takes: as coarse as still gives
 * the device's lanes work): run the plan on the device it was prepared on.  The
 * launch is one workgroup per compute unit at most; inside a workgroup the
 * wavefronts draw their segments from a counter, so which wavefront decodes which
 * segment differs from run to run, the result does not.  (A GEMV's sums are taken
 * in an order that depends on how rows are cut into lanes, i.e. on the launch, never
 * on the run.) */
entro_status entro_plan_init(entro_plan *plan, const entro_tensor *ts, uint32_t count, entro_op op,
                             entro_dtype out_type, void *workspace, uint64_t workspace_bytes,
                             void *hip_stream);

/* The same (Fig. 3's decode, prepared for many tensors) without waiting: the table is built
 * in `staging` (host memory of the caller's, at least entro_plan_staging_bytes, pinned -- hipHostMalloc -- if the copy is to be
 * asynchronous) and copied from there on hip_stream.  The caller keeps `staging` alive
 * and unchanged until that copy has completed (a stream or event wait of its own).
 * ENTRO_ERR_CAPACITY if staging_bytes is too small. */
uint64_t entro_plan_staging_bytes(const entro_tensor *ts, uint32_t count, entro_op op);
entro_status entro_plan_init_staged(entro_plan *plan, const entro_tensor *ts, uint32_t count, entro_op op,
                                    entro_dtype out_type, void *workspace, uint64_t workspace_bytes, void *staging,
                                    uint64_t staging_bytes, void *hip_stream);

/* Enqueue the prepared launch (Fig. 3: all segments of all its tensors at once); no host-side
 * table work, no copies, no waiting. */
entro_status entro_plan_run(const entro_plan *plan, void *hip_stream);

/* Fig. 3's decode, the inverse of Eq. 1 and the product of "Latency Reduction from Huffman
 * Coding" over many tensors: entro_plan_init followed by entro_plan_run (so these wait for
 * the stream once, before their kernel is enqueued; they return without waiting for the kernel). */
entro_status entro_decode_batch(const entro_tensor *ts, uint32_t count, entro_dtype out_type,
                                void *workspace, uint64_t workspace_bytes, void *hip_stream);
entro_status entro_decode_dequant_batch(const entro_tensor *ts, uint32_t count, entro_dtype out_type,
                                        void *workspace, uint64_t workspace_bytes, void *hip_stream);
entro_status entro_decode_gemv_batch(const entro_tensor *ts, uint32_t count, entro_dtype y_type,
                                     void *workspace, uint64_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------ device side: compression
 * The steps before the decode path for weights that already sit in device
 * memory: the three that touch every weight (range, Eq. 1's grid map with the
 * symbol counts of "Huffman weight encoding", the segment-parallel writing of
 * the stream, Fig. 3) run as kernels; the two that touch 2^bits numbers
 * (entro_qparams_from_range, entro_codebook_from_counts) are host calls between
 * them, on values the caller copies back.  Results are those of entro_quantize
 * and entro_encode, bit for bit.  All calls only enqueue work on hip_stream. */

/* The extrema Eq. 1's scale and zero-point are computed from:
 * range16 (device, 16 bytes, 16-byte aligned) receives { float min, float max,
 * uint32 nonfinite (1 if a NaN or Inf occurs, NaNs do not enter min / max),
 * uint32 0 } of w (device, n floats, 16-byte aligned). */
entro_status entro_range_device(const float *w, uint64_t n, void *range16, void *hip_stream);

/* Host: Eq. 1's scale and zero-point from a tensor's range (the formulas given
 * with entro_quantize).  ENTRO_ERR_NONFINITE if `nonfinite` is set or a bound is
 * not finite, ENTRO_ERR_RANGE for a negative minimum under the unsigned scheme
 * or an empty range. */
entro_status entro_qparams_from_range(float min, float max, uint32_t nonfinite, int bits, entro_scheme scheme,
                                      entro_qparams *qp);

/* Host: which of the two grids of Fig. 2 a tensor with this range gets under the
 * mixed scheme ("either unsigned or asymmetric per layer, based on its weight
 * distribution"; the paper states no rule): the unsigned grid, which has no
 * zero-point, exactly when it can represent the tensor, i.e. when no weight is
 * negative (norm gains, for instance); the asymmetric grid otherwise. */
entro_scheme entro_scheme_for_range(float min, float max);

/* Eq. 1's grid map, q[i] = clamp(rint(w[i] / s) + z, 0, 2^bits - 1), one symbol per byte, and the
 * histogram of the symbols ("Huffman weight encoding" starts from it).  w: device, n floats; q: device, n bytes; counts:
 * device, 256 entries, overwritten (entries at and above 2^bits end up 0); all
 * 16-byte aligned.  qp: host.  ENTRO_ERR_RANGE if |zero_point| > 2^24 (the
 * decoders take no such tensor either).  A NaN weight, which entro_range_device
 * reports, quantises to clamp(z). */
entro_status entro_quantize_device(const float *w, uint64_t n, const entro_qparams *qp, uint8_t *q, uint64_t *counts,
                                   void *hip_stream);

/* Host: exact size in bytes (padding included) of the stream that symbols with
 * this histogram make under this codebook ("Huffman weight encoding": sum of count times length); 0 if a counted symbol has no code. */
uint64_t entro_encoded_bytes(const uint64_t *counts, const entro_codebook *cb);

/* "Huffman weight encoding" into Fig. 3's segments on the device: encode q (device, n symbols
 * one per byte) into stream (device, stream_cap
 * bytes, a multiple of 16) and fill offsets (device, entro_num_chunks + 1
 * entries), in the format described at the top; the padded size is
 * entro_encoded_bytes, or follows from offsets[n_chunks].  cb: host.
 * chunk_symbols <= 2^20.  What can only be seen on the device is reported in
 * *status (device, 4 bytes, written by the call): 0 if the stream was written,
 * otherwise nothing was written to `stream`; pass the value, once copied back,
 * to entro_encode_device_status. */
entro_status entro_encode_device(const uint8_t *q, uint64_t n, const entro_codebook *cb, uint32_t chunk_symbols, void *stream,
                                 uint64_t stream_cap, uint64_t *offsets, uint32_t *status, void *hip_stream);

/* Host: the meaning of a status word of entro_encode_device (Fig. 3's encode side): ENTRO_OK,
 * ENTRO_ERR_SYMBOL (a symbol without a code), ENTRO_ERR_CAPACITY (stream_cap too
 * small), ENTRO_ERR_SIZE (the stream would reach 4 GiB). */
entro_status entro_encode_device_status(uint32_t status_word);

/* Text of the last HIP error seen by the calling thread ("" if none) (error reporting; no
 * passage of the paper defines it). */
const char *entro_last_device_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ENTRO_H */
