/*
 * ogq.h -- C ABI of libogq: per-bucket optimal gradient quantization on one MI355X (gfx950).
 *
 * Method: "Optimal Gradient Quantization Condition for Communication-Efficient Distributed
 * Training" (Xu, Huo, Huang; arXiv 2002.11082).  A gradient of n fp32 values is cut into
 * buckets of `bucket_size` consecutive elements (bucket-based quantization, Section 5; the last
 * bucket is shorter when bucket_size does not divide n) and every bucket is quantized on its
 * own: the levels are solved from the bucket's values with the paper's optimal condition, every
 * element is encoded to a level index, and the indices are bit-packed.  The receiving side
 * decodes several workers' packed streams with their own level tables and averages them
 * (server step of Algorithm 2).
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers (HIP global memory on the current device) and
 *     must be 16-byte aligned.  All other pointers are HOST pointers.  The caller allocates and
 *     owns every buffer; the library allocates nothing, never frees, and keeps no state apart
 *     from the thread-local code read by ogq_last_hip_error().
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and the call returns without synchronising.
 *   - Return value: OGQ_OK (0) or a negative ogq_status_t.  On an argument error (every code but
 *     OGQ_ERR_LAUNCH) nothing was enqueued and no output byte was written.  OGQ_ERR_LAUNCH means the HIP
 *     runtime refused a kernel launch of this call (its own return code, not the thread's sticky last
 *     error); nothing is enqueued after the refused launch, but a call that takes two launches
 *     (OGQ_BINGRAD_B / OGQ_SCALED_SIGN with a bucket size dividing 2048, without clipping, when n is not
 *     a multiple of 2048) may already have enqueued its first one.  The library never throws and never aborts.
 *   - Input values must be finite.  Non-finite input gives unspecified levels and codes but no
 *     out-of-bounds access.
 *   - n == 0 is a successful no-op.
 */
#ifndef OGQ_H
#define OGQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OGQ_OK = 0,
    OGQ_ERR_NULL_POINTER = -1,  /* a required pointer is NULL */
    OGQ_ERR_BUCKET_SIZE = -2,   /* bucket_size is 0, not a multiple of 64, or above 32768 */
    OGQ_ERR_BITS = -3,          /* bits outside the range the scheme supports */
    OGQ_ERR_SCHEME = -4,        /* unknown scheme */
    OGQ_ERR_NUM_WORKERS = -5,   /* num_workers is 0 or above OGQ_MAX_WORKERS */
    OGQ_ERR_ALIGNMENT = -6,     /* a device pointer is not 16-byte aligned */
    OGQ_ERR_INDEX_OFFSET = -7,  /* index_offset is not a multiple of 64 */
    OGQ_ERR_LAUNCH = -8,        /* the HIP runtime refused the launch (ogq_last_hip_error()) */
    OGQ_ERR_SIZE = -9,          /* n is too large for the 32-bit bucket grid (n/bucket_size >= 2^31) */
    OGQ_ERR_CLIP = -10,         /* clip_factor is negative or not finite */
    OGQ_ERR_RESERVED = -11      /* the reserved field of the parameters is not 0 */
} ogq_status_t;

typedef enum {
    /* BinGrad-b: two levels, deterministic, biased (Section 3.2, the fully biased binary
     * scheme and its optimal condition).  bits must be 1. */
    OGQ_BINGRAD_B = 0,
    /* ORQ: s = 2^bits levels placed by the optimal condition of Theorem 1 (greedy recursion of
     * Algorithm 1 followed by re-solve sweeps), unbiased random rounding (Section 3.1).
     * bits in 1..3. */
    OGQ_ORQ = 1,
    /* BinGrad-pb: two levels -b_1, +b_1, partially biased (Section 3.2): values outside [-b_1, b_1) go to
     * the nearer level, values inside are rounded at random as in ORQ (same draws).  b_1 minimises
     * |b * #{v > 0} - sum_{v >= b} v| (the scheme's optimal condition for discrete values) over the
     * bucket's positive values, the smaller value on a tie; 0 if the bucket has no positive value.
     * bits must be 1; level_iters is ignored. */
    OGQ_BINGRAD_PB = 2,
    /* ORQ with the paper's level counts s = 2^K + 1 (Algorithm 1's initialisation: 3, 5 or 9 levels);
     * bits = K + 1 in 2..4 is the width of a level index.  With level_iters = 0 the levels are those of
     * Algorithm 1 as printed.  Encoding and packing as for OGQ_ORQ. */
    OGQ_ORQ_PAPER = 3,
    /* The level rules the paper compares against (Section 5, list of methods), on the same kernels, so that
     * their quantization error can be set beside ORQ's and BinGrad's on equal inputs.  level_iters is ignored.
     * Scaled SignSGD (first equation of Section 3.2), per bucket: two levels -m, +m, m = mean |v| (fp64 sum,
     * rounded to fp32); index = (v >= 0), deterministic.  bits must be 1. */
    OGQ_SCALED_SIGN = 4,
    /* QSGD-s / TernGrad (Section 3.1): s = 2^(bits-1) + 1 levels evenly spaced from -M to +M, M the largest
     * magnitude of the bucket: level k = M * (2k - (s-1)) / (s-1) (fp64, rounded to fp32); bits in 2..4
     * (bits = 2 is TernGrad's {-M, 0, +M}).  Random rounding, encoding and packing as for OGQ_ORQ. */
    OGQ_EVEN = 5,
    /* Linear-s (Section 5): s = 2^(bits-1) + 1 levels dividing the bucket's cumulative distribution linearly:
     * level k is the element of 0-based rank floor(k * (len-1) / (s-1)) of the sorted bucket (level 0 the
     * minimum, level s-1 the maximum); bits in 2..4.  Random rounding, encoding and packing as for OGQ_ORQ. */
    OGQ_LINEAR = 6
} ogq_scheme_t;

#define OGQ_MAX_WORKERS 64u
#define OGQ_MAX_BUCKET_SIZE 32768u

typedef struct {
    uint32_t bucket_size;  /* elements per bucket: a multiple of 64 in [64, 32768] (the paper's sweep: 128 .. 32768) */
    uint32_t bits;         /* width of a level index; levels per bucket: see ogq_levels_per_bucket */
    uint32_t scheme;       /* ogq_scheme_t */
    /* BINGRAD_B: number of threshold updates b0 <- (b_{-1} + b_1)/2 after the start b0 = bucket
     * mean (0 = the paper's shortcut).  ORQ: number of sweeps that re-solve every interior level
     * between its current neighbours after the greedy placement. */
    uint32_t level_iters;
    uint64_t seed;         /* Philox key (schemes with random rounding) */
    /* Global index of d_grad[0] (schemes with random rounding; a multiple of 64): element i draws the random number
     * that belongs to global index index_offset + i, so a bucket-aligned shard reproduces the
     * codes of the full vector. */
    uint64_t index_offset;
    /* Gradient clipping before quantization (Section 5, taken over from TernGrad): every bucket value
     * becomes sign(v) * min(|v|, clip_factor * sigma), sigma^2 = population variance of the bucket about
     * its mean (fp64), threshold rounded to fp32; levels and codes are those of the clipped bucket.
     * 0 = off.  The paper uses 2.5 (and 1.7). */
    float clip_factor;
    uint32_t reserved;     /* must be 0 */
} ogq_params_t;

/* Sizes of the outputs of ogq_quantize for a gradient of n elements (pure host arithmetic).
 *   levels_per_bucket = 2 (BINGRAD_B, BINGRAD_PB, SCALED_SIGN), 2^bits (ORQ), 2^(bits-1) + 1 (ORQ_PAPER, EVEN, LINEAR)
 *   num_buckets       = ceil(n / bucket_size)
 *   levels_count      = num_buckets * levels_per_bucket    fp32 values
 *   codes_bytes       = ceil(n / 64) * bits * 8            bytes
 * They return 0 when params is NULL, bucket_size is 0 or scheme / bits do not go together. */
size_t ogq_levels_per_bucket(const ogq_params_t* params);
size_t ogq_num_buckets(size_t n, const ogq_params_t* params);
size_t ogq_levels_count(size_t n, const ogq_params_t* params);
size_t ogq_codes_bytes(size_t n, const ogq_params_t* params);

/* Quantize one worker's gradient: levels + packed codes (what Algorithm 2 has a worker compute,
 * quantize and encode before sending).
 *
 *   d_grad    in   n fp32, device, read once.
 *   d_levels  out  levels_count fp32, device; bucket b owns entries
 *                  [b * levels_per_bucket, (b+1) * levels_per_bucket), non-decreasing.
 *                  BINGRAD_B: {b_{-1}, b_1} = means of the elements below / not below the
 *                  threshold b0 (b0 = fp32 bucket mean, then level_iters midpoint updates);
 *                  a constant bucket gives two equal levels.
 *                  ORQ, ORQ_PAPER: level 0 = bucket minimum, level s-1 = bucket maximum (Corollary 1),
 *                  interior levels are bucket values solving the discrete optimal condition
 *                  (second remark after Theorem 1) between their neighbours.
 *                  The other schemes: see ogq_scheme_t.
 *   d_codes   out  codes_bytes bytes, device.  Bit-plane layout: element i
 *                  belongs to group i/64, lane i%64; bit `lane` of the little-endian 64-bit
 *                  word (group*bits + p) is bit p of the element's level index.  Pad bits of
 *                  the last group are written as 0.
 *                  BINGRAD_B: index = (v >= b0).  SCALED_SIGN: index = (v >= 0).  Every other scheme
 *                  (random rounding): k = last level not above v (at most
 *                  s-2), index = k + [u * (b_{k+1} - b_k) < v - b_k] in fp32, where u is the top
 *                  24 bits of word (j mod 4) of Philox4x32-10(counter = (lo32(j/4), hi32(j/4),
 *                  0, 0), key = (lo32(seed), hi32(seed))) times 2^-24, j = index_offset + i.
 *
 * d_levels and d_codes must not overlap d_grad. */
int ogq_quantize(const float* d_grad, size_t n, const ogq_params_t* params,
                 float* d_levels, void* d_codes, void* hip_stream);

/* Decode num_workers packed streams and average them (server step of Algorithm 2):
 *   d_out[i] = (1/num_workers) * sum_w d_levels[w][(i / bucket_size) * levels_per_bucket + index_w(i)]
 * accumulated in fp64 and rounded once to fp32.
 *
 *   d_codes   in   HOST array of num_workers DEVICE pointers, each to codes_bytes bytes as
 *                  written by ogq_quantize.
 *   d_levels  in   HOST array of num_workers DEVICE pointers, each to levels_count fp32.
 *   d_out     out  n fp32, device; must not overlap any input.
 * All workers share n and params; their level tables differ.  Only bucket_size, bits and scheme of
 * params are read.  The host arrays are copied during the call and may
 * be reused as soon as it returns. */
int ogq_dequantize_average(const void* const* d_codes, const float* const* d_levels,
                           uint32_t num_workers, size_t n, const ogq_params_t* params,
                           float* d_out, void* hip_stream);

/* Bandwidth probes used by the benchmark to find the practical HBM ceiling of the device and to
 * calibrate hardware traffic counters (not part of the method).
 *   ogq_probe_read: streams the first 4*floor(n/4) fp32 of d_src, folds them into one value per
 *                   wavefront and writes OGQ_PROBE_SINK_FLOATS floats to d_sink (device,
 *                   caller-allocated).
 *   ogq_probe_copy: d_dst[i] = d_src[i] for the first 4*floor(n/4) fp32. */
#define OGQ_PROBE_SINK_FLOATS 8192u
int ogq_probe_read(const float* d_src, size_t n, float* d_sink, void* hip_stream);
int ogq_probe_copy(const float* d_src, float* d_dst, size_t n, void* hip_stream);

/* Text for a status code (static storage, never NULL). */
const char* ogq_strerror(int status);

/* The hipError_t value of the last failed launch on this thread (0 if none). */
int ogq_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* OGQ_H */
