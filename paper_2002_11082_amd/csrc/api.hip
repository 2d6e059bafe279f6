// libogq: per-bucket optimal gradient quantization for MI355X (gfx950, wave64): the C ABI declared in ogq.h.
//
// Method: "Optimal Gradient Quantization Condition for Communication-Efficient Distributed
// Training" (arXiv 2002.11082).  A bucket stays with one wavefront (several small buckets share one, a large
// bucket takes the wavefronts of one workgroup) from the HBM load to the packed store, so the gradient is read
// exactly once:
//   bingrad.hip            BinGrad-b (Section 3.2) and Scaled SignSGD: fp64 wave reductions for the mean and the
//                          two conditional means; the code bits of 64 consecutive elements are a lane mask.
//   rounding_kernels.h     ORQ (Theorem 1, its discrete remark, Corollary 1, Algorithm 1; random rounding of
//                          Section 3.1), BinGrad-pb and the evenly spaced / Linear-s comparison rules: every
//                          level solve is a range sum plus an exact rank selection over the bucket grouped in
//                          LDS; Philox4x32-10 draws keyed by (seed, global element index).
//   decode.hip             decode-average (server step of Algorithm 2): a bit-matrix transpose across the lanes turns
//                          the packed words into per-element level indices, which address level tables in LDS
//                          (several workers per look-up through tables of pre-summed level combinations).
// This file validates the arguments and picks the launcher (launch.h).
//
// Compile with -ffp-contract=off: the rounding decision of ORQ is specified op by op in fp32.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch.h"
#include "ogq.h"

namespace ogq {

uint32_t levels_per_bucket(uint32_t scheme, uint32_t bits)
{
    if (scheme == OGQ_BINGRAD_B || scheme == OGQ_BINGRAD_PB || scheme == OGQ_SCALED_SIGN) return bits == 1 ? 2u : 0u;
    if (scheme == OGQ_ORQ) return (bits >= 1 && bits <= 3) ? 1u << bits : 0u;
    if (scheme == OGQ_ORQ_PAPER || scheme == OGQ_EVEN || scheme == OGQ_LINEAR)
        return (bits >= 2 && bits <= 4) ? (1u << (bits - 1)) + 1u : 0u;
    return 0u;
}

hipError_t& launch_status()
{
    static thread_local hipError_t status = hipSuccess;
    return status;
}

}  // namespace ogq

namespace {

thread_local int g_last_hip_error = 0;

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_params(const ogq_params_t* p, bool quantize)
{
    if (!p) return OGQ_ERR_NULL_POINTER;
    if (p->bucket_size == 0 || p->bucket_size % 64 != 0 || p->bucket_size > OGQ_MAX_BUCKET_SIZE)
        return OGQ_ERR_BUCKET_SIZE;
    if (p->scheme > OGQ_LINEAR) return OGQ_ERR_SCHEME;
    if (ogq::levels_per_bucket(p->scheme, p->bits) == 0) return OGQ_ERR_BITS;
    if (p->reserved != 0) return OGQ_ERR_RESERVED;
    if (quantize) {
        if (p->index_offset % 64 != 0) return OGQ_ERR_INDEX_OFFSET;
        if (!(p->clip_factor >= 0.0f) || !(p->clip_factor <= 3.0e38f)) return OGQ_ERR_CLIP;
    }
    return OGQ_OK;
}

// Every entry point that launches calls begin_launches() before its first launch and returns finish_launches():
// the status is the one the runtime returned for these launches, not the thread's sticky last error.
void begin_launches() { ogq::launch_status() = hipSuccess; }

int finish_launches()
{
    const hipError_t e = ogq::launch_status();
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return OGQ_ERR_LAUNCH;
    }
    return OGQ_OK;
}

}  // namespace

extern "C" {

size_t ogq_num_buckets(size_t n, const ogq_params_t* p)
{
    if (!p || p->bucket_size == 0) return 0;
    return n / p->bucket_size + (n % p->bucket_size != 0);
}

size_t ogq_levels_per_bucket(const ogq_params_t* p) { return p ? ogq::levels_per_bucket(p->scheme, p->bits) : 0; }

size_t ogq_levels_count(size_t n, const ogq_params_t* p)
{
    if (!p) return 0;
    return ogq_num_buckets(n, p) * ogq::levels_per_bucket(p->scheme, p->bits);
}

size_t ogq_codes_bytes(size_t n, const ogq_params_t* p)
{
    if (!p || p->bucket_size == 0 || ogq::levels_per_bucket(p->scheme, p->bits) == 0) return 0;
    return (n / 64 + (n % 64 != 0)) * p->bits * 8;
}

int ogq_quantize(const float* d_grad, size_t n, const ogq_params_t* params, float* d_levels, void* d_codes,
                 void* hip_stream)
{
    const int rc = check_params(params, true);
    if (rc != OGQ_OK) return rc;
    if (n == 0) return OGQ_OK;
    if (!d_grad || !d_levels || !d_codes) return OGQ_ERR_NULL_POINTER;
    if (!aligned(d_grad, 16) || !aligned(d_levels, 16) || !aligned(d_codes, 16)) return OGQ_ERR_ALIGNMENT;
    const size_t nb64 = ogq_num_buckets(n, params);
    if (nb64 >= (1ull << 31)) return OGQ_ERR_SIZE;
    const uint32_t nb = (uint32_t)nb64;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const uint32_t d = params->bucket_size;
    begin_launches();
    if (params->scheme == OGQ_BINGRAD_B || params->scheme == OGQ_SCALED_SIGN) {
        ogq::launch_two_level(d_grad, n, params, d_levels, d_codes, st);
    } else {
        const uint32_t chunks = (d + 255) / 256;  // 256-element chunks per bucket
        ogq::RoundingLauncher* launch = chunks <= 1    ? ogq::launch_rounding_c1
                                        : chunks <= 2  ? ogq::launch_rounding_c2
                                        : chunks <= 4  ? ogq::launch_rounding_c4
                                        : chunks <= 8  ? ogq::launch_rounding_c8
                                        : chunks <= 16 ? ogq::launch_rounding_c16
                                        : chunks <= 32 ? ogq::launch_rounding_w2
                                        : chunks <= 64 ? ogq::launch_rounding_w4
                                                       : ogq::launch_rounding_w8;
        launch(d_grad, n, params, nb, d_levels, d_codes, st);
    }
    return finish_launches();
}

int ogq_dequantize_average(const void* const* d_codes, const float* const* d_levels, uint32_t num_workers, size_t n,
                           const ogq_params_t* params, float* d_out, void* hip_stream)
{
    const int rc = check_params(params, false);
    if (rc != OGQ_OK) return rc;
    if (num_workers == 0 || num_workers > OGQ_MAX_WORKERS) return OGQ_ERR_NUM_WORKERS;
    if (n == 0) return OGQ_OK;
    if (!d_codes || !d_levels || !d_out) return OGQ_ERR_NULL_POINTER;
    if (!aligned(d_out, 16)) return OGQ_ERR_ALIGNMENT;
    for (uint32_t w = 0; w < num_workers; ++w) {
        if (!d_codes[w] || !d_levels[w]) return OGQ_ERR_NULL_POINTER;
        if (!aligned(d_codes[w], 16) || !aligned(d_levels[w], 16)) return OGQ_ERR_ALIGNMENT;
    }
    if (ogq_num_buckets(n, params) >= (1ull << 31)) return OGQ_ERR_SIZE;
    begin_launches();
    ogq::launch_decode(d_codes, d_levels, num_workers, n, params, d_out, static_cast<hipStream_t>(hip_stream));
    return finish_launches();
}

int ogq_probe_read(const float* d_src, size_t n, float* d_sink, void* hip_stream)
{
    if (!d_src || !d_sink) return OGQ_ERR_NULL_POINTER;
    if (!aligned(d_src, 16)) return OGQ_ERR_ALIGNMENT;
    if (n == 0) return OGQ_OK;
    begin_launches();
    ogq::launch_probe_read(d_src, n, d_sink, static_cast<hipStream_t>(hip_stream));
    return finish_launches();
}

int ogq_probe_copy(const float* d_src, float* d_dst, size_t n, void* hip_stream)
{
    if (!d_src || !d_dst) return OGQ_ERR_NULL_POINTER;
    if (!aligned(d_src, 16) || !aligned(d_dst, 16)) return OGQ_ERR_ALIGNMENT;
    if (n == 0) return OGQ_OK;
    begin_launches();
    ogq::launch_probe_copy(d_src, d_dst, n, static_cast<hipStream_t>(hip_stream));
    return finish_launches();
}

const char* ogq_strerror(int status)
{
    switch (status) {
        case OGQ_OK: return "ok";
        case OGQ_ERR_NULL_POINTER: return "a required pointer is NULL";
        case OGQ_ERR_BUCKET_SIZE: return "bucket_size must be a multiple of 64 in [64, 32768]";
        case OGQ_ERR_BITS: return "bits not supported by the scheme (BinGrad-b / -pb: 1, ORQ: 1..3, ORQ_PAPER: 2..4)";
        case OGQ_ERR_SCHEME: return "unknown scheme";
        case OGQ_ERR_NUM_WORKERS: return "num_workers must be in [1, 64]";
        case OGQ_ERR_ALIGNMENT: return "device pointers must be 16-byte aligned";
        case OGQ_ERR_INDEX_OFFSET: return "index_offset must be a multiple of 64";
        case OGQ_ERR_LAUNCH: return "HIP kernel launch failed";
        case OGQ_ERR_SIZE: return "n is too large for one call";
        case OGQ_ERR_CLIP: return "clip_factor must be finite and not negative";
        case OGQ_ERR_RESERVED: return "the reserved field of the parameters must be 0";
        default: return "unknown status";
    }
}

int ogq_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"

