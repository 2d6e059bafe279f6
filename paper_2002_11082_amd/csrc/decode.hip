// libogq, decode + average kernel (server step of Algorithm 2 of arXiv 2002.11082) and the bandwidth probes,
// for MI355X (gfx950).
#include "device_common.h"
#include "launch.h"

namespace ogq {

// ----------------------------------------------------------------------------------------------
// Decode + average.  One wavefront decodes a segment of up to 16 packed words (1024 elements)
// that lies inside one bucket; lane l owns element 64*j + l of word j, so the packed words are
// the lane masks of the level selects.
// ----------------------------------------------------------------------------------------------
struct WorkerPtrs {
    const uint64_t* codes[OGQ_MAX_WORKERS];
    const float* levels[OGQ_MAX_WORKERS];
};

constexpr int kSpanWords = 16;  // one wavefront decodes 16 packed word groups = 1024 elements

// Level selected by the packed words of one 64-element group: the words are the lane masks of the
// selects.  S = 2^BITS levels: a full binary tree; S = 2^(BITS-1) + 1 levels (the paper's counts):
// the top bit alone means the last level.
template <int BITS>
__device__ __forceinline__ float select_tree(const bool (&bit)[4], const float* lv)
{
    if constexpr (BITS == 0) {
        return lv[0];
    } else {
        const float lo = select_tree<BITS - 1>(bit, lv);
        const float hi = select_tree<BITS - 1>(bit, lv + (1 << (BITS - 1)));
        return bit[BITS - 1] ? hi : lo;
    }
}

template <int BITS, int S>
__device__ __forceinline__ float select_from_bits(const bool (&bit)[4], const float (&lv)[S])
{
    if constexpr (S == (1 << BITS)) {
        return select_tree<BITS>(bit, lv);
    } else {
        static_assert(S == (1 << (BITS - 1)) + 1, "level count");
        const float low = select_tree<BITS - 1>(bit, lv);
        return bit[BITS - 1] ? lv[S - 1] : low;
    }
}

template <int BITS, int S>
__device__ __forceinline__ float select_level(const uint64_t* __restrict__ w, const float (&lv)[S])
{
    bool bit[4] = {false, false, false, false};
#pragma unroll
    for (int p = 0; p < BITS; ++p) bit[p] = __builtin_amdgcn_inverse_ballot_w64(w[p]);
    if constexpr (S == (1 << BITS)) {
        return select_tree<BITS>(bit, lv);
    } else {
        static_assert(S == (1 << (BITS - 1)) + 1, "level count");
        const float low = select_tree<BITS - 1>(bit, lv);
        return bit[BITS - 1] ? lv[S - 1] : low;
    }
}

// Loads one bucket's level table (wave-uniform address, scalar loads) into vector registers: the
// selects take two vector sources and the packed word as their lane mask.
template <int S>
__device__ __forceinline__ void load_levels(const float* __restrict__ table, float (&lv)[S])
{
    float s[S];
#pragma unroll
    for (int k = 0; k < S; ++k) s[k] = table[k];
#pragma unroll
    for (int k = 0; k < S; ++k) asm("v_mov_b32 %0, %1" : "=v"(lv[k]) : "s"(s[k]));
}

// WPB = packed word groups per bucket when the span splits into whole buckets at fixed places: 16 = the
// span lies in one bucket (bucket_size is a multiple of 1024; its index is word0 / words_per_bucket),
// 1, 2, 4 or 8 = bucket_size 64 .. 512, the span holds 16 / WPB buckets whose level tables are
// consecutive in memory.  Each table is fetched once per span and worker.  WPB = 0: any other bucket
// size, the table is looked up per word group.
template <int BITS, int S, int WPB>
__global__ __launch_bounds__(kBlock) void dequantize_average_kernel(WorkerPtrs ptrs, uint32_t num_workers, size_t n,
                                                                    uint32_t words_per_bucket, uint32_t total_words,
                                                                    double inv_workers, float* __restrict__ out)
{
    const uint32_t span = blockIdx.x * kWavesPerBlock + uniform_u32(threadIdx.x >> 6);
    const uint32_t word0 = span * kSpanWords;
    if (word0 >= total_words) return;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t rest = total_words - word0;
    const uint32_t n_words = rest < (uint32_t)kSpanWords ? rest : (uint32_t)kSpanWords;
    // every element of the span exists: no per-word or per-element bounds tests
    const bool whole = n_words == (uint32_t)kSpanWords && ((size_t)word0 + kSpanWords) * 64 <= n;

    double acc[kSpanWords];
#pragma unroll
    for (int j = 0; j < kSpanWords; ++j) acc[j] = 0.0;

    if (WPB > 0 && whole) {
        // Every element of the span exists and its buckets lie at fixed places: the span's code words and level
        // tables are fetched with vector loads (lane i takes dword i), for several workers at once so that their
        // trips to HBM overlap, and reach the scalar registers through v_readlane.  (Scalar loads, which deliver the
        // lane masks directly, keep too few bytes in flight per wavefront once the streams come from HBM instead of
        // the last-level cache.)
        constexpr int kTables = WPB > 0 ? kSpanWords / WPB : 1;
        constexpr int R = (32 * BITS + 63) / 64;        // registers for the 32 * BITS dwords of code words
        constexpr int LR = (kTables * S + 63) / 64;     // registers for the kTables * S level values
        constexpr uint32_t BATCH = R + LR > 2 ? 4 : 8;  // workers in flight
        const uint32_t first_bucket = WPB == kSpanWords ? word0 / words_per_bucket : word0 / (uint32_t)(WPB > 0 ? WPB : 1);
        for (uint32_t w0 = 0; w0 < num_workers; w0 += BATCH) {
            uint32_t code_reg[BATCH][R];
            float level_reg[BATCH][LR];
#pragma unroll
            for (uint32_t b = 0; b < BATCH; ++b) {
#pragma unroll
                for (int k = 0; k < R; ++k) code_reg[b][k] = 0u;
#pragma unroll
                for (int k = 0; k < LR; ++k) level_reg[b][k] = 0.0f;
                if (w0 + b < num_workers) {
                    const uint32_t* c32 = reinterpret_cast<const uint32_t*>(ptrs.codes[w0 + b] + (size_t)word0 * BITS);
                    const float* tables = ptrs.levels[w0 + b] + (size_t)first_bucket * S;
#pragma unroll
                    for (int k = 0; k < R; ++k) {
                        const uint32_t i = 64u * k + lane;
                        if (i < 32u * BITS) code_reg[b][k] = c32[i];
                    }
#pragma unroll
                    for (int k = 0; k < LR; ++k) {
                        const uint32_t i = 64u * k + lane;
                        if (i < (uint32_t)(kTables * S)) level_reg[b][k] = tables[i];
                    }
                }
            }
#pragma unroll
            for (uint32_t b = 0; b < BATCH; ++b) {
                if (w0 + b < num_workers) {
#pragma unroll
                    for (int t = 0; t < kTables; ++t) {
                        float lv[S];
#pragma unroll
                        for (int k = 0; k < S; ++k) {
                            const int at = t * S + k;
                            lv[k] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(level_reg[b][at / 64]), at % 64));
                        }
#pragma unroll
                        for (int j = t * (WPB > 0 ? WPB : 1); j < (t + 1) * (WPB > 0 ? WPB : 1); ++j) {
                            bool bit[4] = {false, false, false, false};
#pragma unroll
                            for (int p = 0; p < BITS; ++p) {
                                const int d0 = 2 * (j * BITS + p), d1 = d0 + 1;
                                const uint32_t lo = __builtin_amdgcn_readlane(code_reg[b][d0 / 64], d0 % 64);
                                const uint32_t hi = __builtin_amdgcn_readlane(code_reg[b][d1 / 64], d1 % 64);
                                bit[p] = __builtin_amdgcn_inverse_ballot_w64(((uint64_t)hi << 32) | lo);
                            }
                            acc[j] += (double)select_from_bits<BITS, S>(bit, lv);
                        }
                    }
                }
            }
        }
    } else  // the ragged end of the gradient and bucket sizes without a fixed layout: scalar loads, word by word
    for (uint32_t w = 0; w < num_workers; ++w) {
        const uint64_t* __restrict__ cw = ptrs.codes[w] + (size_t)word0 * BITS;
        const float* __restrict__ table = ptrs.levels[w];
        if constexpr (WPB > 0) {
            constexpr int kTables = kSpanWords / WPB;
            const uint32_t first_bucket = WPB == kSpanWords ? word0 / words_per_bucket : word0 / (uint32_t)WPB;
            const float* __restrict__ first_table = table + (size_t)first_bucket * S;
#pragma unroll
            for (int t = 0; t < kTables; ++t)
                if ((uint32_t)(t * WPB) < n_words) {  // a bucket past the end has no table
                    float lv[S];
                    load_levels<S>(first_table + t * S, lv);
#pragma unroll
                    for (int j = t * WPB; j < (t + 1) * WPB; ++j)
                        if ((uint32_t)j < n_words) acc[j] += (double)select_level<BITS, S>(cw + j * BITS, lv);
                }
        } else {
#pragma unroll
            for (int j = 0; j < kSpanWords; ++j)
                if ((uint32_t)j < n_words) {
                    float lv[S];
                    load_levels<S>(table + (size_t)((word0 + j) / words_per_bucket) * S, lv);
                    acc[j] += (double)select_level<BITS, S>(cw + j * BITS, lv);
                }
        }
    }
    float* __restrict__ o = out + (size_t)word0 * 64 + lane;
    if (whole) {
#pragma unroll
        for (int j = 0; j < kSpanWords; ++j)
            __builtin_nontemporal_store((float)(acc[j] * inv_workers), o + 64 * j);  // written once, never re-read here
    } else {
        const size_t first = (size_t)word0 * 64 + lane;
#pragma unroll
        for (int j = 0; j < kSpanWords; ++j)
            if ((uint32_t)j < n_words && first + 64u * j < n)
                __builtin_nontemporal_store((float)(acc[j] * inv_workers), o + 64 * j);
    }
}

// ----------------------------------------------------------------------------------------------
// Bandwidth probes.
// ----------------------------------------------------------------------------------------------
constexpr uint32_t kProbeBlocks = 256 * 8;

__global__ __launch_bounds__(kBlock) void probe_read_kernel(const float4* __restrict__ src, size_t n4,
                                                            float* __restrict__ sink)
{
    float acc = 0.f;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (size_t)gridDim.x * kBlock) {
        const float4 q = src[i];
        acc += (q.x + q.y) + (q.z + q.w);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, kWave);
    if ((threadIdx.x & 63u) == 0) sink[blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)] = acc;
}

__global__ __launch_bounds__(kBlock) void probe_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                            size_t n4)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += (size_t)gridDim.x * kBlock)
        dst[i] = src[i];
}

// ----------------------------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------------------------
void launch_decode(const void* const* d_codes, const float* const* d_levels, uint32_t num_workers, size_t n,
                   const ogq_params_t* p, float* d_out, hipStream_t st)
{
    WorkerPtrs ptrs;
    for (uint32_t w = 0; w < OGQ_MAX_WORKERS; ++w) {
        ptrs.codes[w] = nullptr;
        ptrs.levels[w] = nullptr;
    }
    for (uint32_t w = 0; w < num_workers; ++w) {
        ptrs.codes[w] = static_cast<const uint64_t*>(d_codes[w]);
        ptrs.levels[w] = d_levels[w];
    }
    const uint32_t d = p->bucket_size;
    const uint32_t total_words = (uint32_t)(n / 64 + (n % 64 != 0));
    const uint32_t spans = (total_words + kSpanWords - 1) / kSpanWords;
    const dim3 grid((spans + kWavesPerBlock - 1) / kWavesPerBlock), block(kBlock);
    const double inv = 1.0 / (double)num_workers;
    const uint32_t wpb = d / 64;
    const uint32_t span_elements = kSpanWords * 64;
    const uint32_t fixed_wpb = d % span_elements == 0 ? (uint32_t)kSpanWords : (span_elements % d == 0 ? wpb : 0u);
#define OGQ_LAUNCH_DEQUANT_WPB(BITS, S, WPB)                                                                      \
    launch_kernel((dequantize_average_kernel<BITS, S, WPB>), grid, block, st, ptrs, num_workers, n, wpb, \
                       total_words, inv, d_out)
#define OGQ_LAUNCH_DEQUANT(BITS, S)                                \
    do {                                                           \
        switch (fixed_wpb) {                                       \
            case 16: OGQ_LAUNCH_DEQUANT_WPB(BITS, S, 16); break;   \
            case 8: OGQ_LAUNCH_DEQUANT_WPB(BITS, S, 8); break;     \
            case 4: OGQ_LAUNCH_DEQUANT_WPB(BITS, S, 4); break;     \
            case 2: OGQ_LAUNCH_DEQUANT_WPB(BITS, S, 2); break;     \
            case 1: OGQ_LAUNCH_DEQUANT_WPB(BITS, S, 1); break;     \
            default: OGQ_LAUNCH_DEQUANT_WPB(BITS, S, 0); break;    \
        }                                                          \
    } while (0)
    switch (levels_per_bucket(p->scheme, p->bits)) {
        case 2: OGQ_LAUNCH_DEQUANT(1, 2); break;
        case 4: OGQ_LAUNCH_DEQUANT(2, 4); break;
        case 8: OGQ_LAUNCH_DEQUANT(3, 8); break;
        case 3: OGQ_LAUNCH_DEQUANT(2, 3); break;
        case 5: OGQ_LAUNCH_DEQUANT(3, 5); break;
        default: OGQ_LAUNCH_DEQUANT(4, 9); break;
    }
#undef OGQ_LAUNCH_DEQUANT
#undef OGQ_LAUNCH_DEQUANT_WPB
}

void launch_probe_read(const float* d_src, size_t n, float* d_sink, hipStream_t st)
{
    launch_kernel(probe_read_kernel, dim3(kProbeBlocks), dim3(kBlock), st,
                       reinterpret_cast<const float4*>(d_src), n / 4, d_sink);
}

void launch_probe_copy(const float* d_src, float* d_dst, size_t n, hipStream_t st)
{
    launch_kernel(probe_copy_kernel, dim3(kProbeBlocks), dim3(kBlock), st,
                       reinterpret_cast<const float4*>(d_src), reinterpret_cast<float4*>(d_dst), n / 4);
}

}  // namespace ogq
