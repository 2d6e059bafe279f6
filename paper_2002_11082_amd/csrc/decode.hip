// libogq, decode + average kernel (server step of Algorithm 2 of arXiv 2002.11082) and the bandwidth probes,
// for MI355X (gfx950).
#include <type_traits>

#include "device_common.h"
#include "launch.h"

namespace ogq {

// ----------------------------------------------------------------------------------------------
// Decode + average.  One wavefront decodes a span of up to 16 packed word groups (1024 elements); lane l owns
// element 64*j + l of word group j.  Complete spans of bucket sizes with a fixed layout turn the code bits into
// per-lane level indices and look the levels up in LDS (below); the ragged last span and the other bucket sizes use
// the packed words directly as the lane masks of a tree of selects.
// ----------------------------------------------------------------------------------------------
struct WorkerPtrs {
    const uint64_t* codes[OGQ_MAX_WORKERS];
    const float* levels[OGQ_MAX_WORKERS];
};

constexpr int kSpanWords = 16;  // one wavefront decodes 16 packed word groups = 1024 elements

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

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

// ----------------------------------------------------------------------------------------------
// The span's code bits, turned so that every lane holds the bits of its own elements.  A span's code words are
// 16 * BITS rows of 64 bits (row = word group * BITS + bit plane, one bit per element of the group).  Lane 32 h + r
// loads the half h (32 elements) of rows r, r + 32, ...; a 32 x 32 bit-matrix transpose inside each half of the
// wavefront (five butterfly steps: the partner lane's word, rotated, replaces half of the bits) then leaves, in lane
// 32 h + b, bit `row` of the result = code bit of element 32 h + b of that row's group: the level index of group j
// sits at bits BITS j .. BITS j + BITS - 1 and indexes the bucket's level table in LDS directly.
// ----------------------------------------------------------------------------------------------
struct BitTranspose {
    uint32_t take[5];  // bits a lane takes from its partner at lane distance 16, 8, 4, 2, 1
    uint32_t turn[5];  // right rotation that brings the partner's bits into place
};

__device__ __forceinline__ BitTranspose bit_transpose_setup(uint32_t lane)
{
    BitTranspose t;
    constexpr uint32_t kLow[5] = {0x0000FFFFu, 0x00FF00FFu, 0x0F0F0F0Fu, 0x33333333u, 0x55555555u};
#pragma unroll
    for (int s = 0; s < 5; ++s) {
        const uint32_t j = 16u >> s;
        const bool upper = (lane & j) != 0u;
        // the lower lane of a pair keeps its low blocks and takes the partner's low blocks as its high blocks; the upper
        // lane keeps its high blocks and takes the partner's high blocks as its low blocks
        t.take[s] = upper ? kLow[s] : kLow[s] << j;
        t.turn[s] = upper ? j : 32u - j;
    }
    return t;
}

template <int DIST, int STEP>
__device__ __forceinline__ uint32_t bit_transpose_step(uint32_t x, const BitTranspose& t, uint32_t lane)
{
    const uint32_t y = lane_xor<DIST>(x, lane);
    const uint32_t turned = __builtin_amdgcn_alignbit(y, y, t.turn[STEP]);
    // take ? turned : x, bit by bit, in one instruction (v_bitop3_b32, truth table 0xCA)
    return __builtin_amdgcn_bitop3_b32(t.take[STEP], turned, x, 0xCA);
}

__device__ __forceinline__ uint32_t bit_transpose(uint32_t x, const BitTranspose& t, uint32_t lane)
{
    x = bit_transpose_step<16, 0>(x, t, lane);
    x = bit_transpose_step<8, 1>(x, t, lane);
    x = bit_transpose_step<4, 2>(x, t, lane);
    x = bit_transpose_step<2, 3>(x, t, lane);
    return bit_transpose_step<1, 4>(x, t, lane);
}

// Level index of word group J from the turned code bits (R registers of 32 rows each).
template <int BITS, int J, int R>
__device__ __forceinline__ uint32_t level_index(const uint32_t (&turned)[R])
{
    constexpr int kFirst = BITS * J, kReg = kFirst / 32, kShift = kFirst % 32;
    uint32_t index;
    if constexpr (kShift + BITS <= 32) {
        index = __builtin_amdgcn_ubfe(turned[kReg], (uint32_t)kShift, (uint32_t)BITS);  // one v_bfe_u32
    } else {
        index = __builtin_amdgcn_alignbit(turned[kReg + 1], turned[kReg], (uint32_t)kShift) & ((1u << BITS) - 1u);
    }
    // (kept as it is: folded into the address arithmetic, the extraction turns into a shift, a mask and an addition
    // instead of this bit-field extract and one shift-and-add)
    asm("" : "+v"(index));
    return index;
}

// Runs f(J, index of word group J) for the 16 word groups of a span; an index has BITS bits.
template <int BITS, int J, int R, class F>
__device__ __forceinline__ void for_each_group(const uint32_t (&turned)[R], F&& f)
{
    if constexpr (J < kSpanWords) {
        f(std::integral_constant<int, J>{}, level_index<BITS, J>(turned));
        for_each_group<BITS, J + 1>(turned, f);
    }
}

// WPB = packed word groups per bucket when the span splits into whole buckets at fixed places: 16 = the
// span lies in one bucket (bucket_size is a multiple of 1024; its index is word0 / words_per_bucket),
// 1, 2, 4 or 8 = bucket_size 64 .. 512, the span holds 16 / WPB buckets whose level tables are
// consecutive in memory.  Each table is fetched once per span and worker.  WPB = 0: any other bucket
// size, the table is looked up per word group.
// ONE: the launch has a single worker (its own instantiation: without the fp64 sums of the general case the kernel
// needs half the registers, and twice the wavefronts are in flight to hide the first trip to HBM).
template <int BITS, int S, int WPB, bool ONE>
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
        // tables are fetched with vector loads (one dword per lane and register), for several workers at once so
        // that their trips to HBM overlap.  The code bits are turned into per-lane level indices (bit_transpose), the
        // level tables go to a table in LDS that belongs to this wavefront, and an element's level is one LDS read.
        // (Scalar loads, which would deliver the words as lane masks for a select tree, keep too few bytes in flight
        // per wavefront once the streams come from HBM instead of the last-level cache; moving vector-loaded words
        // to scalar registers costs two v_readlane per word.)
        constexpr int kWpb = WPB > 0 ? WPB : 1;
        constexpr int kTables = kSpanWords / kWpb;
        const BitTranspose turn = bit_transpose_setup(lane);
        const uint32_t half = lane >> 5, row = lane & 31u;
        const uint32_t first_bucket = WPB == kSpanWords ? word0 / words_per_bucket : word0 / (uint32_t)kWpb;
        const uint32_t wave = uniform_u32(threadIdx.x >> 6);
        bool combined = false;
        if constexpr (kTables <= 2 && !ONE) {
          if (num_workers > 1u) {
            combined = true;
            // Several workers per look-up: K workers' indices of an element form one index of K * BITS bits into a
            // table that holds, in fp64, the sum of the K levels for every combination of their indices (built once per
            // span from the K level tables).  One LDS read and one fp64 addition then serve K workers.  The rows of
            // code bits are fetched so that one transpose leaves the K * BITS bits of an element side by side: row
            // (group j, worker i, plane p) is number j * K * BITS + i * BITS + p.
            constexpr int K = BITS >= 4 ? 1 : 6 / BITS;           // workers per look-up
            constexpr int IDX = K * BITS;                         // index bits of a look-up: 6, or 4 for 4-bit codes
            constexpr int ENTRIES = 1 << IDX;                     // at most 64: one table entry per lane
            constexpr int RR = kSpanWords * IDX / 32;             // registers of turned code bits per look-up
            constexpr uint32_t FLIGHT = 3;                        // look-ups whose loads are in flight together
            constexpr int RAW = K * kTables * S;                  // level values of the K workers of a look-up
            static_assert(RAW <= 64 && ENTRIES <= 64, "one lane per level value and per table entry");
            constexpr int WD = 2 * kSpanWords * BITS;             // dwords of one worker's code words of the span
            constexpr int WR = (WD + 63) / 64;                    // registers that fetch them, one dword per lane
            __shared__ double sum_tables[kWavesPerBlock][FLIGHT][kTables][ENTRIES];
            __shared__ float raw_levels[kWavesPerBlock][FLIGHT][RAW];
            __shared__ uint32_t staged_codes[kWavesPerBlock][FLIGHT][K][WD];
            const uint32_t lookups = (num_workers + K - 1) / K;
            for (uint32_t g0 = 0; g0 < lookups; g0 += FLIGHT) {
                // every worker's code words and level tables with plain coalesced loads (the worker is wave-uniform)
                uint32_t fetched[FLIGHT][K][WR];
                float level_reg[FLIGHT][K];
#pragma unroll
                for (uint32_t f = 0; f < FLIGHT; ++f)
#pragma unroll
                    for (int i = 0; i < K; ++i) {
                        const uint32_t w = (g0 + f) * K + i;
#pragma unroll
                        for (int k = 0; k < WR; ++k) fetched[f][i][k] = 0u;  // a worker that does not exist: index 0 ...
                        level_reg[f][i] = 0.0f;                              // ... of a table of zeros
                        if (w < num_workers) {
                            const uint32_t* c32 = reinterpret_cast<const uint32_t*>(ptrs.codes[w] + (size_t)word0 * BITS);
#pragma unroll
                            for (int k = 0; k < WR; ++k)
                                if (64u * k + lane < (uint32_t)WD) fetched[f][i][k] = c32[64u * k + lane];
                            if (lane < (uint32_t)(kTables * S)) level_reg[f][i] = ptrs.levels[w][(size_t)first_bucket * S + lane];
                        }
                    }
                wave_lds_fence();  // the reads of the round before are done
#pragma unroll
                for (uint32_t f = 0; f < FLIGHT; ++f) {
                    if ((g0 + f) * K >= num_workers) continue;  // (wave-uniform) no such look-up
#pragma unroll
                    for (int i = 0; i < K; ++i) {
#pragma unroll
                        for (int k = 0; k < WR; ++k)
                            if (64u * k + lane < (uint32_t)WD) staged_codes[wave][f][i][64u * k + lane] = fetched[f][i][k];
                        if (lane < (uint32_t)(kTables * S)) raw_levels[wave][f][i * (kTables * S) + lane] = level_reg[f][i];
                    }
                }
                wave_lds_fence();
                // the rows in the order of the look-up index: row (group j, worker i, plane p) is number j * IDX + i * BITS + p
                uint32_t code_reg[FLIGHT][RR];
#pragma unroll
                for (int q = 0; q < RR; ++q) {
                    const uint32_t r = 32u * q + row;  // row of code bits this lane takes its half of
                    const uint32_t j = r / IDX, rem = r % IDX, i = rem / BITS, plane = rem % BITS;
#pragma unroll
                    for (uint32_t f = 0; f < FLIGHT; ++f) {
                        code_reg[f][q] = 0u;
                        if ((g0 + f) * K < num_workers) code_reg[f][q] = staged_codes[wave][f][i][2u * (j * BITS + plane) + half];
                    }
                }
                wave_lds_fence();
#pragma unroll
                for (uint32_t f = 0; f < FLIGHT; ++f) {
                    if ((g0 + f) * K < num_workers && lane < (uint32_t)ENTRIES) {
#pragma unroll
                        for (int t = 0; t < kTables; ++t) {
                            double sum = 0.0;
#pragma unroll
                            for (int i = 0; i < K; ++i) {
                                uint32_t index = (lane >> (i * BITS)) & ((1u << BITS) - 1u);
                                index = index < (uint32_t)S ? index : (uint32_t)(S - 1);  // (an index that never occurs)
                                sum += (double)raw_levels[wave][f][(i * kTables + t) * S + index];
                            }
                            sum_tables[wave][f][t][lane] = sum;
                        }
                    }
                }
                wave_lds_fence();
#pragma unroll
                for (uint32_t f = 0; f < FLIGHT; ++f) {
                    if ((g0 + f) * K < num_workers) {
                        uint32_t turned[RR];
#pragma unroll
                        for (int q = 0; q < RR; ++q) turned[q] = bit_transpose(code_reg[f][q], turn, lane);
                        for_each_group<IDX, 0>(turned, [&](auto j, uint32_t index) {
                            acc[decltype(j)::value] += sum_tables[wave][f][decltype(j)::value / kWpb][index];
                        });
                    }
                }
            }
          }
        }
        if (!combined) {
            // One worker per look-up: fp32 level tables in LDS.  A single worker's average is its level itself.
            constexpr int R = (kSpanWords * BITS + 31) / 32;  // registers for the 16 * BITS rows of code bits
            constexpr int LR = (kTables * S + 63) / 64;       // registers for the kTables * S level values
            constexpr uint32_t BATCH = R + LR > 2 ? 4 : 8;    // workers whose loads are in flight together
            __shared__ float level_tables[kWavesPerBlock][BATCH * kTables * S];
            float* my_tables = level_tables[wave];
            constexpr bool one_worker = ONE;
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
                            const uint32_t r = 32u * k + row;  // row of code bits this lane fetches its half of
                            if (r < (uint32_t)(kSpanWords * BITS)) code_reg[b][k] = c32[2u * r + half];
                        }
#pragma unroll
                        for (int k = 0; k < LR; ++k) {
                            const uint32_t i = 64u * k + lane;
                            if (i < (uint32_t)(kTables * S)) level_reg[b][k] = tables[i];
                        }
                    }
                }
                wave_lds_fence();  // the reads of the batch before are done
#pragma unroll
                for (uint32_t b = 0; b < BATCH; ++b) {
#pragma unroll
                    for (int k = 0; k < LR; ++k) {
                        const uint32_t i = 64u * k + lane;
                        if (i < (uint32_t)(kTables * S)) my_tables[b * (kTables * S) + i] = level_reg[b][k];
                    }
                }
                wave_lds_fence();
#pragma unroll
                for (uint32_t b = 0; b < BATCH; ++b) {
                    if (w0 + b < num_workers) {
                        uint32_t turned[R];
#pragma unroll
                        for (int k = 0; k < R; ++k) turned[k] = bit_transpose(code_reg[b][k], turn, lane);
                        const float* table = my_tables + b * (kTables * S);
                        if (one_worker) {
                            float* __restrict__ o1 = out + (size_t)word0 * 64 + lane;
                            for_each_group<BITS, 0>(turned, [&](auto j, uint32_t index) {
                                // written once, never re-read here
                                __builtin_nontemporal_store(table[(decltype(j)::value / kWpb) * S + index], o1 + 64 * decltype(j)::value);
                            });
                            return;
                        }
                        for_each_group<BITS, 0>(turned, [&](auto j, uint32_t index) {
                            acc[decltype(j)::value] += (double)table[(decltype(j)::value / kWpb) * S + index];
                        });
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
#define OGQ_LAUNCH_DEQUANT_WPB(BITS, S, WPB)                                                                              \
    do {                                                                                                                 \
        if (num_workers == 1u)                                                                                           \
            launch_kernel((dequantize_average_kernel<BITS, S, WPB, true>), grid, block, st, ptrs, num_workers, n, wpb,   \
                          total_words, inv, d_out);                                                                      \
        else                                                                                                             \
            launch_kernel((dequantize_average_kernel<BITS, S, WPB, false>), grid, block, st, ptrs, num_workers, n, wpb,  \
                          total_words, inv, d_out);                                                                      \
    } while (0)
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
