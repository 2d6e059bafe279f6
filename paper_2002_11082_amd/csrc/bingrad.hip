// libogq, BinGrad-b and Scaled SignSGD quantize kernels (Section 3.2 of arXiv 2002.11082) for MI355X (gfx950).
// Compile with -ffp-contract=off.
#include "device_common.h"
#include "launch.h"

namespace ogq {

// x unchanged, but opaque to the optimizer: what is derived from it is computed again instead of kept in registers.
__device__ __forceinline__ float reread(float x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// ----------------------------------------------------------------------------------------------
// BinGrad-b quantize.  Lane l register j holds bucket element 64*j + l, so a ballot over
// register j is the packed code word j of the bucket.
// ----------------------------------------------------------------------------------------------
// E registers per lane; FULL: every register of this wavefront holds a bucket element.  g, len, levels2
// and words belong to the whole bucket, of which this wavefront holds the 64*E elements from `first_element` on;
// the wavefront with first_element == 0 writes the levels.  SIGN: Scaled SignSGD instead (first equation of
// Section 3.2): levels -m, +m with m the mean magnitude of the bucket, index = (v >= 0).
template <int E, bool FULL, bool CLIP, bool SIGN, class Team>
__device__ __forceinline__ void bingrad_bucket(Team team, uint32_t first_element, const float* __restrict__ g,
                                               uint32_t len, uint32_t iters, float clip, float* __restrict__ levels2,
                                               uint64_t* __restrict__ words)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t first = first_element + lane;
    float v[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const uint32_t e = first + 64u * j;
        v[j] = (FULL || e < len) ? __builtin_nontemporal_load(g + e) : 0.0f;  // read once: bypass the caches
    }
    if constexpr (CLIP)
        clip_in_registers<E>(
            v, len, clip, [&](int j) { return FULL || (first + 64u * j < len); },
            [&](double x) { return team.sum(wave_sum(x)); });

    double part = 0.0;
    float mag = 0.0f;
#pragma unroll
    for (int j = 0; j < E; ++j) {
        part += (double)(SIGN ? fabsf(v[j]) : v[j]);
        mag = fmaxf(mag, fabsf(v[j]));
    }
    double total = wave_sum(part);
    float largest = wave_max(mag);
    team.sum_and_max(total, largest);
    float b0 = (float)(total / (double)len);  // threshold starts at the bucket mean
    // The upper sum is taken as total - lower sum.  Both are fp64 sums of the bucket's n <= 32768 fp32 values
    // (error below 2^-53 * n^2 * max|v| each, and exact for any bucket whose non-zero values span at most
    // 28 - log2(n) binades: 17 for 2048 elements, 13 for 32768), so the difference is trusted unless it is tiny
    // against the largest element; such a bucket sums its upper side directly.
    const float trust_above = 1e-3f * largest;

    double b_lo = 0.0, b_hi = 0.0;
    uint32_t word_lo = 0, word_hi = 0;  // lane j ends up holding packed word j of this wavefront's elements
    uint32_t prev_n_lo = 0xFFFFFFFFu;
    if constexpr (SIGN) {
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const bool valid = FULL || (first + 64u * j < len);
            const uint64_t hi_mask = __ballot(valid && !(v[j] < 0.0f));
            word_lo = writelane(word_lo, (uint32_t)hi_mask, j);
            word_hi = writelane(word_hi, (uint32_t)(hi_mask >> 32), j);
        }
        b_hi = total / (double)len;
        b_lo = -b_hi;
    } else
    for (uint32_t it = 0;; ++it) {
        double s_lo = 0.0;
        uint32_t below = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const bool valid = FULL || (first + 64u * j < len);
            // (with 64 registers of data the fp64 copies the compiler would keep from the first pass do not fit)
            const float x = E > 32 ? reread(v[j]) : v[j];
            const bool lo = valid && (x < b0);
            const uint64_t lo_mask = __ballot(lo);
            const uint64_t hi_mask = FULL ? ~lo_mask : __ballot(valid && !lo);
            below += lo ? 1u : 0u;
            s_lo += (double)(lo ? x : 0.0f);
            word_lo = writelane(word_lo, (uint32_t)hi_mask, j);
            word_hi = writelane(word_hi, (uint32_t)(hi_mask >> 32), j);
        }
        s_lo = wave_sum(s_lo);
        uint32_t n_lo = wave_sum_u32(below);
        team.sum_and_count(s_lo, n_lo);
        double s_hi = total - s_lo;
        if (!(fabs(s_hi) >= (double)trust_above)) {
            double direct = 0.0;
#pragma unroll
            for (int j = 0; j < E; ++j) {
                const bool valid = FULL || (first + 64u * j < len);
                direct += (double)((valid && !(v[j] < b0)) ? v[j] : 0.0f);
            }
            s_hi = team.sum(wave_sum(direct));
        }
        const uint32_t n_hi = len - n_lo;
        {
            // both conditional means with one division sequence: lane 0 divides the lower side, the
            // other lanes the upper side
            const double num = lane == 0 ? s_lo : s_hi;
            const uint32_t den = lane == 0 ? n_lo : n_hi;
            const double quot = num / (double)(den > 0 ? den : 1u);
            if (n_lo > 0) b_lo = readlane_f64(quot, 0);
            if (n_hi > 0) b_hi = readlane_f64(quot, 1);
        }
        if (n_lo == 0) b_lo = b_hi;  // constant bucket: both levels equal
        if (n_hi == 0) b_hi = b_lo;
        // Further threshold updates are identities once the partition repeats.
        if (it == iters || n_lo == prev_n_lo) break;
        prev_n_lo = n_lo;
        b0 = (float)((b_lo + b_hi) * 0.5);
    }

    if (lane == 0 && first_element == 0) {
        levels2[0] = (float)b_lo;
        levels2[1] = (float)b_hi;
    }
    const uint32_t n_words = (len + 63u) / 64u;
    const uint32_t word = first_element / 64u + lane;
    if (lane < (uint32_t)E && word < n_words) words[word] = ((uint64_t)word_hi << 32) | word_lo;
}

constexpr int kBinGradWaves = 2;  // buckets per workgroup

// At most 4 waves per SIMD and small workgroups: with more, all resident waves load and then
// compute in lock-step and the tail of a launch that is only ~1.5 waves of workgroups deep is not
// overlapped.
template <int E, bool CLIP, bool SIGN>
__global__ __launch_bounds__(kWave* kBinGradWaves) __attribute__((amdgpu_waves_per_eu(4, 4))) void bingrad_quantize_kernel(
    const float* __restrict__ grad, size_t n, uint32_t bucket_size, uint32_t iters, float clip, uint32_t num_buckets,
    float* __restrict__ levels, uint64_t* __restrict__ codes)
{
    const uint32_t bucket = uniform_u32(blockIdx.x * kBinGradWaves + (threadIdx.x >> 6));
    if (bucket >= num_buckets) return;
    const size_t begin = (size_t)bucket * bucket_size;
    const size_t rest = n - begin;
    const uint32_t len = rest < bucket_size ? (uint32_t)rest : bucket_size;
    const float* g = grad + begin;
    float* lv = levels + (size_t)bucket * 2;
    uint64_t* w = codes + begin / 64;
    if (len == 64u * E) bingrad_bucket<E, true, CLIP, SIGN>(OneWave{}, 0u, g, len, iters, clip, lv, w);
    else bingrad_bucket<E, false, CLIP, SIGN>(OneWave{}, 0u, g, len, iters, clip, lv, w);
}

// Buckets of more than 2048 elements: the W = 2, 4, 8 or 16 wavefronts of a workgroup hold one bucket, E = 32
// registers per lane each as for a 2048-element bucket, and combine their sums and counts through LDS.  Above
// 8192 elements E = 64 (without clipping), so that a workgroup is at most 8 wavefronts and two buckets share a
// compute unit: the loads of one overlap the passes of the other.
template <int W, int E, bool CLIP, bool SIGN>
__global__ __launch_bounds__(W* kWave) __attribute__((amdgpu_waves_per_eu(4, 4))) void bingrad_team_kernel(
    const float* __restrict__ grad, size_t n, uint32_t bucket_size, uint32_t iters, float clip, uint32_t num_buckets,
    float* __restrict__ levels, uint64_t* __restrict__ codes)
{
    __shared__ TeamSlot slots[2][W];
    const uint32_t bucket = blockIdx.x;
    if (bucket >= num_buckets) return;
    const size_t begin = (size_t)bucket * bucket_size;
    const size_t rest = n - begin;
    const uint32_t len = rest < bucket_size ? (uint32_t)rest : bucket_size;
    const float* g = grad + begin;
    float* lv = levels + (size_t)bucket * 2;
    uint64_t* w = codes + begin / 64;
    const uint32_t wave = uniform_u32(threadIdx.x >> 6);
    const WaveTeam<W> team{slots, wave, 0u};
    constexpr uint32_t PER_WAVE = 64u * E;
    // A wavefront whose 64 E elements all lie inside the bucket skips the per-element bounds tests.  Both variants
    // reach the same combines in the same order (every branch around one depends on combined values only).
    if (PER_WAVE * (wave + 1u) <= len) bingrad_bucket<E, true, CLIP, SIGN>(team, PER_WAVE * wave, g, len, iters, clip, lv, w);
    else bingrad_bucket<E, false, CLIP, SIGN>(team, PER_WAVE * wave, g, len, iters, clip, lv, w);
}

// ----------------------------------------------------------------------------------------------
// BinGrad-b for bucket sizes that divide 2048: one wavefront quantizes NB = 2048 / bucket_size whole
// buckets at once (registers E*q .. E*q + E - 1 hold its bucket q in the layout above), so that a
// small bucket keeps as many loads in flight per wave as a 2048-element one and the per-bucket
// reductions and divisions are shared.  The NB partial results of a pass are reduced together: a
// step over lane bit 5, 4, 3, ... combines two partner lanes and halves the number of values a lane
// carries, the lanes with the bit clear keeping the even-numbered values and the others the
// odd-numbered ones.  When one value is left lane l holds the result of bucket q(l) = (l with its six
// bits reversed) mod NB, and the remaining low lane bits are reduced as in wave_sum.
// ----------------------------------------------------------------------------------------------
constexpr int kDppXor1From0 = 0xA0;  // quad_perm [0,0,2,2]: an odd lane takes the even lane below it

__device__ __forceinline__ double words_to_f64(uint32_t lo, uint32_t hi)
{
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// swap_halves: first = {a[0..31], b[0..31]}, second = {a[32..63], b[32..63]} (v_permlane32_swap).
// swap_rows: the same over pairs of 16-lane rows: first = {a.row0, b.row0, a.row2, b.row2},
// second = {a.row1, b.row1, a.row3, b.row3} (v_permlane16_swap).
__device__ __forceinline__ void swap_halves(float a, float b, float& first, float& second)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    first = __uint_as_float(r[0]);
    second = __uint_as_float(r[1]);
}

__device__ __forceinline__ void swap_halves(double a, double b, double& first, double& second)
{
    const uint64_t ua = (uint64_t)__double_as_longlong(a), ub = (uint64_t)__double_as_longlong(b);
    const auto lo = __builtin_amdgcn_permlane32_swap((uint32_t)ua, (uint32_t)ub, false, false);
    const auto hi = __builtin_amdgcn_permlane32_swap((uint32_t)(ua >> 32), (uint32_t)(ub >> 32), false, false);
    first = words_to_f64(lo[0], hi[0]);
    second = words_to_f64(lo[1], hi[1]);
}

__device__ __forceinline__ void swap_rows(float a, float b, float& first, float& second)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    first = __uint_as_float(r[0]);
    second = __uint_as_float(r[1]);
}

__device__ __forceinline__ void swap_rows(double a, double b, double& first, double& second)
{
    const uint64_t ua = (uint64_t)__double_as_longlong(a), ub = (uint64_t)__double_as_longlong(b);
    const auto lo = __builtin_amdgcn_permlane16_swap((uint32_t)ua, (uint32_t)ub, false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap((uint32_t)(ua >> 32), (uint32_t)(ub >> 32), false, false);
    first = words_to_f64(lo[0], hi[0]);
    second = words_to_f64(lo[1], hi[1]);
}

template <int DIST>
__device__ __forceinline__ float lane_xor_val(float x, uint32_t lane)
{
    return __uint_as_float(lane_xor<DIST>(__float_as_uint(x), lane));
}

template <int DIST>
__device__ __forceinline__ double lane_xor_val(double x, uint32_t lane)
{
    const uint64_t u = (uint64_t)__double_as_longlong(x);
    return words_to_f64(lane_xor<DIST>((uint32_t)u, lane), lane_xor<DIST>((uint32_t)(u >> 32), lane));
}

template <int CTRL>
__device__ __forceinline__ float dpp_val(float x) { return dpp_f32<CTRL>(x); }
template <int CTRL>
__device__ __forceinline__ double dpp_val(double x) { return dpp_f64<CTRL>(x); }

// One reduction step over lane bit DIST (8, 4 or 2): lanes with the bit clear get a (+) a of the
// partner lane, the others b (+) b of the partner lane.
template <int DIST, class T, class Op>
__device__ __forceinline__ T fold_pair(T a, T b, uint32_t lane, Op op)
{
    const bool odd = (lane & (uint32_t)DIST) != 0;
    const T keep = odd ? b : a, send = odd ? a : b;
    return op(keep, lane_xor_val<DIST>(send, lane));
}

template <int Q>
struct BucketIndex {
    static constexpr int value = Q;
};

// Buckets FIRST .. FIRST + N - 1 of the wavefront, reduced depth first so that only one partial result
// per tree level is alive: leaf(BucketIndex<q>) yields this lane's partial value of bucket q.
template <int N, int FIRST, class T, class Leaf, class Op>
__device__ __forceinline__ T reduce_bucket_tree(uint32_t lane, Leaf& leaf, Op op)
{
    if constexpr (N == 1) {
        return leaf(BucketIndex<FIRST>{});
    } else {
        const T a = reduce_bucket_tree<N / 2, FIRST, T>(lane, leaf, op);
        const T b = reduce_bucket_tree<N / 2, FIRST + N / 2, T>(lane, leaf, op);
        if constexpr (N == 2) {
            T first, second;
            swap_halves(a, b, first, second);
            return op(first, second);
        } else if constexpr (N == 4) {
            T first, second;
            swap_rows(a, b, first, second);
            return op(first, second);
        } else if constexpr (N == 8) {
            return fold_pair<8>(a, b, lane, op);
        } else if constexpr (N == 16) {
            return fold_pair<4>(a, b, lane, op);
        } else {
            return fold_pair<2>(a, b, lane, op);
        }
    }
}

template <int NB, class T, class Leaf, class Op>
__device__ __forceinline__ T reduce_buckets(uint32_t lane, Leaf leaf, Op op)
{
    static_assert(NB == 2 || NB == 4 || NB == 8 || NB == 16 || NB == 32, "buckets per wavefront");
    T r = reduce_bucket_tree<NB, 0, T>(lane, leaf, op);
    // the lane bits that select no bucket
    r = op(r, dpp_val<kDppXor1>(r));
    if constexpr (NB <= 16) r = op(r, dpp_val<kDppXor2>(r));
    if constexpr (NB <= 8) r = op(r, dpp_val<kDppHalfMirror>(r));
    if constexpr (NB <= 4) r = op(r, dpp_val<kDppMirror>(r));
    if constexpr (NB <= 2) {
        T first, second;
        swap_rows(r, r, first, second);
        r = op(first, second);
    }
    return r;
}

constexpr uint32_t reverse6(uint32_t x)
{
    uint32_t r = 0;
    for (int b = 0; b < 6; ++b) r |= ((x >> b) & 1u) << (5 - b);
    return r;
}

constexpr uint32_t kChunk = 2048;  // elements one wavefront of the kernel below quantizes
constexpr uint32_t kMinChunks = 2048;

template <int NB, bool SIGN>
__global__ __launch_bounds__(kWave* kBinGradWaves) __attribute__((amdgpu_waves_per_eu(4, 4))) void bingrad_chunk_kernel(
    const float* __restrict__ grad, uint32_t num_chunks, uint32_t iters, float* __restrict__ levels,
    uint64_t* __restrict__ codes)
{
    constexpr int R = kChunk / 64, E = R / NB;
    constexpr uint32_t D = 64u * E;             // bucket size
    constexpr uint32_t kFreeBits = 64u / NB - 1u;  // lane bits that select no bucket; bit 0 is always among them
    const uint32_t chunk = uniform_u32(blockIdx.x * kBinGradWaves + (threadIdx.x >> 6));
    if (chunk >= num_chunks) return;
    const uint32_t lane = threadIdx.x & 63u;
    const float* g = grad + (size_t)chunk * kChunk;
    float v[R];
#pragma unroll
    for (int j = 0; j < R; ++j) v[j] = __builtin_nontemporal_load(g + 64u * j + lane);

    const auto add = [](double a, double b) { return a + b; };
    const auto larger = [](float a, float b) { return fmaxf(a, b); };
    // From here on lane l works for bucket q(l); the lane with the free bits clear ("home") and the one
    // above it divide the lower and the upper side of that bucket.
    const double total = reduce_buckets<NB, double>(
        lane,
        [&](auto q) {
            double s = 0.0;
#pragma unroll
            for (int j = 0; j < E; ++j) {
                const float x = v[decltype(q)::value * E + j];
                s += (double)(SIGN ? fabsf(x) : x);
            }
            return s;
        },
        add);
    const float trust_above = 1e-3f * reduce_buckets<NB, float>(  // see bingrad_bucket
                                          lane,
                                          [&](auto q) {
                                              float m = 0.0f;
#pragma unroll
                                              for (int j = 0; j < E; ++j) m = fmaxf(m, fabsf(v[decltype(q)::value * E + j]));
                                              return m;
                                          },
                                          larger);
    float b0 = (float)(total / (double)D);
    const bool upper = (lane & 1u) != 0;
    const bool home = (lane & kFreeBits) == 0;

    double b_lo = 0.0, b_hi = 0.0;
    uint32_t word_lo = 0, word_hi = 0;  // lane j ends up holding packed word j of the chunk
    uint32_t prev_n_lo = 0xFFFFFFFFu;
    if constexpr (SIGN) {  // Scaled SignSGD: see bingrad_bucket
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint64_t hi_mask = ~__ballot(v[j] < 0.0f);
            word_lo = writelane(word_lo, (uint32_t)hi_mask, j);
            word_hi = writelane(word_hi, (uint32_t)(hi_mask >> 32), j);
        }
        b_hi = total / (double)D;
        b_lo = -b_hi;
    } else
    for (uint32_t it = 0;; ++it) {
        uint32_t n_lo = 0;
        const double s_lo = reduce_buckets<NB, double>(
            lane,
            [&](auto q) {
                constexpr int kQ = decltype(q)::value;
                const float threshold = readlane_f32(b0, (int)reverse6(kQ));
                double s = 0.0;
                uint32_t below = 0;
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    const int reg = kQ * E + j;
                    const bool lo = v[reg] < threshold;
                    const uint64_t lo_mask = __ballot(lo);
                    const uint64_t hi_mask = ~lo_mask;
                    below += (uint32_t)__popcll(lo_mask);
                    s += (double)(lo ? v[reg] : 0.0f);
                    word_lo = writelane(word_lo, (uint32_t)hi_mask, reg);
                    word_hi = writelane(word_hi, (uint32_t)(hi_mask >> 32), reg);
                }
                n_lo = writelane(n_lo, below, (int)reverse6(kQ));
                return s;
            },
            add);
        n_lo = dpp_u32<kDppXor1From0>(n_lo);
        double s_hi = total - s_lo;
        const bool doubtful = !(fabs(s_hi) >= (double)trust_above);
        if (__ballot(doubtful) != 0) {
            const double direct = reduce_buckets<NB, double>(
                lane,
                [&](auto q) {
                    constexpr int kQ = decltype(q)::value;
                    const float threshold = readlane_f32(b0, (int)reverse6(kQ));
                    double s = 0.0;
#pragma unroll
                    for (int j = 0; j < E; ++j) s += (double)(!(v[kQ * E + j] < threshold) ? v[kQ * E + j] : 0.0f);
                    return s;
                },
                add);
            if (doubtful) s_hi = direct;
        }
        const uint32_t n_hi = D - n_lo;
        const double num = upper ? s_hi : s_lo;
        const uint32_t den = upper ? n_hi : n_lo;
        const double quot = num / (double)(den > 0 ? den : 1u);
        const double other = dpp_f64<kDppXor1>(quot);
        const double mean_lo = upper ? other : quot, mean_hi = upper ? quot : other;
        b_lo = n_lo > 0 ? mean_lo : mean_hi;  // constant bucket: both levels equal
        b_hi = n_hi > 0 ? mean_hi : mean_lo;
        // Further threshold updates are identities for a bucket once its partition repeats.
        if (it == iters || __ballot(home && n_lo != prev_n_lo) == 0) break;
        prev_n_lo = n_lo;
        b0 = (float)((b_lo + b_hi) * 0.5);
    }

    if (home) {
        const uint32_t q = (__brev(lane) >> 26) & (uint32_t)(NB - 1);
        float2 pair;
        pair.x = (float)b_lo;
        pair.y = (float)b_hi;
        *reinterpret_cast<float2*>(levels + ((size_t)chunk * NB + q) * 2) = pair;
    }
    if (lane < (uint32_t)R) codes[(size_t)chunk * R + lane] = ((uint64_t)word_hi << 32) | word_lo;
}

// ----------------------------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------------------------
template <int E>
void launch_bingrad(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                    hipStream_t st)
{
    const dim3 grid((nb + kBinGradWaves - 1) / kBinGradWaves), block(kWave * kBinGradWaves);
    const bool clip = p->clip_factor > 0.0f, sign = p->scheme == OGQ_SCALED_SIGN;
#define OGQ_LAUNCH(CLIP, SIGN)                                                                                        \
    launch_kernel((bingrad_quantize_kernel<E, CLIP, SIGN>), grid, block, st, g, n, p->bucket_size,           \
                       p->level_iters, p->clip_factor, nb, lv, static_cast<uint64_t*>(codes))
    if (sign) {
        if (clip) OGQ_LAUNCH(true, true);
        else OGQ_LAUNCH(false, true);
    } else {
        if (clip) OGQ_LAUNCH(true, false);
        else OGQ_LAUNCH(false, false);
    }
#undef OGQ_LAUNCH
}

template <int W, int E = 32>
void launch_bingrad_team(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                         hipStream_t st)
{
    const dim3 grid(nb), block(W * kWave);
    const bool clip = p->clip_factor > 0.0f, sign = p->scheme == OGQ_SCALED_SIGN;
#define OGQ_LAUNCH(CLIP, SIGN)                                                                               \
    launch_kernel((bingrad_team_kernel<W, E, CLIP, SIGN>), grid, block, st, g, n, p->bucket_size,   \
                       p->level_iters, p->clip_factor, nb, lv, static_cast<uint64_t*>(codes))
    if constexpr (E <= 32) {  // 64 registers of data leave no room for the clipping passes: the caller picks E = 32
        if (clip) {
            if (sign) OGQ_LAUNCH(true, true);
            else OGQ_LAUNCH(true, false);
            return;
        }
    }
    if (sign) OGQ_LAUNCH(false, true);
    else OGQ_LAUNCH(false, false);
#undef OGQ_LAUNCH
}

template <int NB>
void launch_bingrad_chunks_of(const float* g, uint32_t chunks, const ogq_params_t* p, float* lv, uint64_t* words,
                              hipStream_t st)
{
    const dim3 grid((chunks + kBinGradWaves - 1) / kBinGradWaves), block(kWave * kBinGradWaves);
    if (p->scheme == OGQ_SCALED_SIGN)
        launch_kernel((bingrad_chunk_kernel<NB, true>), grid, block, st, g, chunks, p->level_iters, lv, words);
    else
        launch_kernel((bingrad_chunk_kernel<NB, false>), grid, block, st, g, chunks, p->level_iters, lv, words);
}

void launch_bingrad_chunks(const float* g, uint32_t chunks, const ogq_params_t* p, float* lv, void* codes, hipStream_t st)
{
    uint64_t* words = static_cast<uint64_t*>(codes);
    switch (kChunk / p->bucket_size) {
        case 2: launch_bingrad_chunks_of<2>(g, chunks, p, lv, words, st); break;
        case 4: launch_bingrad_chunks_of<4>(g, chunks, p, lv, words, st); break;
        case 8: launch_bingrad_chunks_of<8>(g, chunks, p, lv, words, st); break;
        case 16: launch_bingrad_chunks_of<16>(g, chunks, p, lv, words, st); break;
        default: launch_bingrad_chunks_of<32>(g, chunks, p, lv, words, st); break;
    }
}

void launch_two_level(const float* g, size_t n, const ogq_params_t* p, float* lv, void* codes, hipStream_t st)
{
    const uint32_t d = p->bucket_size;
    // Whole chunks of 2048 elements go to the kernel that packs several buckets into a wavefront; what
    // is left (fewer than 2048 elements) takes the one-bucket-per-wavefront kernel below.  Buckets of
    // 512 and 1024 elements stay with that kernel for gradients too short to give every SIMD a chunk
    // or two (it was the faster one below about four million elements).
    const size_t chunks = n / kChunk;
    if (p->clip_factor == 0.0f && d <= kChunk / 2 && kChunk % d == 0 && chunks > 0 &&
        (d <= 256 || chunks >= kMinChunks)) {
        launch_bingrad_chunks(g, (uint32_t)chunks, p, lv, codes, st);
        const size_t done = chunks * kChunk;
        if (done == n) return;
        g += done;
        lv += done / d * 2;
        codes = static_cast<uint64_t*>(codes) + done / 64;
        n -= done;
    }
    const uint32_t nb = (uint32_t)(n / d + (n % d != 0));
    const uint32_t regs = d / 64;
    if (regs <= 1) launch_bingrad<1>(g, n, p, nb, lv, codes, st);
    else if (regs <= 2) launch_bingrad<2>(g, n, p, nb, lv, codes, st);
    else if (regs <= 4) launch_bingrad<4>(g, n, p, nb, lv, codes, st);
    else if (regs <= 8) launch_bingrad<8>(g, n, p, nb, lv, codes, st);
    else if (regs <= 16) launch_bingrad<16>(g, n, p, nb, lv, codes, st);
    else if (regs <= 32) launch_bingrad<32>(g, n, p, nb, lv, codes, st);
    else if (regs <= 64) launch_bingrad_team<2>(g, n, p, nb, lv, codes, st);
    else if (regs <= 128) launch_bingrad_team<4>(g, n, p, nb, lv, codes, st);
    else if (p->clip_factor > 0.0f) {
        // the clipping passes need the registers a second 2048 elements per wavefront would take
        if (regs <= 256) launch_bingrad_team<8>(g, n, p, nb, lv, codes, st);
        else launch_bingrad_team<16>(g, n, p, nb, lv, codes, st);
    } else if (regs <= 256) launch_bingrad_team<4, 64>(g, n, p, nb, lv, codes, st);
    else launch_bingrad_team<8, 64>(g, n, p, nb, lv, codes, st);
}

}  // namespace ogq
