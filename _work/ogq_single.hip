// libogq: per-bucket optimal gradient quantization for MI355X (gfx950, wave64).
//
// Method: "Optimal Gradient Quantization Condition for Communication-Efficient Distributed
// Training" (arXiv 2002.11082).  One wavefront owns one bucket from the HBM load to the packed
// store, so the gradient is read exactly once:
//   BinGrad-b (Section 3.2): fp64 wave reductions for the mean and the two conditional means,
//     the code bit of 64 consecutive elements is the ballot of (v >= b0).
//   ORQ (Theorem 1, its discrete remark, Corollary 1, Algorithm 1; random rounding of
//     Section 3.1): every level solve is a range sum plus an exact rank selection over the
//     register-resident bucket; Philox4x32-10 draws keyed by (seed, global element index).
//   Decode-average (server step of Algorithm 2): the packed 64-bit words are used directly as
//     lane masks of v_cndmask selects over the bucket's level table.
//
// Compile with -ffp-contract=off: the rounding decision of ORQ is specified op by op in fp32.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ogq.h"

namespace {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWave * kWavesPerBlock;

thread_local int g_last_hip_error = 0;

// ----------------------------------------------------------------------------------------------
// wave-level helpers
// ----------------------------------------------------------------------------------------------
// Cross-lane moves within a row of 16 lanes (DPP): quad_perm [1,0,3,2], quad_perm [2,3,0,1],
// row_half_mirror, row_mirror.  After the four steps of a butterfly every lane of a row holds the
// row's result; the four rows are then combined through readlane.
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x)
{
    return __uint_as_float(dpp_u32<CTRL>(__float_as_uint(x)));
}

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x)
{
    const uint64_t u = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = dpp_u32<CTRL>((uint32_t)u), hi = dpp_u32<CTRL>((uint32_t)(u >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

__device__ __forceinline__ double readlane_f64(double x, int lane)
{
    const uint64_t u = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)u, lane);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(u >> 32), lane);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

__device__ __forceinline__ float readlane_f32(float x, int lane)
{
    return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x), lane));
}

// v_writelane_b32 through the compiler's own intrinsic (the compiler then inserts the wait states the
// instruction needs after a VALU write of its scalar source; hand-written asm would not get them).
extern "C" __device__ uint32_t ogq_llvm_writelane(uint32_t value, uint32_t lane, uint32_t old) __asm("llvm.amdgcn.writelane.i32");

// Lane `lane` of `dst` takes the wave-uniform value `value`; the other lanes keep theirs.
__device__ __forceinline__ uint32_t writelane(uint32_t dst, uint32_t value, int lane)
{
    return ogq_llvm_writelane(value, (uint32_t)lane, dst);
}

// Wave-wide sum; the result is wave-uniform.
__device__ __forceinline__ double wave_sum(double x)
{
    x += dpp_f64<kDppXor1>(x);
    x += dpp_f64<kDppXor2>(x);
    x += dpp_f64<kDppHalfMirror>(x);
    x += dpp_f64<kDppMirror>(x);
    return (readlane_f64(x, 0) + readlane_f64(x, 16)) + (readlane_f64(x, 32) + readlane_f64(x, 48));
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x)
{
    x += dpp_u32<kDppXor1>(x);
    x += dpp_u32<kDppXor2>(x);
    x += dpp_u32<kDppHalfMirror>(x);
    x += dpp_u32<kDppMirror>(x);
    return (__builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16)) +
           (__builtin_amdgcn_readlane(x, 32) + __builtin_amdgcn_readlane(x, 48));
}

__device__ __forceinline__ float wave_min(float x)
{
    x = fminf(x, dpp_f32<kDppXor1>(x));
    x = fminf(x, dpp_f32<kDppXor2>(x));
    x = fminf(x, dpp_f32<kDppHalfMirror>(x));
    x = fminf(x, dpp_f32<kDppMirror>(x));
    return fminf(fminf(readlane_f32(x, 0), readlane_f32(x, 16)), fminf(readlane_f32(x, 32), readlane_f32(x, 48)));
}

__device__ __forceinline__ float wave_max(float x)
{
    x = fmaxf(x, dpp_f32<kDppXor1>(x));
    x = fmaxf(x, dpp_f32<kDppXor2>(x));
    x = fmaxf(x, dpp_f32<kDppHalfMirror>(x));
    x = fmaxf(x, dpp_f32<kDppMirror>(x));
    return fmaxf(fmaxf(readlane_f32(x, 0), readlane_f32(x, 16)), fmaxf(readlane_f32(x, 32), readlane_f32(x, 48)));
}

constexpr int kDppRor8 = 0x128;   // rotate by 8 inside a row of 16 lanes: partner lane ^ 8
constexpr int kDppRowShl4 = 0x104;  // lane i takes lane i + 4 of its row
constexpr int kDppRowShr4 = 0x114;  // lane i takes lane i - 4 of its row

// Value held by lane (lane ^ DIST).
template <int DIST>
__device__ __forceinline__ uint32_t lane_xor(uint32_t x, uint32_t lane)
{
    if constexpr (DIST == 1) {
        return dpp_u32<kDppXor1>(x);
    } else if constexpr (DIST == 2) {
        return dpp_u32<kDppXor2>(x);
    } else if constexpr (DIST == 4) {
        // banks (groups of 4 lanes) 0 and 2 of every row take the lane 4 above, banks 1 and 3 the lane 4 below
        int y = __builtin_amdgcn_update_dpp((int)x, (int)x, kDppRowShl4, 0xF, 0x5, false);
        y = __builtin_amdgcn_update_dpp(y, (int)x, kDppRowShr4, 0xF, 0xA, false);
        return (uint32_t)y;
    } else if constexpr (DIST == 8) {
        return dpp_u32<kDppRor8>(x);
    } else if constexpr (DIST == 16) {
        // rows (0,1) and (2,3) trade places
        const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        return (lane & 16u) ? r[0] : r[1];
    } else {
        // the two halves of the wave trade places
        const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
        return (lane & 32u) ? r[0] : r[1];
    }
}

// Gradient clipping of a register-resident bucket (Section 5): v <- sign(v) * min(|v|, c * sigma) with
// sigma^2 the population variance about the bucket mean, both in fp64.  valid(j) tells whether
// register j of this lane holds a bucket element; bucket_sum(x) adds x over all lanes that hold the bucket.
template <int N, class ValidFn, class SumFn>
__device__ __forceinline__ void clip_in_registers(float (&v)[N], uint32_t len, float c, ValidFn valid, SumFn bucket_sum)
{
    double part = 0.0;
#pragma unroll
    for (int j = 0; j < N; ++j) part += valid(j) ? (double)v[j] : 0.0;
    const double mean = bucket_sum(part) / (double)len;
    part = 0.0;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const double dv = (double)v[j] - mean;
        part += valid(j) ? dv * dv : 0.0;
    }
    const double sigma = sqrt(bucket_sum(part) / (double)len);
    const float limit = (float)((double)c * sigma);
#pragma unroll
    for (int j = 0; j < N; ++j) v[j] = fminf(fmaxf(v[j], -limit), limit);
}

template <int N, class ValidFn>
__device__ __forceinline__ void clip_in_registers(float (&v)[N], uint32_t len, float c, ValidFn valid)
{
    clip_in_registers<N>(v, len, c, valid, [](double x) { return wave_sum(x); });
}

__device__ __forceinline__ uint32_t uniform_u32(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }

__device__ __forceinline__ float uniform_f32(float x)
{
    return __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(x)));
}

__device__ __forceinline__ double uniform_f64(double x)
{
    uint64_t u = (uint64_t)__double_as_longlong(x);
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
    uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// ----------------------------------------------------------------------------------------------
// BinGrad-b quantize.  Lane l register j holds bucket element 64*j + l, so a ballot over
// register j is the packed code word j of the bucket.  A bucket is held by one wavefront, or by the
// two wavefronts of a workgroup (elements 0..2047 and 2048..4095): the Team types say how a
// wave-wide result becomes a bucket-wide one.
// ----------------------------------------------------------------------------------------------
struct OneWave {
    __device__ __forceinline__ double sum(double x) { return x; }
    __device__ __forceinline__ void sum_and_max(double&, float&) {}
    __device__ __forceinline__ void sum_and_count(double&, uint32_t&) {}
};

// All wavefronts of the team call every combine in the same order (their control flow depends on combined
// values only).  Two alternating LDS slots are enough: a wavefront that writes a slot for the second time has
// passed the barrier in between, which the others reach only after they have read the first value.
struct TeamSlot {
    double sum;
    uint32_t a, b;
};

template <int W>
struct WaveTeam {
    TeamSlot (*slots)[W];  // [2][W] in LDS: [call parity][wavefront]
    uint32_t wave;
    uint32_t calls;
    __device__ __forceinline__ const TeamSlot* exchange(double sum, uint32_t a, uint32_t b)
    {
        TeamSlot* slot = slots[calls & 1u];
        ++calls;
        if ((threadIdx.x & 63u) == 0) {
            slot[wave].sum = sum;
            slot[wave].a = a;
            slot[wave].b = b;
        }
        __syncthreads();
        return slot;
    }
    __device__ __forceinline__ double sum(double x)
    {
        const TeamSlot* s = exchange(x, 0u, 0u);
        double r = s[0].sum;
#pragma unroll
        for (int w = 1; w < W; ++w) r += s[w].sum;
        return r;
    }
    __device__ __forceinline__ void sum_and_max(double& x, float& m)
    {
        const TeamSlot* s = exchange(x, __float_as_uint(m), 0u);
        x = s[0].sum;
        m = __uint_as_float(s[0].a);
#pragma unroll
        for (int w = 1; w < W; ++w) {
            x += s[w].sum;
            m = fmaxf(m, __uint_as_float(s[w].a));
        }
    }
    __device__ __forceinline__ void sum_and_count(double& x, uint32_t& c)
    {
        const TeamSlot* s = exchange(x, c, 0u);
        x = s[0].sum;
        c = s[0].a;
#pragma unroll
        for (int w = 1; w < W; ++w) {
            x += s[w].sum;
            c += s[w].a;
        }
    }
};

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
    // The upper sum is taken as total - lower sum.  Both are fp64 sums of at most 4096 fp32 values
    // (error below 2^-53 * n^2 * max|v| each, and exact for any bucket whose values span fewer than
    // ~18 binades), so the difference is trusted unless it is tiny against the largest element; such
    // a bucket sums its upper side directly.
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
            const bool lo = valid && (v[j] < b0);
            const uint64_t lo_mask = __ballot(lo);
            const uint64_t hi_mask = FULL ? ~lo_mask : __ballot(valid && !lo);
            below += lo ? 1u : 0u;
            s_lo += (double)(lo ? v[j] : 0.0f);
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

// Buckets of more than 2048 elements: the W = 2, 4, 8 or 16 wavefronts of a workgroup hold one bucket, 32
// registers per lane each as for a 2048-element bucket, and combine their sums and counts through LDS.
template <int W, bool CLIP, bool SIGN>
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
    if (len == 2048u * W) bingrad_bucket<32, true, CLIP, SIGN>(team, 2048u * wave, g, len, iters, clip, lv, w);
    else bingrad_bucket<32, false, CLIP, SIGN>(team, 2048u * wave, g, len, iters, clip, lv, w);
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
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter (c0, c1, 0, 0), key (k0, k1).
// ----------------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1, uint32_t (&r)[4])
{
    uint32_t c2 = 0, c3 = 0;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t pa = (uint64_t)0xD2511F53u * c0;
        const uint64_t pb = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    r[0] = c0; r[1] = c1; r[2] = c2; r[3] = c3;
}

// ----------------------------------------------------------------------------------------------
// ORQ quantize.  One wavefront (= one workgroup) owns one bucket.  Lane l holds, for chunk c, the
// four consecutive bucket elements 256*c + 4*l + {0,1,2,3} (one 16-byte load), which are also the
// four elements that share one Philox block.
//
// A level solve needs (a) counts and sums of the elements below a level and (b) the element of a
// given rank.  The bucket is therefore grouped once, in LDS, by a monotone bin of the value (sign,
// exponent and top mantissa bits, relative to the largest magnitude of the bucket; everything more
// than 16 binades below that shares the two centre bins).  Per-bin counts and fp64 sums are
// prefix-summed; after that a solve touches one bin: the bin holding the wanted rank is sorted
// across the 64 lanes, and the counts and sums below the chosen element are added to the bin's
// prefix.  All values of a regular bin share sign and exponent, so its fp64 sum is exact.
// ----------------------------------------------------------------------------------------------
// Order-preserving map of fp32 onto unsigned integers.
__device__ __forceinline__ uint32_t float_to_key(float f)
{
    const uint32_t u = __float_as_uint(f);
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}

__device__ __forceinline__ float key_to_float(uint32_t k)
{
    const uint32_t u = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
    return __uint_as_float(u);
}

// Order of the greedy solves (Algorithm 1): the level in the middle of [l, r] is solved from the
// two outer levels, then both halves are treated the same way; the middle index is rounded down
// when s is not of the form 2^K + 1.  Each step is packed as 4 bits of k, l, r; five steps per word.
struct GreedyOrder {
    uint64_t packed[2];
    int count;
};

constexpr void greedy_visit(GreedyOrder& o, int l, int r)
{
    if (r - l < 2) return;
    const int mid = (l + r) / 2;
    o.packed[o.count / 5] |= (uint64_t)(mid | (l << 4) | (r << 8)) << (12 * (o.count % 5));
    ++o.count;
    greedy_visit(o, l, mid);
    greedy_visit(o, mid, r);
}

template <int S>
constexpr GreedyOrder greedy_order()
{
    GreedyOrder o{{0, 0}, 0};
    greedy_visit(o, 0, S - 1);
    return o;
}

// LDS of one bucket: D = element capacity, B = number of bins.
template <int D_, int B_>
struct OrqLds {
    static constexpr int D = D_, B = B_;
    // fp32 bit patterns (-0 stored as +0) grouped by bin, unsorted inside a bin.  Position i lives at
    // word i + i/32, so that the 64 lanes reading consecutive blocks of D/64 positions hit distinct banks.
    uint32_t grouped[D + D / 32];
    uint32_t bin_start[B + 4];  // histogram, then first position of each bin; [B] = bucket length
    double block_prefix[64];    // fp64 sum of all positions before block l (block = D/64 positions)
    // per level k: value; #{v < value}; #{v <= value}; sum{v < value}; sum{v <= value}; the rank it
    // was picked at (0 = not picked by rank)
    double lvl_sum_lt[10];
    double lvl_sum_le[10];
    float lvl_value[10];
    uint32_t lvl_count_lt[10];
    uint32_t lvl_count_le[10];
    uint32_t lvl_rank[10];
};

__device__ __forceinline__ uint32_t skewed(uint32_t position) { return position + (position >> 5); }

__device__ __forceinline__ uint32_t umin32(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint32_t umax32(uint32_t a, uint32_t b) { return a > b ? a : b; }

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x)
{
    x = umax32(x, dpp_u32<kDppXor1>(x));
    x = umax32(x, dpp_u32<kDppXor2>(x));
    x = umax32(x, dpp_u32<kDppHalfMirror>(x));
    x = umax32(x, dpp_u32<kDppMirror>(x));
    return umax32(umax32(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
                  umax32(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) { return ~wave_max_u32(~x); }

// Inclusive scans over the lanes in ascending lane order.
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t x, uint32_t lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t y = (uint32_t)__shfl_up((int)x, off, kWave);
        x += (lane >= (uint32_t)off) ? y : 0u;
    }
    return x;
}

__device__ __forceinline__ double wave_inclusive_scan_f64(double x, uint32_t lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double y = __shfl_up(x, off, kWave);
        x += (lane >= (uint32_t)off) ? y : 0.0;
    }
    return x;
}

// Ascending bitonic sort of one key per lane across the 64 lanes.
template <int K, int DIST>
__device__ __forceinline__ uint32_t bitonic_step(uint32_t x, uint32_t lane)
{
    const uint32_t y = lane_xor<DIST>(x, lane);
    const bool ascending = (lane & (uint32_t)K) == 0;
    const bool lower = (lane & (uint32_t)DIST) == 0;
    const uint32_t mn = umin32(x, y), mx = umax32(x, y);
    return (ascending == lower) ? mn : mx;
}

__device__ __forceinline__ uint32_t wave_sort_u32(uint32_t x, uint32_t lane)
{
    x = bitonic_step<2, 1>(x, lane);
    x = bitonic_step<4, 2>(x, lane);   x = bitonic_step<4, 1>(x, lane);
    x = bitonic_step<8, 4>(x, lane);   x = bitonic_step<8, 2>(x, lane);   x = bitonic_step<8, 1>(x, lane);
    x = bitonic_step<16, 8>(x, lane);  x = bitonic_step<16, 4>(x, lane);  x = bitonic_step<16, 2>(x, lane);
    x = bitonic_step<16, 1>(x, lane);
    x = bitonic_step<32, 16>(x, lane); x = bitonic_step<32, 8>(x, lane);  x = bitonic_step<32, 4>(x, lane);
    x = bitonic_step<32, 2>(x, lane);  x = bitonic_step<32, 1>(x, lane);
    x = bitonic_step<64, 32>(x, lane); x = bitonic_step<64, 16>(x, lane); x = bitonic_step<64, 8>(x, lane);
    x = bitonic_step<64, 4>(x, lane);  x = bitonic_step<64, 2>(x, lane);  x = bitonic_step<64, 1>(x, lane);
    return x;
}

// The bucket element of a given rank, with the counts and sums of the bucket elements strictly
// below it and not above it.
struct Picked {
    uint32_t key;
    uint32_t count_lt, count_le;
    double sum_lt, sum_le;
};

// The element of 1-based rank `rank`, which lies in bin `bin`.  BLOCK = positions per entry of the fp64
// block prefix (at most 64).
template <int BLOCK, class Lds>
__device__ __forceinline__ Picked pick_in_bin(const Lds& lds, uint32_t bin, uint32_t rank, uint32_t lane)
{
    static_assert(BLOCK <= 64, "the head of a block is read one position per lane");
    const uint32_t first = uniform_u32(lds.bin_start[bin]);
    const uint32_t count = uniform_u32(lds.bin_start[bin + 1]) - first;
    const uint32_t r_in = rank - first;  // 1-based rank inside the bin

    // sum of everything before the bin = prefix of its block + the block's positions before `first`
    const uint32_t block = first / BLOCK;
    const uint32_t block_first = block * BLOCK;
    const double before_block = uniform_f64(lds.block_prefix[block]);
    const float head = lane < first - block_first ? __uint_as_float(lds.grouped[skewed(block_first + lane)]) : 0.0f;

    uint32_t key, c_lt, c_le;
    double s_lt;
    if (count <= 64u) {
        const uint32_t mine =
            lane < count ? float_to_key(__uint_as_float(lds.grouped[skewed(first + lane)])) : 0xFFFFFFFFu;
        const uint32_t sorted = wave_sort_u32(mine, lane);
        key = __builtin_amdgcn_readlane(sorted, r_in - 1u);
        const bool lt = sorted < key;
        const bool le = (sorted <= key) && (lane < count);
        c_lt = (uint32_t)__popcll(__ballot(lt));
        c_le = (uint32_t)__popcll(__ballot(le));
        s_lt = wave_sum((double)head + (lt ? (double)key_to_float(sorted) : 0.0));
    } else {
        // a crowded bin (many equal or nearly equal values): bisection on the key over all its chunks
        uint32_t prefix = 0;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t cand = prefix | (1u << bit);
            uint32_t below = 0;
            for (uint32_t base = 0; base < count; base += 64u) {
                const uint32_t i = base + lane;
                const uint32_t k = i < count ? float_to_key(__uint_as_float(lds.grouped[skewed(first + i)])) : 0xFFFFFFFFu;
                below += (uint32_t)__popcll(__ballot(k < cand));
            }
            if (below < r_in) prefix = cand;
        }
        key = prefix;
        c_lt = 0;
        c_le = 0;
        double part = (double)head;
        for (uint32_t base = 0; base < count; base += 64u) {
            const uint32_t i = base + lane;
            const float x = i < count ? __uint_as_float(lds.grouped[skewed(first + i)]) : 0.0f;
            const uint32_t k = i < count ? float_to_key(x) : 0xFFFFFFFFu;
            const bool lt = k < key;
            c_lt += (uint32_t)__popcll(__ballot(lt));
            c_le += (uint32_t)__popcll(__ballot(k <= key && i < count));
            part += lt ? (double)x : 0.0;
        }
        s_lt = wave_sum(part);
    }
    Picked p;
    p.key = key;
    p.count_lt = first + c_lt;
    p.count_le = first + c_le;
    p.sum_lt = before_block + s_lt;
    p.sum_le = p.sum_lt + (double)(c_le - c_lt) * (double)key_to_float(key);
    return p;
}

// rank is 1-based, 1 <= rank <= bucket length.  my_start[t] = bin_start[lane * PER + t], kept in registers.
template <int D, int B>
__device__ __forceinline__ Picked pick_rank(const OrqLds<D, B>& lds, const uint32_t (&my_start)[B / 64],
                                            uint32_t rank, uint32_t lane)
{
    constexpr int PER = B / 64;
    // the bin holding the rank: the last bin whose first position is below the rank
    uint32_t starts_below = 0;
#pragma unroll
    for (int t = 0; t < PER; ++t) starts_below += (my_start[t] < rank) ? 1u : 0u;
    const uint32_t bin = wave_sum_u32(starts_below) - 1u;  // bin_start[0] = 0 < rank: at least one
    return pick_in_bin<D / 64>(lds, bin, rank, lane);
}

// The same with the bin found by two looks into LDS (every (B/64)-th bin start, then the B/64 bins in between):
// no registers are tied up by the bin starts.
template <class Lds>
__device__ __forceinline__ Picked pick_rank_by_lookup(const Lds& lds, uint32_t rank, uint32_t lane)
{
    constexpr uint32_t PER = Lds::B / 64;
    static_assert(PER <= 64, "one lane per bin of a segment");
    const uint32_t segment = (uint32_t)__popcll(__ballot(lds.bin_start[lane * PER] < rank)) - 1u;
    const bool below = lane < PER && lds.bin_start[segment * PER + (lane < PER ? lane : 0u)] < rank;
    const uint32_t bin = segment * PER + (uint32_t)__popcll(__ballot(below)) - 1u;
    return pick_in_bin<64>(lds, bin, rank, lane);
}

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Returns x unchanged but hides it from common-subexpression elimination, so that values derived
// from the register-resident bucket are recomputed in each phase instead of being kept alive.
__device__ __forceinline__ float recompute_from(float x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// ---- encode (random rounding, Section 3.1) + pack ------------------------------------------------
// v: the 256*C elements a wavefront holds (lane l, chunk c: elements 256c + 4l + {0..3} of the range that
// starts at global element `begin` and has `len` valid elements; FULL: len == 256*C); lv: the levels.
template <int C, int S, int BITS, bool FULL>
__device__ __forceinline__ void orq_encode(const float (&v)[C][4], const float (&lv)[S], uint32_t len, size_t begin,
                                           uint64_t seed, uint64_t index_offset, uint32_t* __restrict__ codes32)
{
    const uint32_t lane = threadIdx.x & 63u;
    // Per element only the level compares, the selects of (level below, interval width) and the rounding
    // test run on the vector unit; the level index is assembled from the compare masks on the scalar unit
    // (the masks are a thermometer code of the interval, to which the rounding bit is added with carry).
    float width[S - 1];
#pragma unroll
    for (int k = 0; k < S - 1; ++k) width[k] = lv[k + 1] - lv[k];
    uint32_t bit_of[4];  // where element k of this lane sits in its 32-bit half of a packed word
#pragma unroll
    for (int k = 0; k < 4; ++k) bit_of[k] = 1u << (4u * (lane & 7u) + k);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    const uint32_t padded_len = (len + 63u) & ~63u;
    const size_t word0 = begin / 64;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const uint64_t block = (index_offset + begin + 256u * c + 4u * lane) >> 2;
        uint32_t r[4];
        philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), k0, k1, r);
        uint32_t plane[BITS];
#pragma unroll
        for (int p = 0; p < BITS; ++p) plane[p] = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float x = v[c][k];
            // interval: last level not above x, at most S-2
            uint64_t not_below[S];  // [t]: lanes whose element is >= level t, t = 1 .. S-2
            float base = lv[0], w = width[0];
#pragma unroll
            for (int t = 1; t < S - 1; ++t) {
                const bool ge = lv[t] <= x;
                not_below[t] = __ballot(ge);
                base = ge ? lv[t] : base;
                w = ge ? width[t] : w;
            }
            const float delta = x - base;
            const float u = (float)(r[k] >> 8) * 0x1p-24f;
            const float scaled = u * w;
            uint64_t carry = __ballot(scaled < delta);  // rounded up
            if constexpr (!FULL) carry &= __ballot(256u * c + 4u * lane + k < len);
#pragma unroll
            for (int p = 0; p < BITS; ++p) {
                // bit p of the number of levels 1..S-2 not above x
                uint64_t index_bit = 0;
#pragma unroll
                for (int j = 1; (j << p) <= S - 2; j += 2) {
                    const int lo_t = j << p, hi_t = (j + 1) << p;
                    index_bit |= hi_t <= S - 2 ? (not_below[lo_t] & ~not_below[hi_t]) : not_below[lo_t];
                }
                if constexpr (!FULL) index_bit &= __ballot(256u * c + 4u * lane + k < len);
                const uint64_t code_bit = index_bit ^ carry;
                carry &= index_bit;
                plane[p] |= __builtin_amdgcn_inverse_ballot_w64(code_bit) ? bit_of[k] : 0u;
            }
        }
        // OR over the 8 lanes that make up one 32-bit half of a packed word
#pragma unroll
        for (int p = 0; p < BITS; ++p) {
            uint32_t x = plane[p];
            x |= dpp_u32<kDppXor1>(x);
            x |= dpp_u32<kDppXor2>(x);
            x |= dpp_u32<kDppHalfMirror>(x);
            const uint32_t first = 256u * c + 32u * (lane >> 3);  // first element of this half word
            if ((lane & 7u) == 0 && first < padded_len) {
                const size_t word = (word0 + 4u * c + (lane >> 4)) * BITS + p;
                codes32[word * 2 + ((lane >> 3) & 1u)] = x;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Where the levels come from; all rules share the random-rounding encoder.
//   kOptimal: ORQ (Theorem 1, Algorithm 1).
//   kPb: BinGrad-pb (Section 3.2): two levels -b_1, +b_1 from the scheme's optimal condition instead of the
//        bucket extremes; the encoder then clamps everything outside them.
//   kEven: QSGD-s / TernGrad (Section 3.1): S levels evenly spaced from -M to +M, M the largest magnitude.
//   kLinear: Linear-s (Section 5): the order statistics at the fractions k/(S-1) of the sorted bucket.
enum LevelRule { kOptimal = 0, kPb = 1, kEven = 2, kLinear = 3 };

// The level solves of one bucket, run by one wavefront once the bucket is grouped in LDS and the level
// records of the two ends are set.  pick(rank) returns the element of that 1-based rank (Picked); `zeros` is the
// number of zeros in the bucket (BinGrad-pb only).  Interior levels end up in lds.lvl_value; returns b_1 for
// BinGrad-pb.
template <int S, int RULE, class Lds, class PickFn>
__device__ __forceinline__ float orq_solve_levels(Lds& lds, PickFn pick, uint32_t len, uint32_t zeros, uint32_t sweeps,
                                                  uint32_t lane)
{
    constexpr bool PB = RULE == kPb;
    float pb_level = 0.0f;
    if constexpr (PB) {
        // ---- b_1: minimise |b * #{v > 0} - sum_{v >= b} v| over the positive bucket values.  The
        //      difference grows with b, so the minimiser is one of the two values around its sign
        //      change, which a bisection over the ranks of the positive values finds. -------------
                const uint32_t not_positive = uniform_u32(lds.bin_start[Lds::B / 2]) + zeros;  // negatives fill the lower bins
        const uint32_t positives = len - not_positive;
        const double total = uniform_f64(lds.lvl_sum_le[S - 1]);
        if (positives > 0u) {
            uint32_t lo = not_positive + 1u, hi = len;  // 1-based ranks; the largest value always has gap >= 0
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                const Picked p = pick(mid);
                const double gap = (double)key_to_float(p.key) * (double)positives - (total - p.sum_lt);
                if (gap >= 0.0) hi = mid;
                else lo = mid + 1u;
            }
            const Picked up = pick(lo);
            const double gap_up = (double)key_to_float(up.key) * (double)positives - (total - up.sum_lt);
            pb_level = key_to_float(up.key);
            if (up.count_lt > not_positive) {  // a smaller positive value exists: rank count_lt is the next one down
                const Picked down = pick(up.count_lt);
                const double gap_down =
                    (double)key_to_float(down.key) * (double)positives - (total - down.sum_lt);
                if (fabs(gap_down) <= fabs(gap_up)) pb_level = key_to_float(down.key);  // ties take the smaller value
            }
        }
    }

    if constexpr (RULE == kLinear) {
        for (uint32_t k = 1; k + 1 < (uint32_t)S; ++k) {
            const uint32_t rank = 1u + (uint32_t)(((uint64_t)k * (len - 1u)) / (uint32_t)(S - 1));
            const Picked p = pick(rank);
            if (lane == 0u) lds.lvl_value[k] = key_to_float(p.key);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // ---- level solves: greedy recursion (Algorithm 1), then re-solve sweeps ------------------
    if constexpr (S > 2 && RULE == kOptimal) {
    constexpr GreedyOrder order = greedy_order<S>();
    const uint32_t steps = order.count + sweeps * (S - 2);
    for (uint32_t step = 0; step < steps; ++step) {
        uint32_t k, l, r;
        if (step < (uint32_t)order.count) {
            const uint32_t e = step < 5u ? (uint32_t)(order.packed[0] >> (12 * step))
                                         : (uint32_t)(order.packed[1] >> (12 * (step - 5u)));
            k = e & 15u; l = (e >> 4) & 15u; r = (e >> 8) & 15u;
        } else {
            k = 1u + (step - order.count) % (S - 2);
            l = k - 1u; r = k + 1u;
        }
        const float L = uniform_f32(lds.lvl_value[l]);
        const float R = uniform_f32(lds.lvl_value[r]);
        const uint32_t cnt_lt_L = uniform_u32(lds.lvl_count_lt[l]);
        const uint32_t cnt_le_R = uniform_u32(lds.lvl_count_le[r]);
        const double sum_lt_L = uniform_f64(lds.lvl_sum_lt[l]);
        const double sum_le_R = uniform_f64(lds.lvl_sum_le[r]);
        bool copy_left = !(L < R);
        Picked p;
        uint32_t rank = 0;
        if (!copy_left) {
            // S = sum_{L<=v<=R} (v - L),  T = S / (R - L),  level = element of rank #{v<=R} - floor(T)
            const double Ssum = (sum_le_R - sum_lt_L) - (double)L * (double)(cnt_le_R - cnt_lt_L);
            const double T = Ssum / ((double)R - (double)L);
            double m = floor(T);
            if (!(m >= 0.0)) m = 0.0;
            rank = (m >= (double)cnt_le_R) ? 1u : cnt_le_R - (uint32_t)m;
            rank = rank < 1u ? 1u : (rank > len ? len : rank);
            if (rank == uniform_u32(lds.lvl_rank[k])) continue;  // same element as last time
            p = pick(rank);
            if (key_to_float(p.key) < L) copy_left = true;
        }
        __builtin_amdgcn_wave_barrier();
        if (lane == 0u) {
            if (copy_left) {
                // the level coincides with the left end (L == R, or rounding put it below L)
                lds.lvl_value[k] = L;
                lds.lvl_count_lt[k] = cnt_lt_L;
                lds.lvl_sum_lt[k] = sum_lt_L;
                lds.lvl_count_le[k] = (L < R) ? uniform_u32(lds.lvl_count_le[l]) : cnt_le_R;
                lds.lvl_sum_le[k] = (L < R) ? uniform_f64(lds.lvl_sum_le[l]) : sum_le_R;
                lds.lvl_rank[k] = 0u;
            } else {
                lds.lvl_value[k] = key_to_float(p.key);
                lds.lvl_count_lt[k] = p.count_lt;
                lds.lvl_count_le[k] = p.count_le;
                lds.lvl_sum_lt[k] = p.sum_lt;
                lds.lvl_sum_le[k] = p.sum_le;
                lds.lvl_rank[k] = rank;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    }
    return pb_level;
}

template <int C>
struct OrqShape {
    static constexpr int D = 256 * C;               // element capacity of the wave
    static constexpr int B = C >= 16 ? 512 : 256;   // bins
    static constexpr int SHIFT = C >= 16 ? 19 : 20; // magnitude bits dropped: keeps exponent + 4 (3) mantissa bits
};

// FULL: the bucket has exactly 256*C elements (no padding, no per-element validity tests).
// S levels per bucket, BITS bits per level index (S = 2^BITS, or 2^(BITS-1) + 1 for the paper's counts).
template <int C, int S, int BITS, bool FULL, bool CLIP, int RULE>
__device__ __forceinline__ void orq_bucket(OrqLds<OrqShape<C>::D, OrqShape<C>::B>& lds, const float* __restrict__ g,
                                           uint32_t len, size_t begin, uint32_t bucket, uint32_t sweeps, float clip,
                                           uint64_t seed, uint64_t index_offset, float* __restrict__ levels,
                                           uint32_t* __restrict__ codes32)
{
    static_assert(S >= 2 && S <= 9 && S <= (1 << BITS), "level count does not fit the index width");
    constexpr int D = OrqShape<C>::D;
    constexpr int B = OrqShape<C>::B;
    constexpr int PER = B / 64;   // bins per lane in the prefix step
    constexpr int HALF = B / 2;   // bins per sign
    constexpr int SHIFT = OrqShape<C>::SHIFT;
    constexpr bool full = FULL;
    constexpr bool PB = RULE == kPb;
    const uint32_t lane = threadIdx.x & 63u;

    // ---- load (read once: bypass the caches); padding holds +0 and is never binned or encoded ----
    float v[C][4];
    if (full) {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const floatx4 q = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + 256 * c + 4 * lane));
            v[c][0] = q.x; v[c][1] = q.y; v[c][2] = q.z; v[c][3] = q.w;
        }
    } else {
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t e = 256u * c + 4u * lane + k;
                v[c][k] = e < len ? g[e] : 0.0f;
            }
    }

    if constexpr (CLIP) {
        float(&flat)[4 * C] = reinterpret_cast<float(&)[4 * C]>(v);
        clip_in_registers<4 * C>(flat, len, clip, [&](int j) { return full || (64u * (j & ~3) + 4u * lane + (j & 3) < len); });
    }

    // ---- extremes ------------------------------------------------------------------------------
    float lane_min = __uint_as_float(0x7F800000u), lane_max = __uint_as_float(0xFF800000u);
    uint32_t lane_zeros = 0;
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool valid = full || (256u * c + 4u * lane + k < len);
            lane_min = fminf(lane_min, valid ? v[c][k] : __uint_as_float(0x7F800000u));
            lane_max = fmaxf(lane_max, valid ? v[c][k] : __uint_as_float(0xFF800000u));
            if constexpr (PB) lane_zeros += (valid && v[c][k] == 0.0f) ? 1u : 0u;
        }
    const float bucket_min = wave_min(lane_min) + 0.0f;  // -0 -> +0
    const float bucket_max = wave_max(lane_max) + 0.0f;
    const uint32_t key_min = float_to_key(bucket_min), key_max = float_to_key(bucket_max);
    const uint32_t mag_max = umax32(__float_as_uint(bucket_min) & 0x7FFFFFFFu, __float_as_uint(bucket_max) & 0x7FFFFFFFu);
    const uint32_t t_max = mag_max >> SHIFT;
    const uint32_t t_low = t_max > (uint32_t)(HALF - 1) ? t_max - (uint32_t)(HALF - 1) : 0u;

    float pb_level = 0.0f;
    if constexpr ((S > 2 && RULE != kEven) || PB) {
        // ---- histogram: the returning LDS add hands every element its position inside its bin ------
#pragma unroll
        for (int t = 0; t < PER; ++t) lds.bin_start[lane * PER + t] = 0u;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        uint32_t slot[C][4];  // bin | position inside the bin << 16
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool valid = full || (256u * c + 4u * lane + k < len);
                const uint32_t bits = __float_as_uint(recompute_from(v[c][k]) + 0.0f);
                const uint32_t t = (bits & 0x7FFFFFFFu) >> SHIFT;
                const uint32_t u = t > t_low ? umin32(t - t_low, (uint32_t)(HALF - 1)) : 0u;  // 0 .. HALF-1 (the clamp only acts on NaN)
                const uint32_t bin = (bits >> 31) ? (uint32_t)(HALF - 1) - u : (uint32_t)HALF + u;
                slot[c][k] = 0u;
                if (valid) slot[c][k] = bin | (atomicAdd(&lds.bin_start[bin], 1u) << 16);
            }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- exclusive prefix over the bin counts (lane l owns bins l*PER .. l*PER+PER-1) ------------
        uint32_t my_start[PER];
        {
            uint32_t cnt[PER];
            uint32_t tot = 0;
#pragma unroll
            for (int t = 0; t < PER; ++t) {
                cnt[t] = lds.bin_start[lane * PER + t];
                tot += cnt[t];
            }
            uint32_t run = wave_inclusive_scan_u32(tot, lane) - tot;
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int t = 0; t < PER; ++t) {
                my_start[t] = run;
                lds.bin_start[lane * PER + t] = run;
                run += cnt[t];
            }
            if (lane == 63u) lds.bin_start[B] = run;  // = len
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- scatter the values into their bins ---------------------------------------------------
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool valid = full || (256u * c + 4u * lane + k < len);
                if (valid) {
                    const uint32_t bin = slot[c][k] & 0xFFFFu, pos = slot[c][k] >> 16;
                    lds.grouped[skewed(lds.bin_start[bin] + pos)] = __float_as_uint(recompute_from(v[c][k]) + 0.0f);
                }
            }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- fp64 prefix of the grouped values at block granularity (lane l sums block l) ------------
        {
            constexpr uint32_t BLOCK = D / 64;
            double part = 0.0;
#pragma unroll
            for (uint32_t i = 0; i < BLOCK; ++i) {
                const uint32_t position = lane * BLOCK + i;
                const float x = position < len ? __uint_as_float(lds.grouped[skewed(position)]) : 0.0f;
                part += (double)x;
            }
            const double incl = wave_inclusive_scan_f64(part, lane);
            lds.block_prefix[lane] = incl - part;
            if (lane == 63u) {
                // the top level is only ever the right end of a solve
                lds.lvl_count_le[S - 1] = len;
                lds.lvl_sum_le[S - 1] = incl;
                lds.lvl_count_lt[S - 1] = len;
                lds.lvl_sum_lt[S - 1] = incl;
            }
        }
        if (lane == 0u) {
            // the bottom level is only ever the left end of a solve
            lds.lvl_count_lt[0] = 0u;
            lds.lvl_sum_lt[0] = 0.0;
            lds.lvl_count_le[0] = 0u;
            lds.lvl_sum_le[0] = 0.0;
        }
        if (lane < (uint32_t)S) {
            lds.lvl_value[lane] = key_to_float(lane == (uint32_t)(S - 1) ? key_max : key_min);
            lds.lvl_rank[lane] = 0u;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        const uint32_t zeros = PB ? wave_sum_u32(lane_zeros) : 0u;
        pb_level = orq_solve_levels<S, RULE>(
            lds, [&](uint32_t rank) { return pick_rank<D, B>(lds, my_start, rank, lane); }, len, zeros, sweeps, lane);
    }

    // every lane holds its own copy of the levels (the selects of the encoder take vector sources)
    float lv[S];
    if constexpr (RULE == kEven) {
        const double largest = (double)__uint_as_float(mag_max);
#pragma unroll
        for (int k = 0; k < S; ++k) lv[k] = (float)(largest * (double)(2 * k - (S - 1)) / (double)(S - 1));
    } else {
        lv[0] = PB ? -pb_level : key_to_float(key_min);
        lv[S - 1] = PB ? pb_level : key_to_float(key_max);
#pragma unroll
        for (int k = 1; k < S - 1; ++k) lv[k] = lds.lvl_value[k];
    }

    if (lane == 0) {
#pragma unroll
        for (int k = 0; k < S; ++k) levels[(size_t)bucket * S + k] = lv[k];
    }

    orq_encode<C, S, BITS, FULL>(v, lv, len, begin, seed, index_offset, codes32);
}

template <int C, int S, int BITS, bool CLIP, int RULE>
__global__ __launch_bounds__(kWave) void orq_quantize_kernel(const float* __restrict__ grad, size_t n,
                                                             uint32_t bucket_size, uint32_t sweeps, float clip,
                                                             uint32_t num_buckets, uint64_t seed,
                                                             uint64_t index_offset, float* __restrict__ levels,
                                                             uint32_t* __restrict__ codes32)
{
    __shared__ OrqLds<OrqShape<C>::D, OrqShape<C>::B> lds;
    const uint32_t bucket = blockIdx.x;
    if (bucket >= num_buckets) return;
    const size_t begin = (size_t)bucket * bucket_size;
    const size_t rest = n - begin;
    const uint32_t len = rest < bucket_size ? (uint32_t)rest : bucket_size;
    if (len == (uint32_t)OrqShape<C>::D)
        orq_bucket<C, S, BITS, true, CLIP, RULE>(lds, grad + begin, len, begin, bucket, sweeps, clip, seed, index_offset, levels, codes32);
    else
        orq_bucket<C, S, BITS, false, CLIP, RULE>(lds, grad + begin, len, begin, bucket, sweeps, clip, seed, index_offset, levels, codes32);
}

// ----------------------------------------------------------------------------------------------
// ORQ and the other random-rounding rules for buckets above 4096 elements (up to 32768): the W = 2, 4 or 8
// wavefronts of a workgroup own one bucket, wavefront w holding bucket elements [4096 w, 4096 (w + 1)) in the
// register layout of orq_bucket.  All of them build the grouping of the whole bucket in LDS (histogram, bin
// starts, scatter, fp64 block prefix) with workgroup barriers in between; the level solves are serial and run
// on wavefront 0 alone; then every wavefront encodes its own elements.
// ----------------------------------------------------------------------------------------------
template <int W>
struct OrqTeamLds {
    static constexpr int D = 4096 * W;
    static constexpr int B = W >= 4 ? 2048 : 1024;   // bins
    static constexpr int SHIFT = W >= 4 ? 17 : 18;   // magnitude bits dropped: exponent + 6 (5) mantissa bits
    uint32_t grouped[D + D / 32];
    uint32_t bin_start[B + 4];
    double block_prefix[D / 64];  // fp64 sum of all positions before block i of 64 positions
    double lvl_sum_lt[10];
    double lvl_sum_le[10];
    float lvl_value[10];
    uint32_t lvl_count_lt[10];
    uint32_t lvl_count_le[10];
    uint32_t lvl_rank[10];
    TeamSlot slots[2][W];
};

template <int W, int S, int BITS, bool FULL, int RULE>
__device__ __forceinline__ void orq_team_bucket(OrqTeamLds<W>& lds, const float* __restrict__ g, uint32_t len,
                                                size_t begin, uint32_t bucket, uint32_t sweeps, float clip,
                                                uint64_t seed, uint64_t index_offset, float* __restrict__ levels,
                                                uint32_t* __restrict__ codes32)
{
    constexpr int C = 16;
    constexpr int D = OrqTeamLds<W>::D;
    constexpr int B = OrqTeamLds<W>::B;
    constexpr int HALF = B / 2;
    constexpr int SHIFT = OrqTeamLds<W>::SHIFT;
    constexpr bool PB = RULE == kPb;
    constexpr uint32_t THREADS = 64u * W;
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = uniform_u32(tid >> 6);
    const uint32_t first = 4096u * wave;  // first bucket element of this wavefront
    const uint32_t my_len = len > first ? (len - first < 4096u ? len - first : 4096u) : 0u;
    WaveTeam<W> team{lds.slots, wave, 0u};

    float v[C][4];
    if (FULL) {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const floatx4 q =
                __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + first + 256 * c + 4 * lane));
            v[c][0] = q.x; v[c][1] = q.y; v[c][2] = q.z; v[c][3] = q.w;
        }
    } else {
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t e = 256u * c + 4u * lane + k;
                v[c][k] = e < my_len ? g[first + e] : 0.0f;
            }
    }

    if (clip > 0.0f) {  // the same for every thread of the grid
        float(&flat)[4 * C] = reinterpret_cast<float(&)[4 * C]>(v);
        clip_in_registers<4 * C>(
            flat, len, clip, [&](int j) { return FULL || (64u * (j & ~3) + 4u * lane + (j & 3) < my_len); },
            [&](double x) { return team.sum(wave_sum(x)); });
    }

    // ---- extremes of the whole bucket ----------------------------------------------------------------
    float lane_min = __uint_as_float(0x7F800000u), lane_max = __uint_as_float(0xFF800000u);
    uint32_t lane_zeros = 0;
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool valid = FULL || (256u * c + 4u * lane + k < my_len);
            lane_min = fminf(lane_min, valid ? v[c][k] : __uint_as_float(0x7F800000u));
            lane_max = fmaxf(lane_max, valid ? v[c][k] : __uint_as_float(0xFF800000u));
            if constexpr (PB) lane_zeros += (valid && v[c][k] == 0.0f) ? 1u : 0u;
        }
    float bucket_min = wave_min(lane_min), bucket_max = wave_max(lane_max);
    uint32_t zeros = PB ? wave_sum_u32(lane_zeros) : 0u;
    {
        const TeamSlot* s = team.exchange((double)zeros, __float_as_uint(bucket_min), __float_as_uint(bucket_max));
        double z = 0.0;
#pragma unroll
        for (int w = 0; w < W; ++w) {
            bucket_min = fminf(bucket_min, __uint_as_float(s[w].a));
            bucket_max = fmaxf(bucket_max, __uint_as_float(s[w].b));
            z += s[w].sum;
        }
        zeros = (uint32_t)z;
    }
    bucket_min += 0.0f;  // -0 -> +0
    bucket_max += 0.0f;
    const uint32_t key_min = float_to_key(bucket_min), key_max = float_to_key(bucket_max);
    const uint32_t mag_max = umax32(__float_as_uint(bucket_min) & 0x7FFFFFFFu, __float_as_uint(bucket_max) & 0x7FFFFFFFu);
    const uint32_t t_max = mag_max >> SHIFT;
    const uint32_t t_low = t_max > (uint32_t)(HALF - 1) ? t_max - (uint32_t)(HALF - 1) : 0u;

    if constexpr ((S > 2 && RULE != kEven) || PB) {
        // ---- histogram: the returning LDS add hands every element its position inside its bin ------------
        for (uint32_t i = tid; i < (uint32_t)B; i += THREADS) lds.bin_start[i] = 0u;
        __syncthreads();
        uint32_t slot[C][4];  // bin | position inside the bin << 16
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool valid = FULL || (256u * c + 4u * lane + k < my_len);
                const uint32_t bits = __float_as_uint(recompute_from(v[c][k]) + 0.0f);
                const uint32_t t = (bits & 0x7FFFFFFFu) >> SHIFT;
                const uint32_t u = t > t_low ? umin32(t - t_low, (uint32_t)(HALF - 1)) : 0u;  // 0 .. HALF-1 (the clamp only acts on NaN)
                const uint32_t bin = (bits >> 31) ? (uint32_t)(HALF - 1) - u : (uint32_t)HALF + u;
                slot[c][k] = 0u;
                if (valid) slot[c][k] = bin | (atomicAdd(&lds.bin_start[bin], 1u) << 16);
            }
        __syncthreads();

        // ---- exclusive prefix over the bin counts (wavefront 0; lane l owns bins l*PER .. l*PER+PER-1) ------
        if (wave == 0u) {
            constexpr uint32_t PER = B / 64;
            uint32_t tot = 0;
            for (uint32_t i = 0; i < PER; ++i) tot += lds.bin_start[lane * PER + i];
            uint32_t run = wave_inclusive_scan_u32(tot, lane) - tot;
            for (uint32_t i = 0; i < PER; ++i) {
                const uint32_t count = lds.bin_start[lane * PER + i];
                lds.bin_start[lane * PER + i] = run;
                run += count;
            }
            if (lane == 63u) lds.bin_start[B] = run;  // = len
        }
        __syncthreads();

        // ---- scatter the values into their bins -------------------------------------------------------
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool valid = FULL || (256u * c + 4u * lane + k < my_len);
                if (valid) {
                    const uint32_t bin = slot[c][k] & 0xFFFFu, pos = slot[c][k] >> 16;
                    lds.grouped[skewed(lds.bin_start[bin] + pos)] = __float_as_uint(recompute_from(v[c][k]) + 0.0f);
                }
            }
        __syncthreads();

        // ---- fp64 prefix of the grouped values per block of 64 positions (thread t sums block t) ----------
        {
            double part = 0.0;
            for (uint32_t i = 0; i < 64u; ++i) {
                const uint32_t position = tid * 64u + i;
                const float x = position < len ? __uint_as_float(lds.grouped[skewed(position)]) : 0.0f;
                part += (double)x;
            }
            const double incl = wave_inclusive_scan_f64(part, lane);
            const TeamSlot* s = team.exchange(readlane_f64(incl, 63), 0u, 0u);
            double before = 0.0, total = 0.0;
#pragma unroll
            for (int w = 0; w < W; ++w) {
                if ((uint32_t)w < wave) before += s[w].sum;
                total += s[w].sum;
            }
            lds.block_prefix[tid] = before + (incl - part);
            if (tid == 0u) {
                // the bottom level is only ever the left end of a solve, the top level the right end
                lds.lvl_count_lt[0] = 0u;
                lds.lvl_sum_lt[0] = 0.0;
                lds.lvl_count_le[0] = 0u;
                lds.lvl_sum_le[0] = 0.0;
                lds.lvl_count_le[S - 1] = len;
                lds.lvl_sum_le[S - 1] = total;
                lds.lvl_count_lt[S - 1] = len;
                lds.lvl_sum_lt[S - 1] = total;
            }
            if (tid < (uint32_t)S) {
                lds.lvl_value[tid] = key_to_float(tid == (uint32_t)(S - 1) ? key_max : key_min);
                lds.lvl_rank[tid] = 0u;
            }
        }
        __syncthreads();

        // ---- the level solves are serial: wavefront 0 ---------------------------------------------------------
        if (wave == 0u) {
            const float pb_level = orq_solve_levels<S, RULE>(
                lds, [&](uint32_t rank) { return pick_rank_by_lookup(lds, rank, lane); }, len, zeros, sweeps, lane);
            if (PB && lane == 0u) {
                lds.lvl_value[0] = -pb_level;
                lds.lvl_value[S - 1] = pb_level;
            }
        }
        __syncthreads();
    }

    float lv[S];
    if constexpr (RULE == kEven) {
        const double largest = (double)__uint_as_float(mag_max);
#pragma unroll
        for (int k = 0; k < S; ++k) lv[k] = (float)(largest * (double)(2 * k - (S - 1)) / (double)(S - 1));
    } else if constexpr (S == 2 && !PB) {
        lv[0] = key_to_float(key_min);
        lv[1] = key_to_float(key_max);
    } else {
#pragma unroll
        for (int k = 0; k < S; ++k) lv[k] = lds.lvl_value[k];
    }
    if (tid == 0u) {
#pragma unroll
        for (int k = 0; k < S; ++k) levels[(size_t)bucket * S + k] = lv[k];
    }

    orq_encode<C, S, BITS, FULL>(v, lv, my_len, begin + first, seed, index_offset, codes32);
}

template <int W, int S, int BITS, int RULE>
__global__ __launch_bounds__(W* kWave) void orq_team_kernel(const float* __restrict__ grad, size_t n,
                                                            uint32_t bucket_size, uint32_t sweeps, float clip,
                                                            uint32_t num_buckets, uint64_t seed, uint64_t index_offset,
                                                            float* __restrict__ levels, uint32_t* __restrict__ codes32)
{
    __shared__ OrqTeamLds<W> lds;
    const uint32_t bucket = blockIdx.x;
    if (bucket >= num_buckets) return;
    const size_t begin = (size_t)bucket * bucket_size;
    const size_t rest = n - begin;
    const uint32_t len = rest < bucket_size ? (uint32_t)rest : bucket_size;
    if (len == (uint32_t)OrqTeamLds<W>::D)
        orq_team_bucket<W, S, BITS, true, RULE>(lds, grad + begin, len, begin, bucket, sweeps, clip, seed, index_offset, levels, codes32);
    else
        orq_team_bucket<W, S, BITS, false, RULE>(lds, grad + begin, len, begin, bucket, sweeps, clip, seed, index_offset, levels, codes32);
}

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

    for (uint32_t w = 0; w < num_workers; ++w) {
        const uint64_t* __restrict__ cw = ptrs.codes[w] + (size_t)word0 * BITS;
        const float* __restrict__ table = ptrs.levels[w];
        if constexpr (WPB > 0) {
            constexpr int kTables = kSpanWords / WPB;
            const uint32_t first_bucket = WPB == kSpanWords ? word0 / words_per_bucket : word0 / (uint32_t)WPB;
            const float* __restrict__ first_table = table + (size_t)first_bucket * S;
            if (whole) {
#pragma unroll
                for (int t = 0; t < kTables; ++t) {
                    float lv[S];
                    load_levels<S>(first_table + t * S, lv);
#pragma unroll
                    for (int j = t * WPB; j < (t + 1) * WPB; ++j) acc[j] += (double)select_level<BITS, S>(cw + j * BITS, lv);
                }
            } else {
#pragma unroll
                for (int t = 0; t < kTables; ++t)
                    if ((uint32_t)(t * WPB) < n_words) {  // a bucket past the end has no table
                        float lv[S];
                        load_levels<S>(first_table + t * S, lv);
#pragma unroll
                        for (int j = t * WPB; j < (t + 1) * WPB; ++j)
                            if ((uint32_t)j < n_words) acc[j] += (double)select_level<BITS, S>(cw + j * BITS, lv);
                    }
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
// Levels per bucket, 0 for a scheme / bits combination that does not exist.
uint32_t levels_per_bucket(uint32_t scheme, uint32_t bits)
{
    if (scheme == OGQ_BINGRAD_B || scheme == OGQ_BINGRAD_PB || scheme == OGQ_SCALED_SIGN) return bits == 1 ? 2u : 0u;
    if (scheme == OGQ_ORQ) return (bits >= 1 && bits <= 3) ? 1u << bits : 0u;
    if (scheme == OGQ_ORQ_PAPER || scheme == OGQ_EVEN || scheme == OGQ_LINEAR)
        return (bits >= 2 && bits <= 4) ? (1u << (bits - 1)) + 1u : 0u;
    return 0u;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_params(const ogq_params_t* p, bool quantize)
{
    if (!p) return OGQ_ERR_NULL_POINTER;
    if (p->bucket_size == 0 || p->bucket_size % 64 != 0 || p->bucket_size > OGQ_MAX_BUCKET_SIZE)
        return OGQ_ERR_BUCKET_SIZE;
    if (p->scheme > OGQ_LINEAR) return OGQ_ERR_SCHEME;
    if (levels_per_bucket(p->scheme, p->bits) == 0) return OGQ_ERR_BITS;
    if (quantize) {
        if (p->index_offset % 64 != 0) return OGQ_ERR_INDEX_OFFSET;
        if (!(p->clip_factor >= 0.0f) || !(p->clip_factor <= 3.0e38f)) return OGQ_ERR_CLIP;
    }
    return OGQ_OK;
}

int finish_launch()
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return OGQ_ERR_LAUNCH;
    }
    return OGQ_OK;
}

template <int E>
void launch_bingrad(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                    hipStream_t st)
{
    const dim3 grid((nb + kBinGradWaves - 1) / kBinGradWaves), block(kWave * kBinGradWaves);
    const bool clip = p->clip_factor > 0.0f, sign = p->scheme == OGQ_SCALED_SIGN;
#define OGQ_LAUNCH(CLIP, SIGN)                                                                                        \
    hipLaunchKernelGGL((bingrad_quantize_kernel<E, CLIP, SIGN>), grid, block, 0, st, g, n, p->bucket_size,           \
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

template <int W>
void launch_bingrad_team(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                         hipStream_t st)
{
    const dim3 grid(nb), block(W * kWave);
    const bool clip = p->clip_factor > 0.0f, sign = p->scheme == OGQ_SCALED_SIGN;
#define OGQ_LAUNCH(CLIP, SIGN)                                                                               \
    hipLaunchKernelGGL((bingrad_team_kernel<W, CLIP, SIGN>), grid, block, 0, st, g, n, p->bucket_size,      \
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

template <int NB>
void launch_bingrad_chunks_of(const float* g, uint32_t chunks, const ogq_params_t* p, float* lv, uint64_t* words,
                              hipStream_t st)
{
    const dim3 grid((chunks + kBinGradWaves - 1) / kBinGradWaves), block(kWave * kBinGradWaves);
    if (p->scheme == OGQ_SCALED_SIGN)
        hipLaunchKernelGGL((bingrad_chunk_kernel<NB, true>), grid, block, 0, st, g, chunks, p->level_iters, lv, words);
    else
        hipLaunchKernelGGL((bingrad_chunk_kernel<NB, false>), grid, block, 0, st, g, chunks, p->level_iters, lv, words);
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

template <int C, int S, int BITS, int RULE = kOptimal>
void launch_orq(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes, hipStream_t st)
{
    if (p->clip_factor > 0.0f)
        hipLaunchKernelGGL((orq_quantize_kernel<C, S, BITS, true, RULE>), dim3(nb), dim3(kWave), 0, st, g, n, p->bucket_size,
                           p->level_iters, p->clip_factor, nb, p->seed, p->index_offset, lv,
                           static_cast<uint32_t*>(codes));
    else
        hipLaunchKernelGGL((orq_quantize_kernel<C, S, BITS, false, RULE>), dim3(nb), dim3(kWave), 0, st, g, n, p->bucket_size,
                           p->level_iters, p->clip_factor, nb, p->seed, p->index_offset, lv,
                           static_cast<uint32_t*>(codes));
}

template <int C, int RULE>
void launch_paper_counts(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                         hipStream_t st)
{
    switch (p->bits) {  // 2^(bits-1) + 1 levels
        case 2: launch_orq<C, 3, 2, RULE>(g, n, p, nb, lv, codes, st); break;
        case 3: launch_orq<C, 5, 3, RULE>(g, n, p, nb, lv, codes, st); break;
        default: launch_orq<C, 9, 4, RULE>(g, n, p, nb, lv, codes, st); break;
    }
}

template <int C>
void launch_orq_levels(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                       hipStream_t st)
{
    switch (p->scheme) {
        case OGQ_BINGRAD_PB: launch_orq<C, 2, 1, kPb>(g, n, p, nb, lv, codes, st); break;
        case OGQ_ORQ:
            switch (p->bits) {
                case 1: launch_orq<C, 2, 1>(g, n, p, nb, lv, codes, st); break;
                case 2: launch_orq<C, 4, 2>(g, n, p, nb, lv, codes, st); break;
                default: launch_orq<C, 8, 3>(g, n, p, nb, lv, codes, st); break;
            }
            break;
        case OGQ_EVEN: launch_paper_counts<C, kEven>(g, n, p, nb, lv, codes, st); break;
        case OGQ_LINEAR: launch_paper_counts<C, kLinear>(g, n, p, nb, lv, codes, st); break;
        default: launch_paper_counts<C, kOptimal>(g, n, p, nb, lv, codes, st); break;  // OGQ_ORQ_PAPER
    }
}

// Buckets above 4096 elements: W wavefronts per bucket.
template <int W, int S, int BITS, int RULE = kOptimal>
void launch_orq_team(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes, hipStream_t st)
{
    hipLaunchKernelGGL((orq_team_kernel<W, S, BITS, RULE>), dim3(nb), dim3(W * kWave), 0, st, g, n, p->bucket_size,
                       p->level_iters, p->clip_factor, nb, p->seed, p->index_offset, lv, static_cast<uint32_t*>(codes));
}

template <int W, int RULE>
void launch_team_paper_counts(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                              hipStream_t st)
{
    switch (p->bits) {  // 2^(bits-1) + 1 levels
        case 2: launch_orq_team<W, 3, 2, RULE>(g, n, p, nb, lv, codes, st); break;
        case 3: launch_orq_team<W, 5, 3, RULE>(g, n, p, nb, lv, codes, st); break;
        default: launch_orq_team<W, 9, 4, RULE>(g, n, p, nb, lv, codes, st); break;
    }
}

template <int W>
void launch_orq_team_levels(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                            hipStream_t st)
{
    switch (p->scheme) {
        case OGQ_BINGRAD_PB: launch_orq_team<W, 2, 1, kPb>(g, n, p, nb, lv, codes, st); break;
        case OGQ_ORQ:
            switch (p->bits) {
                case 1: launch_orq_team<W, 2, 1>(g, n, p, nb, lv, codes, st); break;
                case 2: launch_orq_team<W, 4, 2>(g, n, p, nb, lv, codes, st); break;
                default: launch_orq_team<W, 8, 3>(g, n, p, nb, lv, codes, st); break;
            }
            break;
        case OGQ_EVEN: launch_team_paper_counts<W, kEven>(g, n, p, nb, lv, codes, st); break;
        case OGQ_LINEAR: launch_team_paper_counts<W, kLinear>(g, n, p, nb, lv, codes, st); break;
        default: launch_team_paper_counts<W, kOptimal>(g, n, p, nb, lv, codes, st); break;  // OGQ_ORQ_PAPER
    }
}

}  // namespace

extern "C" {

size_t ogq_num_buckets(size_t n, const ogq_params_t* p)
{
    if (!p || p->bucket_size == 0) return 0;
    return n / p->bucket_size + (n % p->bucket_size != 0);
}

size_t ogq_levels_per_bucket(const ogq_params_t* p) { return p ? levels_per_bucket(p->scheme, p->bits) : 0; }

size_t ogq_levels_count(size_t n, const ogq_params_t* p)
{
    if (!p) return 0;
    return ogq_num_buckets(n, p) * levels_per_bucket(p->scheme, p->bits);
}

size_t ogq_codes_bytes(size_t n, const ogq_params_t* p)
{
    if (!p || p->bucket_size == 0 || levels_per_bucket(p->scheme, p->bits) == 0) return 0;
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
    uint32_t nb = (uint32_t)nb64;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const uint32_t d = params->bucket_size;
    if (params->scheme == OGQ_BINGRAD_B || params->scheme == OGQ_SCALED_SIGN) {
        // Whole chunks of 2048 elements go to the kernel that packs several buckets into a wavefront; what
        // is left (fewer than 2048 elements) takes the one-bucket-per-wavefront kernel below.  Buckets of
        // 512 and 1024 elements stay with that kernel for gradients too short to give every SIMD a chunk
        // or two (it was the faster one below about four million elements).
        const size_t chunks = n / kChunk;
        if (params->clip_factor == 0.0f && d <= kChunk / 2 && kChunk % d == 0 && chunks > 0 &&
            (d <= 256 || chunks >= kMinChunks)) {
            launch_bingrad_chunks(d_grad, (uint32_t)chunks, params, d_levels, d_codes, st);
            const size_t done = chunks * kChunk;
            if (done == n) return finish_launch();
            d_grad += done;
            d_levels += done / d * 2;
            d_codes = static_cast<uint64_t*>(d_codes) + done / 64;
            n -= done;
        }
        nb = (uint32_t)ogq_num_buckets(n, params);
        const uint32_t regs = d / 64;
        if (regs <= 1) launch_bingrad<1>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (regs <= 2) launch_bingrad<2>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (regs <= 4) launch_bingrad<4>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (regs <= 8) launch_bingrad<8>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (regs <= 16) launch_bingrad<16>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (regs <= 32) launch_bingrad<32>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (regs <= 64) launch_bingrad_team<2>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (regs <= 128) launch_bingrad_team<4>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (regs <= 256) launch_bingrad_team<8>(d_grad, n, params, nb, d_levels, d_codes, st);
        else launch_bingrad_team<16>(d_grad, n, params, nb, d_levels, d_codes, st);
    } else {
        const uint32_t chunks = (d + 255) / 256;
        if (chunks <= 1) launch_orq_levels<1>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (chunks <= 2) launch_orq_levels<2>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (chunks <= 4) launch_orq_levels<4>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (chunks <= 8) launch_orq_levels<8>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (chunks <= 16) launch_orq_levels<16>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (chunks <= 32) launch_orq_team_levels<2>(d_grad, n, params, nb, d_levels, d_codes, st);
        else if (chunks <= 64) launch_orq_team_levels<4>(d_grad, n, params, nb, d_levels, d_codes, st);
        else launch_orq_team_levels<8>(d_grad, n, params, nb, d_levels, d_codes, st);
    }
    return finish_launch();
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
    WorkerPtrs ptrs;
    for (uint32_t w = 0; w < OGQ_MAX_WORKERS; ++w) {
        ptrs.codes[w] = nullptr;
        ptrs.levels[w] = nullptr;
    }
    for (uint32_t w = 0; w < num_workers; ++w) {
        if (!d_codes[w] || !d_levels[w]) return OGQ_ERR_NULL_POINTER;
        if (!aligned(d_codes[w], 16) || !aligned(d_levels[w], 16)) return OGQ_ERR_ALIGNMENT;
        ptrs.codes[w] = static_cast<const uint64_t*>(d_codes[w]);
        ptrs.levels[w] = d_levels[w];
    }
    const size_t nb = ogq_num_buckets(n, params);
    if (nb >= (1ull << 31)) return OGQ_ERR_SIZE;
    const uint32_t d = params->bucket_size;
    const uint32_t total_words = (uint32_t)(n / 64 + (n % 64 != 0));
    const uint32_t spans = (total_words + kSpanWords - 1) / kSpanWords;
    const dim3 grid((spans + kWavesPerBlock - 1) / kWavesPerBlock), block(kBlock);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const double inv = 1.0 / (double)num_workers;
    const uint32_t wpb = d / 64;
    const uint32_t span_elements = kSpanWords * 64;
    const uint32_t fixed_wpb = d % span_elements == 0 ? (uint32_t)kSpanWords : (span_elements % d == 0 ? wpb : 0u);
#define OGQ_LAUNCH_DEQUANT_WPB(BITS, S, WPB)                                                                      \
    hipLaunchKernelGGL((dequantize_average_kernel<BITS, S, WPB>), grid, block, 0, st, ptrs, num_workers, n, wpb, \
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
    switch (levels_per_bucket(params->scheme, params->bits)) {
        case 2: OGQ_LAUNCH_DEQUANT(1, 2); break;
        case 4: OGQ_LAUNCH_DEQUANT(2, 4); break;
        case 8: OGQ_LAUNCH_DEQUANT(3, 8); break;
        case 3: OGQ_LAUNCH_DEQUANT(2, 3); break;
        case 5: OGQ_LAUNCH_DEQUANT(3, 5); break;
        default: OGQ_LAUNCH_DEQUANT(4, 9); break;
    }
#undef OGQ_LAUNCH_DEQUANT
#undef OGQ_LAUNCH_DEQUANT_WPB
    return finish_launch();
}

int ogq_probe_read(const float* d_src, size_t n, float* d_sink, void* hip_stream)
{
    if (!d_src || !d_sink) return OGQ_ERR_NULL_POINTER;
    if (!aligned(d_src, 16)) return OGQ_ERR_ALIGNMENT;
    if (n == 0) return OGQ_OK;
    hipLaunchKernelGGL(probe_read_kernel, dim3(kProbeBlocks), dim3(kBlock), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<const float4*>(d_src), n / 4, d_sink);
    return finish_launch();
}

int ogq_probe_copy(const float* d_src, float* d_dst, size_t n, void* hip_stream)
{
    if (!d_src || !d_dst) return OGQ_ERR_NULL_POINTER;
    if (!aligned(d_src, 16) || !aligned(d_dst, 16)) return OGQ_ERR_ALIGNMENT;
    if (n == 0) return OGQ_OK;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(kProbeBlocks), dim3(kBlock), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<const float4*>(d_src), reinterpret_cast<float4*>(d_dst), n / 4);
    return finish_launch();
}

const char* ogq_strerror(int status)
{
    switch (status) {
        case OGQ_OK: return "ok";
        case OGQ_ERR_NULL_POINTER: return "a required pointer is NULL";
        case OGQ_ERR_BUCKET_SIZE: return "bucket_size must be a multiple of 64 in [64, 4096]";
        case OGQ_ERR_BITS: return "bits not supported by the scheme (BinGrad-b / -pb: 1, ORQ: 1..3, ORQ_PAPER: 2..4)";
        case OGQ_ERR_SCHEME: return "unknown scheme";
        case OGQ_ERR_NUM_WORKERS: return "num_workers must be in [1, 64]";
        case OGQ_ERR_ALIGNMENT: return "device pointers must be 16-byte aligned";
        case OGQ_ERR_INDEX_OFFSET: return "index_offset must be a multiple of 64";
        case OGQ_ERR_LAUNCH: return "HIP kernel launch failed";
        case OGQ_ERR_SIZE: return "n is too large for one call";
        case OGQ_ERR_CLIP: return "clip_factor must be finite and not negative";
        default: return "unknown status";
    }
}

int ogq_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
