// Internal header of libogq: wave-level helpers shared by its kernel sources (gfx950, wave64).
// Everything here is inline device code or a compile-time constant; nothing is exported.
#ifndef OGQ_DEVICE_COMMON_H
#define OGQ_DEVICE_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ogq.h"

namespace ogq {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWave * kWavesPerBlock;

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

// Wave-wide sum; the result is wave-uniform.  Four butterfly steps leave every row's sum in all of its lanes; two row
// broadcasts (DPP row_bcast:15 into rows 1 and 3, row_bcast:31 into rows 2 and 3) then add them up as (r0 + r1) + (r2 + r3)
// in the last row, from which one lane is read.
__device__ __forceinline__ double wave_sum(double x)
{
    x += dpp_f64<kDppXor1>(x);
    x += dpp_f64<kDppXor2>(x);
    x += dpp_f64<kDppHalfMirror>(x);
    x += dpp_f64<kDppMirror>(x);
    const uint64_t u = (uint64_t)__double_as_longlong(x);
    const uint32_t lo15 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, 0x142, 0xA, 0xF, false);
    const uint32_t hi15 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), 0x142, 0xA, 0xF, false);
    x += __longlong_as_double((long long)(((uint64_t)hi15 << 32) | lo15));  // rows 0 and 2 add +0.0
    const uint64_t w = (uint64_t)__double_as_longlong(x);
    const uint32_t lo31 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)w, 0x143, 0xC, 0xF, false);
    const uint32_t hi31 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(w >> 32), 0x143, 0xC, 0xF, false);
    x += __longlong_as_double((long long)(((uint64_t)hi31 << 32) | lo31));
    return readlane_f64(x, 63);
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
// A bucket is held by one wavefront, or by the W wavefronts of a workgroup: the Team types say how a
// wave-wide result becomes a bucket-wide one.
// ----------------------------------------------------------------------------------------------
struct OneWave {
    static constexpr int kSize = 1;
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
    static constexpr int kSize = W;
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

}  // namespace ogq
#endif  // OGQ_DEVICE_COMMON_H
