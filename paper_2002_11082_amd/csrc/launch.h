// Internal header of libogq: the host-side launchers each kernel source exports to the C ABI in api.hip.
// A launcher only enqueues, through launch_kernel below, which keeps the status the runtime returns for that launch.
#ifndef OGQ_LAUNCH_H
#define OGQ_LAUNCH_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "ogq.h"

namespace ogq {

// Status of the launches of the current entry-point call on this thread (api.hip clears it on entry and reads it
// before returning).  It is the value hipLaunchKernel itself returns, so an error that some earlier call of the
// process left in the runtime's per-thread error state is neither mistaken for ours nor cleared.
hipError_t& launch_status();

template <class... P, size_t... I>
inline hipError_t launch_with(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t st, std::tuple<P...>& params,
                              std::index_sequence<I...>)
{
    void* pointers[] = {static_cast<void*>(&std::get<I>(params))...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, pointers, 0, st);
}

// Enqueues kernel<<<grid, block, 0, st>>>(args...).  After a failed launch the later launches of the same call are
// left out.
template <class... P, class... A>
inline void launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t st, A&&... args)
{
    if (launch_status() != hipSuccess) return;
    std::tuple<P...> params(static_cast<P>(std::forward<A>(args))...);
    launch_status() = launch_with(kernel, grid, block, st, params, std::index_sequence_for<P...>{});
}

// Levels per bucket, 0 for a scheme / bits combination that does not exist.
uint32_t levels_per_bucket(uint32_t scheme, uint32_t bits);

// BinGrad-b and Scaled SignSGD (bingrad.hip): picks the kernel for the bucket size and gradient length.
void launch_two_level(const float* g, size_t n, const ogq_params_t* p, float* lv, void* codes, hipStream_t st);

// The schemes with random rounding (rounding_part.hip, one object file per bucket capacity): _cN = buckets of
// at most 256*N elements (one wavefront each, two for N = 16), _wN = N wavefronts per bucket of at most 4096*N
// elements.
// nb = number of buckets.
typedef void RoundingLauncher(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                              hipStream_t st);
RoundingLauncher launch_rounding_c1, launch_rounding_c2, launch_rounding_c4, launch_rounding_c8, launch_rounding_c16,
    launch_rounding_w2, launch_rounding_w4, launch_rounding_w8;

// Decode + average and the bandwidth probes (decode.hip).  Pointers already validated.
void launch_decode(const void* const* d_codes, const float* const* d_levels, uint32_t num_workers, size_t n,
                   const ogq_params_t* p, float* d_out, hipStream_t st);
void launch_probe_read(const float* d_src, size_t n, float* d_sink, hipStream_t st);
void launch_probe_copy(const float* d_src, float* d_dst, size_t n, hipStream_t st);

}  // namespace ogq
#endif  // OGQ_LAUNCH_H
