// Test infrastructure: stand-ins for the kernel launchers of libogq, so that the argument validation and dispatch of
// api.hip can be built for the host alone (g++, AddressSanitizer + UndefinedBehaviorSanitizer) and exercised on a
// machine without a GPU.  Every launcher records a refused launch instead of touching a device.
#include "launch.h"

namespace ogq {

static void refuse() { launch_status() = hipErrorInvalidDevice; }

void launch_two_level(const float*, size_t, const ogq_params_t*, float*, void*, hipStream_t) { refuse(); }

#define OGQ_STUB(name) \
    void name(const float*, size_t, const ogq_params_t*, uint32_t, float*, void*, hipStream_t) { refuse(); }
OGQ_STUB(launch_rounding_c1)
OGQ_STUB(launch_rounding_c2)
OGQ_STUB(launch_rounding_c4)
OGQ_STUB(launch_rounding_c8)
OGQ_STUB(launch_rounding_c16)
OGQ_STUB(launch_rounding_w2)
OGQ_STUB(launch_rounding_w4)
OGQ_STUB(launch_rounding_w8)
#undef OGQ_STUB

void launch_decode(const void* const*, const float* const*, uint32_t, size_t, const ogq_params_t*, float*, hipStream_t)
{
    refuse();
}
void launch_probe_read(const float*, size_t, float*, hipStream_t) { refuse(); }
void launch_probe_copy(const float*, float*, size_t, hipStream_t) { refuse(); }

}  // namespace ogq
